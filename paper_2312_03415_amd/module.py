"""torch.autograd front end of the library: a LoRA linear layer whose forward and backward run in
the computation graphs runlora_select picks for its shape (arxiv 2312.03415, Section 2), and a
helper that swaps it in for the nn.Linear modules of a model (Section 3 applies RunLoRA to every
attention and MLP linear).

Nothing is computed here: tensors are flattened to [n, d] views, buffers are allocated with torch,
and every product runs inside the HIP library through binding.runlora_forward / runlora_backward.

    layer = RunLoRALinear.from_linear(nn_linear, r=16, alpha=32)     # W frozen, A and B trainable
    y = layer(x)                                                     # x [..., d_in] -> [..., d_out]
    wrap_linears(model, r=16, alpha=32, targets=("q_proj", "v_proj"))
    vera = RunVeRALinear(weight, A_shared, B_shared)                 # frozen A, B; trainable vectors d, b
"""
import math

import torch
from torch import nn

from . import binding as rl

# one scratch buffer per device, shared by every layer (calls on a device are ordered on its current
# stream and nothing lives in the workspace between two calls)
_workspaces = {}


def _workspace(device, nbytes):
    ws = _workspaces.get(device)
    if ws is None or ws.numel() < nbytes:
        ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
        _workspaces[device] = ws
    return ws


class RunLoRAFunction(torch.autograd.Function):
    """y = x W + bias + scale (x A) B with W and bias frozen; gradients for x, A and B (Eq. 1, Eq. 3).

    pair = (forward variant, backward variant) as runlora_select returns them; keep_merged lets
    forward2 hold W + scale AB for a merged backward (i*o elements kept until the backward ran), keep_t
    lets forward1 hold scale XA for the backwards that would form it again (n*r elements);
    dropout = (p, seed) or None: LoRA dropout on the adapter's input (mask defined in runlora.h; the
    backward regenerates it from the seed the forward recorded).
    """

    @staticmethod
    def forward(ctx, x, W, A, B, bias, scale, pair, keep_merged, dropout=None, keep_t=False):
        fwd, bwd = pair
        i, o = W.shape
        r = A.shape[1]
        x2 = x.reshape(-1, i)
        if x2.stride(-1) != 1 or x2.stride(0) % 8 != 0 or x2.data_ptr() % 16 != 0:
            x2 = x2.contiguous()
        n = x2.shape[0]
        code = rl.dtype_code(x.dtype)
        y = torch.empty((n, o), dtype=x.dtype, device=x.device)
        keeps_t = fwd == rl.FWD_DEFAULT or (keep_t and fwd in (rl.FWD1, rl.FWD3) and bwd in (1, 5, 6, 7))
        T = torch.empty((n, r), dtype=x.dtype, device=x.device) if keeps_t else None
        M = None
        if keep_merged and fwd == rl.FWD2 and bwd in rl.BWD_MERGED:
            M = torch.empty((i, o), dtype=x.dtype, device=x.device)
        saved = rl.new_saved(T, M)
        ws = _workspace(x.device, rl.runlora_workspace_bytes(fwd, bwd, n, i, o, r, code))
        p, seed = dropout if dropout else (None, 0)
        rl.runlora_forward(fwd, x2, W, A, B, y, saved, workspace=ws, scale=scale, bias=bias, dropout_p=p, dropout_seed=seed)
        ctx.saved = saved
        ctx.bwd = bwd
        ctx.keep = (T, M)          # buffers *saved points into
        ctx.x_shape = x.shape
        ctx.save_for_backward(x2, W, A, B)
        return y.view(*x.shape[:-1], o)

    @staticmethod
    def backward(ctx, dy):
        x2, W, A, B = ctx.saved_tensors
        i, o = W.shape
        r = A.shape[1]
        n = x2.shape[0]
        dy2 = dy.reshape(n, o)
        if dy2.stride(-1) != 1 or dy2.stride(0) % 8 != 0 or dy2.data_ptr() % 16 != 0:
            dy2 = dy2.contiguous()
        need_x, _, need_a, need_b = ctx.needs_input_grad[:4]
        dx = torch.empty((n, i), dtype=x2.dtype, device=x2.device) if need_x else None
        dA = torch.empty_like(A) if need_a else None
        dB = torch.empty_like(B) if need_b else None
        code = rl.dtype_code(dy.dtype)
        ws = _workspace(dy.device, rl.runlora_workspace_bytes(-1, ctx.bwd, n, i, o, r, code))
        rl.runlora_backward(ctx.bwd, dy2, ctx.saved, W, A, B, dx, dA, dB, workspace=ws)
        if dx is not None:
            dx = dx.view(ctx.x_shape)
        return dx, None, dA, dB, None, None, None, None, None, None


class RunLoRALinear(nn.Module):
    """LoRA-augmented linear layer: frozen W [d_in, d_out] (the orientation of Eq. 1, Y = XW) and
    optional frozen bias, trainable A [d_in, r] and B [r, d_out], scale = alpha / r.

    The (forward, backward) pair is chosen per token count by runlora_select the first time that
    count is seen (criterion 2 when keep_merged, 3 when keep_t), or fixed with pair=(f, b).
    """

    def __init__(self, weight, r, alpha=None, bias=None, pair=None, keep_merged=False, dropout=0.0, keep_t=False):
        super().__init__()
        d_in, d_out = weight.shape
        self.d_in, self.d_out, self.r = d_in, d_out, r
        self.scale = 1.0 if alpha is None else float(alpha) / r
        self.weight = nn.Parameter(weight.contiguous(), requires_grad=False)
        self.bias = nn.Parameter(bias.contiguous(), requires_grad=False) if bias is not None else None
        # the usual LoRA start: A random, B zero, so that the layer starts as the frozen one
        self.lora_A = nn.Parameter(torch.randn(d_in, r, dtype=weight.dtype, device=weight.device) / math.sqrt(d_in))
        self.lora_B = nn.Parameter(torch.zeros(r, d_out, dtype=weight.dtype, device=weight.device))
        self.pair = pair
        self.keep_merged = keep_merged
        self.keep_t = keep_t
        self.dropout = float(dropout)  # LoRA dropout probability, applied in training mode only
        self.last_dropout_seed = None  # seed of the most recent training-mode forward (for reproducing its mask)
        self._pairs = {}

    @classmethod
    def from_linear(cls, linear, r, alpha=None, pair=None, keep_merged=False, dropout=0.0):
        """nn.Linear keeps its weight as [d_out, d_in]; the layer holds the transposed copy."""
        w = linear.weight.detach().t().contiguous()
        b = linear.bias.detach() if linear.bias is not None else None
        return cls(w, r, alpha, b, pair, keep_merged, dropout)

    def pair_for(self, n_tokens):
        if self.pair is not None:
            return self.pair
        p = self._pairs.get(n_tokens)
        if p is None:
            code = rl.dtype_code(self.weight.dtype)
            p = rl.runlora_select(n_tokens, self.d_in, self.d_out, self.r, code, criterion=2 if self.keep_merged else (3 if self.keep_t else None))
            self._pairs[n_tokens] = p
        return p

    def forward(self, x):
        n = x.numel() // self.d_in
        if self.training and self.dropout > 0.0:
            # with dropout only forward1 / backward1 (or the default chain) exist; a fresh seed per call
            # from torch's CPU generator, so that torch.manual_seed makes runs repeatable
            self.last_dropout_seed = int(torch.randint(0, 2 ** 31 - 1, (1,)).item())
            pair = self.pair if self.pair in ((0, 0), (0, 1), (1, 1)) else (1, 1)
            return RunLoRAFunction.apply(x, self.weight, self.lora_A, self.lora_B, self.bias, self.scale, pair, False,
                                         (self.dropout, self.last_dropout_seed), self.keep_t)
        return RunLoRAFunction.apply(x, self.weight, self.lora_A, self.lora_B, self.bias, self.scale,
                                     self.pair_for(n), self.keep_merged, None, self.keep_t)

    def extra_repr(self):
        return f"d_in={self.d_in}, d_out={self.d_out}, r={self.r}, scale={self.scale:g}, bias={self.bias is not None}"


class RunVeRAFunction(torch.autograd.Function):
    """y = x W + bias + scale ((x A) diag(d)) B diag(b) with W, bias, A and B frozen; gradients for x, d and b
    (runlora_vera_forward / runlora_vera_backward: the LoRA graphs on B~ = diag(d) B diag(b))."""

    @staticmethod
    def forward(ctx, x, W, A, B, d, b, bias, scale, pair):
        fwd, bwd = pair
        i, o = W.shape
        r = A.shape[1]
        x2 = x.reshape(-1, i)
        if x2.stride(-1) != 1 or x2.stride(0) % 8 != 0 or x2.data_ptr() % 16 != 0:
            x2 = x2.contiguous()
        n = x2.shape[0]
        code = rl.dtype_code(x.dtype)
        y = torch.empty((n, o), dtype=x.dtype, device=x.device)
        T = torch.empty((n, r), dtype=x.dtype, device=x.device) if fwd == rl.FWD_DEFAULT else None
        saved = rl.new_saved(T)
        ws = _workspace(x.device, rl.runlora_vera_workspace_bytes(fwd, bwd, n, i, o, r, code))
        rl.runlora_vera_forward(fwd, x2, W, A, B, d, b, y, saved, ws, scale=scale, bias=bias)
        ctx.saved = saved
        ctx.bwd = bwd
        ctx.keep = T
        ctx.x_shape = x.shape
        ctx.save_for_backward(x2, W, A, B, d, b)
        return y.view(*x.shape[:-1], o)

    @staticmethod
    def backward(ctx, dy):
        x2, W, A, B, d, b = ctx.saved_tensors
        i, o = W.shape
        r = A.shape[1]
        n = x2.shape[0]
        dy2 = dy.reshape(n, o)
        if dy2.stride(-1) != 1 or dy2.stride(0) % 8 != 0 or dy2.data_ptr() % 16 != 0:
            dy2 = dy2.contiguous()
        need = ctx.needs_input_grad
        dx = torch.empty((n, i), dtype=x2.dtype, device=x2.device) if need[0] else None
        dd = torch.empty_like(d) if need[4] else None
        db = torch.empty_like(b) if need[5] else None
        code = rl.dtype_code(dy.dtype)
        ws = _workspace(dy.device, rl.runlora_vera_workspace_bytes(-1, ctx.bwd, n, i, o, r, code))
        rl.runlora_vera_backward(ctx.bwd, dy2, ctx.saved, W, A, B, d, b, dx, dd, db, ws)
        if dx is not None:
            dx = dx.view(ctx.x_shape)
        return dx, None, None, None, dd, db, None, None, None


class RunVeRALinear(nn.Module):
    """VeRA layer: frozen W [d_in, d_out] (+ bias) and frozen random A [d_in, r], B [r, d_out] (pass the
    same tensors to every layer to share them, as VeRA does), trainable vectors d [r] (start 0.1) and
    b [d_out] (start 0, so that the layer starts as the frozen one)."""

    def __init__(self, weight, A, B, bias=None, scale=1.0, pair=None, d_init=0.1):
        super().__init__()
        d_in, d_out = weight.shape
        r = A.shape[1]
        if A.shape != (d_in, r) or B.shape != (r, d_out):
            raise ValueError("A must be [d_in, r] and B [r, d_out]")
        self.d_in, self.d_out, self.r, self.scale, self.pair = d_in, d_out, r, float(scale), pair
        self.weight = nn.Parameter(weight.contiguous(), requires_grad=False)
        self.bias = nn.Parameter(bias.contiguous(), requires_grad=False) if bias is not None else None
        self.register_buffer("vera_A", A, persistent=False)
        self.register_buffer("vera_B", B, persistent=False)
        self.vera_d = nn.Parameter(torch.full((r,), d_init, dtype=weight.dtype, device=weight.device))
        self.vera_b = nn.Parameter(torch.zeros(d_out, dtype=weight.dtype, device=weight.device))
        self._pairs = {}

    def pair_for(self, n_tokens):
        if self.pair is not None:
            return self.pair
        p = self._pairs.get(n_tokens)
        if p is None:
            p = rl.runlora_select(n_tokens, self.d_in, self.d_out, self.r, rl.dtype_code(self.weight.dtype))
            self._pairs[n_tokens] = p
        return p

    def forward(self, x):
        return RunVeRAFunction.apply(x, self.weight, self.vera_A, self.vera_B, self.vera_d, self.vera_b, self.bias,
                                     self.scale, self.pair_for(x.numel() // self.d_in))

    def extra_repr(self):
        return f"d_in={self.d_in}, d_out={self.d_out}, r={self.r}, scale={self.scale:g}, bias={self.bias is not None}"


class RunDoRAFunction(torch.autograd.Function):
    """y = x ((W + scale A B) diag(m / c)) + bias, c the column norms of W + scale A B held constant in the backward
    pass; gradients for x, A, B and m (runlora_dora_forward / runlora_dora_backward: forward2 and one of the merged
    backward graphs, the merge kernel scaling W's columns on the way)."""

    @staticmethod
    def forward(ctx, x, W, A, B, m, bias, scale, bwd):
        i, o = W.shape
        r = A.shape[1]
        x2 = x.reshape(-1, i)
        if x2.stride(-1) != 1 or x2.stride(0) % 8 != 0 or x2.data_ptr() % 16 != 0:
            x2 = x2.contiguous()
        n = x2.shape[0]
        code = rl.dtype_code(x.dtype)
        y = torch.empty((n, o), dtype=x.dtype, device=x.device)
        c = torch.empty((o,), dtype=torch.float32, device=x.device)
        saved = rl.new_saved(None)
        ws = _workspace(x.device, rl.runlora_dora_workspace_bytes(rl.FWD2, bwd, n, i, o, r, code))
        rl.runlora_dora_forward(rl.FWD2, x2, W, A, B, m, y, saved, c, ws, scale=scale, bias=bias)
        ctx.saved = saved
        ctx.bwd = bwd
        ctx.bias = bias
        ctx.x_shape = x.shape
        ctx.save_for_backward(x2, W, A, B, m, c, y)  # y is the tensor handed to the caller: no copy is kept
        return y.view(*x.shape[:-1], o)

    @staticmethod
    def backward(ctx, dy):
        x2, W, A, B, m, c, y = ctx.saved_tensors
        i, o = W.shape
        r = A.shape[1]
        n = x2.shape[0]
        dy2 = dy.reshape(n, o)
        if dy2.stride(-1) != 1 or dy2.stride(0) % 8 != 0 or dy2.data_ptr() % 16 != 0:
            dy2 = dy2.contiguous()
        need = ctx.needs_input_grad
        dx = torch.empty((n, i), dtype=x2.dtype, device=x2.device) if need[0] else None
        dA = torch.empty_like(A) if need[2] else None
        dB = torch.empty_like(B) if need[3] else None
        dm = torch.empty_like(m) if need[4] else None
        code = rl.dtype_code(dy.dtype)
        ws = _workspace(dy.device, rl.runlora_dora_workspace_bytes(-1, ctx.bwd, n, i, o, r, code))
        rl.runlora_dora_backward(ctx.bwd, dy2, ctx.saved, W, A, B, m, c, y, dx, dA, dB, dm, ws, bias=ctx.bias)
        if dx is not None:
            dx = dx.view(ctx.x_shape)
        return dx, None, dA, dB, dm, None, None, None


class RunDoRALinear(nn.Module):
    """DoRA layer: frozen W [d_in, d_out] (+ bias), trainable A [d_in, r], B [r, d_out] (B starts at 0) and
    magnitudes m [d_out], which start at the column norms of W so that the layer starts as the frozen one.
    16-bit dtypes, r <= 128.  bwd: the merged backward graph (4, 5, 7 or 8); None = the one of the four with the
    smallest modelled time for the token count of the call (the time model of runlora_select)."""

    def __init__(self, weight, r, alpha=None, bias=None, bwd=None):
        super().__init__()
        d_in, d_out = weight.shape
        self.d_in, self.d_out, self.r, self.bwd = d_in, d_out, r, bwd
        self.scale = float(alpha) / r if alpha is not None else 1.0
        self.weight = nn.Parameter(weight.contiguous(), requires_grad=False)
        self.bias = nn.Parameter(bias.contiguous(), requires_grad=False) if bias is not None else None
        self.lora_A = nn.Parameter(torch.randn(d_in, r, dtype=weight.dtype, device=weight.device) / math.sqrt(d_in))
        self.lora_B = nn.Parameter(torch.zeros(r, d_out, dtype=weight.dtype, device=weight.device))
        self.dora_m = nn.Parameter(weight.float().norm(dim=0).to(weight.dtype))
        self._bwds = {}

    @classmethod
    def from_linear(cls, linear, r, alpha=None, bwd=None):
        """nn.Linear keeps its weight as [d_out, d_in]; the layer holds the transposed copy."""
        w = linear.weight.detach().t().contiguous()
        b = linear.bias.detach() if linear.bias is not None else None
        return cls(w, r, alpha, b, bwd)

    def bwd_for(self, n_tokens):
        if self.bwd is not None:
            return self.bwd
        b = self._bwds.get(n_tokens)
        if b is None:
            code = rl.dtype_code(self.weight.dtype)
            b = min((4, 5, 7, 8), key=lambda v: rl.runlora_model_time_us(1, v, n_tokens, self.d_in, self.d_out, self.r, code))
            self._bwds[n_tokens] = b
        return b

    def forward(self, x):
        return RunDoRAFunction.apply(x, self.weight, self.lora_A, self.lora_B, self.dora_m, self.bias, self.scale,
                                     self.bwd_for(x.numel() // self.d_in))

    def extra_repr(self):
        return f"d_in={self.d_in}, d_out={self.d_out}, r={self.r}, scale={self.scale:g}, bias={self.bias is not None}"


def wrap_linears(model, r, alpha=None, targets=None, pair=None, keep_merged=False, dropout=0.0, adapter="lora"):
    """Replace nn.Linear submodules of `model` by RunLoRALinear, or by RunDoRALinear with adapter="dora" (all of
    them, or those whose attribute name is in `targets`); every other parameter of the model is frozen.
    Returns the replaced names."""
    if adapter not in ("lora", "dora"):
        raise ValueError("adapter must be 'lora' or 'dora'")
    if adapter == "dora" and (pair is not None or keep_merged or dropout):
        raise ValueError("the DoRA layer takes none of pair / keep_merged / dropout")
    replaced = []
    for name, module in list(model.named_modules()):
        for child_name, child in list(module.named_children()):
            if isinstance(child, nn.Linear) and (targets is None or child_name in targets):
                new = (RunDoRALinear.from_linear(child, r, alpha) if adapter == "dora"
                       else RunLoRALinear.from_linear(child, r, alpha, pair, keep_merged, dropout))
                setattr(module, child_name, new)
                replaced.append(f"{name}.{child_name}" if name else child_name)
    for pname, p in model.named_parameters():
        if not (pname.endswith("lora_A") or pname.endswith("lora_B") or pname.endswith("dora_m")):
            p.requires_grad_(False)
    return replaced
