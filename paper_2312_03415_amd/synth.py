"""Seeded synthetic inputs for the LoRA-linear layer: shared by the tests, the bench and the
smoke check, for both the HIP library and the CPU oracle.

Holds no arithmetic of the method itself: only a counter-based random number generator
(splitmix64 -> Box-Muller), rounding of the drawn values to the storage dtype, and the table
of workload shapes.  Every value depends only on (seed, stream id, element index), so any
machine produces the same bits.

The workloads stand in for what the paper trains on (LoRA adapters on the attention / MLP
linears of OPT, Llama and RoBERTa, Section 3): transformer-shaped X, W, A, B, dY with
Gaussian entries; N(0, v) below means variance v.
"""
from dataclasses import dataclass

import numpy as np

BASE_SEED = 20231203
STREAM_X, STREAM_W, STREAM_A, STREAM_B, STREAM_DY, STREAM_Q, STREAM_SCALE = 1, 2, 3, 4, 5, 6, 7

_U64 = np.uint64
_MASK = (1 << 64) - 1


def _splitmix64(x: np.ndarray) -> np.ndarray:
    """One splitmix64 output step applied to each counter value (uint64, wraps mod 2^64)."""
    with np.errstate(over="ignore"):
        z = x + _U64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> _U64(30))) * _U64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> _U64(27))) * _U64(0x94D049BB133111EB)
        return z ^ (z >> _U64(31))


def _key(seed: int, stream: int) -> np.uint64:
    k = _splitmix64(np.array([(seed * 0x100000001B3 + stream) & _MASK], dtype=_U64))
    return _splitmix64(k)[0]


def uniform01(seed: int, stream: int, count: int, lane: int = 0, start: int = 0) -> np.ndarray:
    """count doubles in (0,1); element e uses counter 2*(start+e)+lane under the stream key."""
    idx = (np.arange(start, start + count, dtype=_U64) << _U64(1)) + _U64(lane)
    with np.errstate(over="ignore"):
        bits = _splitmix64(idx ^ _key(seed, stream))
    return ((bits >> _U64(11)).astype(np.float64) + 0.5) * (1.0 / (1 << 53))


def normal(seed: int, stream: int, shape, variance: float = 1.0) -> np.ndarray:
    """N(0, variance) float64 array; chunked so large tensors stay within a few hundred MB."""
    count = int(np.prod(shape))
    out = np.empty(count, dtype=np.float64)
    step = 1 << 22
    for s in range(0, count, step):
        c = min(step, count - s)
        u1 = uniform01(seed, stream, c, 0, s)
        u2 = uniform01(seed, stream, c, 1, s)
        out[s:s + c] = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    out *= np.sqrt(variance)
    return out.reshape(shape)


def integers(seed: int, stream: int, shape, low: int, high: int) -> np.ndarray:
    """Uniform integers in [low, high] as int8."""
    count = int(np.prod(shape))
    u = uniform01(seed, stream, count, 0, 0)
    return (np.floor(u * (high - low + 1)).astype(np.int64) + low).astype(np.int8).reshape(shape)


# ---- storage dtypes ------------------------------------------------------------------------

DTYPES = ("f32", "f16", "bf16")


def to_bf16_bits(a64: np.ndarray) -> np.ndarray:
    """Round float64 -> bfloat16 (nearest even, via float32) and return the 16-bit patterns."""
    f32 = np.ascontiguousarray(a64, dtype=np.float32)
    u = f32.view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def from_bf16_bits(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def store(a64: np.ndarray, dtype: str) -> np.ndarray:
    """Round drawn values to the storage dtype; bf16 is carried as uint16 bit patterns."""
    if dtype == "f32":
        return np.ascontiguousarray(a64, dtype=np.float32)
    if dtype == "f16":
        return np.ascontiguousarray(a64, dtype=np.float16)
    if dtype == "bf16":
        return to_bf16_bits(a64)
    raise ValueError(dtype)


def widen(stored: np.ndarray, dtype: str) -> np.ndarray:
    """Exact float64 value of what `store` produced (what both sides compute from)."""
    if dtype == "bf16":
        return from_bf16_bits(stored)
    return stored.astype(np.float64)


# ---- workloads -----------------------------------------------------------------------------

@dataclass(frozen=True)
class Layer:
    name: str
    n: int      # tokens = batch * seq
    i: int      # d_in
    o: int      # d_out
    r: int      # LoRA rank
    dtype: str
    index: int = 0  # offsets the RNG streams so that layers of one workload differ


def layer_inputs(L: Layer, seed: int = BASE_SEED, b_variance=None):
    """Stored X, W, A, B, dY of one layer: X,dY ~ N(0,1); W,A ~ N(0,1/i); B ~ N(0,0.1/r)."""
    off = 16 * L.index
    bv = (0.1 / L.r) if b_variance is None else b_variance
    t = {
        "X": normal(seed, off + STREAM_X, (L.n, L.i), 1.0),
        "W": normal(seed, off + STREAM_W, (L.i, L.o), 1.0 / L.i),
        "A": normal(seed, off + STREAM_A, (L.i, L.r), 1.0 / L.i),
        "B": normal(seed, off + STREAM_B, (L.r, L.o), bv),
        "dY": normal(seed, off + STREAM_DY, (L.n, L.o), 1.0),
    }
    return {k: store(v, L.dtype) for k, v in t.items()}


def int4_weight(L: Layer, seed: int = BASE_SEED, group: int = 64):
    """Symmetric 4-bit frozen weight: q ~ U{-7..7} (int8, unpacked), one fp16 scale per
    (group of `group` rows along d_in, column); scale = U(0.5,1.5)/(4.32*sqrt(i)) so that the
    dequantised W has variance close to 1/i (4.32 = std of U{-7..7})."""
    off = 16 * L.index
    q = integers(seed, off + STREAM_Q, (L.i, L.o), -7, 7)
    g = (L.i + group - 1) // group
    u = uniform01(seed, off + STREAM_SCALE, g * L.o).reshape(g, L.o)
    scale = ((0.5 + u) / (4.32 * np.sqrt(L.i))).astype(np.float16)
    return q, scale


def config_tiny_f32():
    return [Layer("tiny", 256, 768, 768, 8, "f32", 0)]


def config_opt13b_mlp(dtype="bf16"):
    return [Layer("fc1", 4096, 2048, 8192, 16, dtype, 0), Layer("fc2", 4096, 8192, 2048, 16, dtype, 1)]


def config_llama7b(r: int, dtype="bf16"):
    n = 8192
    return [
        Layer("q", n, 4096, 4096, r, dtype, 0), Layer("k", n, 4096, 4096, r, dtype, 1),
        Layer("v", n, 4096, 4096, r, dtype, 2), Layer("o", n, 4096, 4096, r, dtype, 3),
        Layer("gate", n, 4096, 11008, r, dtype, 4), Layer("up", n, 4096, 11008, r, dtype, 5),
        Layer("down", n, 11008, 4096, r, dtype, 6),
    ]


def config_selector_sweep(dtype="f16"):
    out = []
    for a, n in enumerate((128, 1024, 16384)):
        for b, r in enumerate((8, 64, 256, 1024)):
            out.append(Layer(f"n{n}_r{r}", n, 4096, 4096, r, dtype, 4 * a + b))
    return out


def config_qlora():
    return [Layer("qlora", 4096, 5120, 13824, 64, "bf16", 0)]
