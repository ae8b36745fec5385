// Constants of the selector's time model, measured on one MI355X with this library's own kernels
// (see the calibration script next to the Python binding).  Regenerate after changing a kernel.
#pragma once
#include "gemm.hpp"

namespace rl {

struct ModelConstants {
  // sustained TFLOP/s of each tile shape on a large problem; [0] = bf16/fp16, [1] = fp32
  double tile_tflops[2][CFG_COUNT];
  double stream_tbps;  // sustained HBM streaming rate of the skinny kernels, TB/s
  double launch_us;    // fixed cost per kernel launch on one stream
};

inline const ModelConstants& model_constants() {
  static const ModelConstants c = {
      {{850.0, 700.0, 150.0, 250.0, 150.0, 250.0, 900.0, 1000.0}, {125.0, 110.0, 20.0, 30.0, 20.0, 30.0, 125.0, 125.0}},
      3.0,
      3.0,
  };
  return c;
}

}  // namespace rl
