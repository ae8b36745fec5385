#define RL_T float
#define RL_BK 32
#define RL_FN gemm_launch_f32
#define RL_SKINNY_FN skinny_launch_f32
#define RL_PIPE 0
#include "gemm_launch.inc"
