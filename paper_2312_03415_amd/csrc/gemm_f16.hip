#define RL_T _Float16
#define RL_BK 64
#define RL_FN gemm_launch_f16
#define RL_SKINNY_FN skinny_launch_f16
#define RL_MERGE_FN merge_launch_f16
#define RL_PIPE 1
#include "gemm_launch.inc"
