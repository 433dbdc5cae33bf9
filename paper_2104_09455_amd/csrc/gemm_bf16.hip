// Kernel instantiations for bf16 operands.
#define ABFT_DT abft::DT_BF16
#define ABFT_LAUNCH_NAME launch_gemm_bf16
#include "gemm_launch.inc"
