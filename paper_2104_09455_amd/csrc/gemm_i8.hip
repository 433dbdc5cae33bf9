// Kernel instantiations for i8 operands.
#define ABFT_DT abft::DT_I8
#define ABFT_LAUNCH_NAME launch_gemm_i8
#include "gemm_launch.inc"
