// Kernel instantiations for f16 operands.
#define ABFT_DT abft::DT_F16
#define ABFT_LAUNCH_NAME launch_gemm_f16
#define ABFT_CHAIN_LAUNCH_NAME launch_mlp_chain_f16
#include "gemm_launch.inc"
