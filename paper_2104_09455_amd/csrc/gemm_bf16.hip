// Kernel instantiations for bf16 operands.
#define ABFT_DT abft::DT_BF16
#define ABFT_LAUNCH_NAME launch_gemm_bf16
#define ABFT_CHAIN_LAUNCH_NAME launch_mlp_chain_bf16
#include "gemm_launch.inc"
