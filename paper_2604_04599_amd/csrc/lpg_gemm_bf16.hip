// MFMA GEMM kernels, BF16 operands -> BF16 result: every tile configuration.
#include "lpg_gemm.h"

namespace lpg {

hipError_t launch_gemm_bf16(const GemmArgs &a, int cfg, hipStream_t st) { return launch_gemm_dtype<BF16, BF16>(a, cfg, st); }

hipError_t launch_gemm_gather_bf16(const GatherArgs &a, hipStream_t st) { return launch_gemm_gather_dtype<BF16, BF16>(a, st); }

}  // namespace lpg
