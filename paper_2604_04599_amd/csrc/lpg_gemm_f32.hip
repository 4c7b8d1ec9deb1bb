// MFMA GEMM kernels, F32 operands -> F32 result: every tile configuration.
#include "lpg_gemm.h"

namespace lpg {

hipError_t launch_gemm_f32(const GemmArgs &a, int cfg, hipStream_t st) { return launch_gemm_dtype<F32, F32>(a, cfg, st); }

hipError_t launch_gemm_gather_f32(const GatherArgs &a, hipStream_t st) { return launch_gemm_gather_dtype<F32, F32>(a, st); }

}  // namespace lpg
