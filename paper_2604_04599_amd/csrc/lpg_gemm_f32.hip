// MFMA GEMM kernels, F32 operands -> F32 result: every tile configuration.
#include "lpg_gemm.h"

namespace lpg {

hipError_t launch_gemm_f32(const GemmArgs &a, int cfg, hipStream_t st) { return launch_gemm_dtype<F32, F32>(a, cfg, st); }

}  // namespace lpg
