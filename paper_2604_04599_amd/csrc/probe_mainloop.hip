// Stand-alone probe of what bounds the GEMM main loops on gfx950 (not part of the library; built as
// its own executable and run by `bench.py --probe`).  Two questions, both answered with kernels that
// touch no user data and whose loops have fixed trip counts:
//
// 1. What does the chip give a kernel that issues nothing but MFMAs (the practical peak, with the
//    power limit's effect on real operand values)?  256 workgroups x 16 waves, four independent
//    accumulators per wave, operands in registers: zero or pseudo-random in [-1, 1).
//
// 2. Where do the cycles of the bf16 256 x 256 tile's half-K-block step go?  The step is rebuilt
//    piece by piece: 8 waves of 4 x 2 accumulator tiles, 32 MFMAs per SIMD and step (1056 cycles
//    alone), then the wave's 12 LDS fragment reads, the barrier, and the step's global->LDS
//    transfers (TPW fragments of 1 KiB per wave and step, into a ring of NS stages, from a 64 KiB
//    window per workgroup that stays in L2).  All data is zero: the clock stays at its maximum.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdint>

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

#define CHECK(x)                                                                          \
    do {                                                                                  \
        hipError_t e_ = (x);                                                              \
        if (e_ != hipSuccess) {                                                           \
            fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));                       \
            return 1;                                                                     \
        }                                                                                 \
    } while (0)

__device__ inline float pseudo_random(unsigned s)
{
    s ^= s >> 16; s *= 0x7feb352dU; s ^= s >> 15; s *= 0x846ca68bU; s ^= s >> 16;
    return (float)(int)(s & 0xffff) / 32768.0f - 1.0f;
}

// ---- 1. MFMAs only
template <bool BF>
__global__ void __launch_bounds__(1024) mfma_only(int iters, int random, float *out)
{
    f32x16 acc[4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[a][e] = 0.f;
    bf16x8 xb[4], yb[4];
    float xf[4], yf[4];
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const unsigned id = (blockIdx.x * 1024 + threadIdx.x) * 4 + a;
        xf[a] = random ? pseudo_random(2 * id + 1) : 0.0f;
        yf[a] = random ? pseudo_random(2 * id + 2) : 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            xb[a][e] = (__bf16)(random ? pseudo_random((2 * id + 1) * 8 + e) : 0.0f);
            yb[a][e] = (__bf16)(random ? pseudo_random((2 * id + 2) * 8 + e) : 0.0f);
        }
    }
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            if constexpr (BF) acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xb[a], yb[a], acc[a], 0, 0, 0);
            else acc[a] = __builtin_amdgcn_mfma_f32_32x32x2f32(xf[a], yf[a], acc[a], 0, 0, 0);
        }
    }
    float s = 0;
#pragma unroll
    for (int a = 0; a < 4; ++a) s += acc[a][0];
    if (s == 123.456f) out[threadIdx.x] = s;  // keeps the result alive; never true in practice
}

// ---- 2. the step of the bf16 256 x 256 tile
template <bool READS, bool BAR, int TPW, int NS>
__global__ void __launch_bounds__(512) step_probe(int steps, float *out, const char *gsrc)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];  // NS stages x 16 groups x 2 fragments x 1 KiB
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wl = wave & 1, wr = wave >> 1;
    for (int i = threadIdx.x; i < NS * 32768 / 16; i += 512) ((uint4 *)smem)[i] = make_uint4(0, 0, 0, 0);
    __syncthreads();
    f32x16 acc[4][2];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[a][q][e] = 0.f;
    uint4 lf[2][4], rf[2][2];
    auto rd = [&](int buf, int stage, int c) {
        const char *base = smem + stage * 32768 + lane * 16;
#pragma unroll
        for (int a = 0; a < 4; ++a) lf[buf][a] = *(const uint4 *)(base + ((wl * 4 + a) * 2 + c) * 1024);
#pragma unroll
        for (int q = 0; q < 2; ++q) rf[buf][q] = *(const uint4 *)(base + ((8 + wr * 2 + q) * 2 + c) * 1024);
    };
    rd(0, 0, 0);
    const uint32_t sbase = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)smem;
    const char *win = gsrc + (size_t)blockIdx.x * 65536 + lane * 16;  // 64 KiB window per workgroup
    for (int s = 0; s < steps; ++s) {
        const int stage = s % NS, nxt = (s + 1) % NS, fill = (s + NS - 1) % NS;
#pragma unroll
        for (int i = 0; i < TPW; ++i) {  // this step's transfers: fragment f of the stage being filled
            const int f = i * 8 + wave;
            const char *g = win + ((s * 32 + f) & 63) * 1024;
            const uint32_t dst = sbase + fill * 32768 + f * 1024;
            asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(dst) : "memory", "m0");
        }
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            if (READS) {
                if (c == 0) rd(1, stage, 1);
                else rd(0, nxt, 0);
            }
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int q = 0; q < 2; ++q)
                    acc[a][q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, rf[c][q]),
                                                                        __builtin_bit_cast(bf16x8, lf[c][a]), acc[a][q], 0, 0, 0);
        }
        if (TPW) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 2) * TPW) : "memory");
        if (BAR) __syncthreads();
        asm volatile("" ::: "memory");
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    float t = 0;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int q = 0; q < 2; ++q) t += acc[a][q][0];
    if (t == 123.456f) out[threadIdx.x] = t;
}

static hipEvent_t e0, e1;

template <bool BF>
static int run_mfma_only(const char *name, int random, float *out)
{
    const int iters = BF ? 1000000 : 500000;
    float ms = 0;
    for (int rep = 0; rep < 3; ++rep) {
        CHECK(hipEventRecord(e0));
        hipLaunchKernelGGL(mfma_only<BF>, dim3(256), dim3(1024), 0, 0, iters, random, out);
        CHECK(hipEventRecord(e1));
        CHECK(hipEventSynchronize(e1));
        CHECK(hipEventElapsedTime(&ms, e0, e1));
    }
    const double flops = 256.0 * 16 * 4 * (double)iters * (BF ? 32768 : 4096);
    printf("{\"probe\": \"mfma_only\", \"what\": \"%s\", \"ms\": %.1f, \"tflops\": %.1f}\n", name, ms, flops / (ms * 1e-3) / 1e12);
    fflush(stdout);
    return 0;
}

template <bool READS, bool BAR, int TPW, int NS>
static int run_step(const char *name, float *out, const char *gsrc)
{
    const int steps = 200000;
    CHECK(hipFuncSetAttribute((const void *)step_probe<READS, BAR, TPW, NS>, hipFuncAttributeMaxDynamicSharedMemorySize,
                              NS * 32768));
    float ms = 0;
    for (int rep = 0; rep < 3; ++rep) {
        CHECK(hipEventRecord(e0));
        hipLaunchKernelGGL((step_probe<READS, BAR, TPW, NS>), dim3(256), dim3(512), NS * 32768, 0, steps, out, gsrc);
        CHECK(hipEventRecord(e1));
        CHECK(hipEventSynchronize(e1));
        CHECK(hipEventElapsedTime(&ms, e0, e1));
    }
    printf("{\"probe\": \"bf16_step\", \"what\": \"%s\", \"ms\": %.1f, \"cycles_per_step_at_2.4GHz\": %.0f, \"mfma_alone\": 1056}\n",
           name, ms, ms * 1e-3 * 2.4e9 / steps);
    fflush(stdout);
    return 0;
}

int main()
{
    float *out;
    char *gsrc;
    CHECK(hipMalloc(&out, 4096));
    CHECK(hipMalloc(&gsrc, 256 * 65536));
    CHECK(hipMemset(gsrc, 0, 256 * 65536));
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    if (run_mfma_only<true>("bf16 32x32x16, zero operands", 0, out)) return 1;
    if (run_mfma_only<true>("bf16 32x32x16, operands uniform in [-1, 1)", 1, out)) return 1;
    if (run_mfma_only<false>("fp32 32x32x2, zero operands", 0, out)) return 1;
    if (run_mfma_only<false>("fp32 32x32x2, operands uniform in [-1, 1)", 1, out)) return 1;
    if (run_step<false, false, 0, 2>("MFMAs only", out, gsrc)) return 1;
    if (run_step<false, true, 0, 2>("MFMAs + barrier", out, gsrc)) return 1;
    if (run_step<true, false, 0, 2>("MFMAs + LDS reads", out, gsrc)) return 1;
    if (run_step<true, true, 0, 2>("MFMAs + LDS reads + barrier", out, gsrc)) return 1;
    if (run_step<true, true, 1, 3>("... + 8 KiB of global->LDS transfers per step, 3 stages", out, gsrc)) return 1;
    if (run_step<true, true, 2, 3>("... + 16 KiB per step, 3 stages", out, gsrc)) return 1;
    if (run_step<true, true, 4, 2>("... + 32 KiB per step (what the tile needs), 2 stages", out, gsrc)) return 1;
    if (run_step<true, true, 4, 3>("... + 32 KiB per step, 3 stages", out, gsrc)) return 1;
    if (run_step<true, true, 4, 4>("... + 32 KiB per step, 4 stages", out, gsrc)) return 1;
    return 0;
}
