// Device code of the GPU path: pack / unpack / elementwise / MFMA GEMM for gfx950.
//
// Packed layout (see include/lpg.h): blocks of 4 KiB = 32 free indices x KB
// contraction indices, each made of four 1 KiB fragments; a fragment is the
// 64-lane x 16-byte register image of an MFMA operand.  Lane l = 32*h + fl of
// fragment c holds free index fl and k = KF*c + 8*(v/4) + 4*h + v%4, v < KV.
#include "lpg_internal.h"

namespace lpg {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct F32 {
    typedef uint32_t raw;
    static constexpr int ES = 4, KV = 4, KF = 8, KB = 32;
};
struct BF16 {
    typedef uint16_t raw;
    static constexpr int ES = 2, KV = 8, KF = 16, KB = 64;
};

// fp32 -> bf16 bit pattern, round to nearest, ties to even; NaN stays NaN.
__device__ __forceinline__ uint32_t bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ float bf16_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

template <typename S, typename D>
__device__ __forceinline__ typename D::raw convert_raw(typename S::raw x)
{
    if constexpr (S::ES == D::ES) {
        return x;
    } else if constexpr (S::ES == 4 && D::ES == 2) {
        return (typename D::raw)bf16_rne(__uint_as_float(x));
    } else {
        return (typename D::raw)((uint32_t)x << 16);
    }
}

// ---------------------------------------------------------------------------------
// pack / unpack.  One workgroup of 256 threads moves one block (32 f x KB k).
// PACK = true: canonical -> packed (zero padding written); false: packed -> canonical.
// C = canonical element type, P = packed element type.
// KC = true: canonical is contiguous along k (sk == 1); thread t handles free index
//   t/8 and the (t%8)-th eighth of the block's k range, so 8 neighbouring lanes touch
//   one contiguous run of the canonical row and one contiguous 128-byte run of a
//   fragment half.
// KC = false: canonical is contiguous along f (sf == 1); thread t owns the 16 packed
//   bytes at t*16 and touches KV canonical elements, lanes running along f.
template <bool PACK, typename C, typename P, bool KC>
__global__ __launch_bounds__(256) void pack_kernel(PackArgs a)
{
    typedef typename C::raw craw;
    typedef typename P::raw praw;
    constexpr int KV = P::KV, KF = P::KF, KB = P::KB;
    const int g = blockIdx.x, kb = blockIdx.y, b = blockIdx.z;
    const int t = threadIdx.x;
    const char *cbase = a.canon + (int64_t)(b / a.c_div) * a.c_slot;
    char *pblock = a.packed + (int64_t)(b / a.p_div) * a.p_slot + (int64_t)kb * a.p_kbs +
                   (int64_t)g * kBlockBytes;
    craw *canon = (craw *)cbase;

    if constexpr (KC) {
        const int fl = t >> 3, piece = t & 7;
        const int64_t f = (int64_t)g * 32 + fl;
        constexpr int PER = KB / 8;  // consecutive k per thread: 4 (fp32) or 8 (bf16)
        const int64_t kbase = (int64_t)kb * KB + piece * PER;
        // k = KF*c + 8*u + 4*h + j for j < 4:   fp32: piece = 2c + h (u = 0);
        // bf16: piece = 2c + u, the eight k split into h = 0 (first four) and h = 1.
        if constexpr (P::ES == 4) {
            const int c = piece >> 1, h = piece & 1;
            praw *dst = (praw *)(pblock + c * kFragBytes + h * 512 + fl * 16);
            if constexpr (PACK) {
                praw v[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int64_t k = kbase + j;
                    v[j] = (f < a.F && k < a.K) ? convert_raw<C, P>(canon[f * a.sf + k]) : (praw)0;
                }
                *(uint4 *)dst = make_uint4(v[0], v[1], v[2], v[3]);
            } else {
                const uint4 q = *(const uint4 *)dst;
                const praw v[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int64_t k = kbase + j;
                    if (f < a.F && k < a.K) canon[f * a.sf + k] = convert_raw<P, C>(v[j]);
                }
            }
        } else {
            const int c = piece >> 1, u = piece & 1;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                praw *dst = (praw *)(pblock + c * kFragBytes + h * 512 + fl * 16 + u * 8);
                if constexpr (PACK) {
                    praw v[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int64_t k = kbase + 4 * h + j;
                        v[j] = (f < a.F && k < a.K) ? convert_raw<C, P>(canon[f * a.sf + k])
                                                    : (praw)0;
                    }
                    *(uint2 *)dst = make_uint2((uint32_t)v[0] | ((uint32_t)v[1] << 16),
                                               (uint32_t)v[2] | ((uint32_t)v[3] << 16));
                } else {
                    const uint2 q = *(const uint2 *)dst;
                    const praw v[4] = {(praw)(q.x & 0xffff), (praw)(q.x >> 16),
                                       (praw)(q.y & 0xffff), (praw)(q.y >> 16)};
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int64_t k = kbase + 4 * h + j;
                        if (f < a.F && k < a.K) canon[f * a.sf + k] = convert_raw<P, C>(v[j]);
                    }
                }
            }
        }
    } else {
        const int c = t >> 6, lane = t & 63, h = lane >> 5, fl = lane & 31;
        const int64_t f = (int64_t)g * 32 + fl;
        praw *dst = (praw *)(pblock + t * 16);
        praw v[KV];
        if constexpr (!PACK) {
            const uint4 q = *(const uint4 *)dst;
            if constexpr (P::ES == 4) {
                v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
            } else {
                const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                for (int j = 0; j < 8; ++j) v[j] = (praw)((w[j >> 1] >> (16 * (j & 1))) & 0xffff);
            }
        }
#pragma unroll
        for (int j = 0; j < KV; ++j) {
            const int64_t k = (int64_t)kb * KB + KF * c + 8 * (j >> 2) + 4 * h + (j & 3);
            const bool in = (f < a.F && k < a.K);
            if constexpr (PACK)
                v[j] = in ? convert_raw<C, P>(canon[k * a.sk + f]) : (praw)0;
            else if (in)
                canon[k * a.sk + f] = convert_raw<P, C>(v[j]);
        }
        if constexpr (PACK) {
            if constexpr (P::ES == 4) {
                *(uint4 *)dst = make_uint4(v[0], v[1], v[2], v[3]);
            } else {
                uint32_t w[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) w[j] = (uint32_t)v[2 * j] | ((uint32_t)v[2 * j + 1] << 16);
                *(uint4 *)dst = make_uint4(w[0], w[1], w[2], w[3]);
            }
        }
    }
}

template <bool PACK>
static hipError_t launch_pack_impl(const PackArgs &a, int cdt, int pdt, hipStream_t st)
{
    if (a.ngroups <= 0 || a.nkb <= 0 || a.batch <= 0) return hipSuccess;
    dim3 grid(a.ngroups, a.nkb, a.batch), block(256);
    const bool kc = (a.sk == 1);
#define LPG_PACK_CASE(CT, PT)                                                          \
    do {                                                                               \
        if (kc)                                                                        \
            hipLaunchKernelGGL((pack_kernel<PACK, CT, PT, true>), grid, block, 0, st, a); \
        else                                                                           \
            hipLaunchKernelGGL((pack_kernel<PACK, CT, PT, false>), grid, block, 0, st, a); \
    } while (0)
    if (cdt == LPG_F32 && pdt == LPG_F32) LPG_PACK_CASE(F32, F32);
    else if (cdt == LPG_BF16 && pdt == LPG_BF16) LPG_PACK_CASE(BF16, BF16);
    else if (cdt == LPG_F32 && pdt == LPG_BF16) LPG_PACK_CASE(F32, BF16);
    else return hipErrorInvalidValue;
#undef LPG_PACK_CASE
    return hipGetLastError();
}

hipError_t launch_pack(const PackArgs &a, int src_dtype, int dst_dtype, hipStream_t st)
{
    return launch_pack_impl<true>(a, src_dtype, dst_dtype, st);
}
hipError_t launch_unpack(const PackArgs &a, int src_dtype, int dst_dtype, hipStream_t st)
{
    // src is packed, dst canonical
    return launch_pack_impl<false>(a, dst_dtype, src_dtype, st);
}

// ---------------------------------------------------------------------------------
// elementwise: flat over 16-byte chunks; the same chunk index means the same logical
// element in every buffer because all share one layout.
__device__ __forceinline__ float silu_f(float g) { return g / (1.0f + __expf(-g)); }

__device__ __forceinline__ float ew_apply(int op, float a, float b, float s)
{
    switch (op) {
        case LPG_EW_SCALE: return s * a;
        case LPG_EW_ADD: return a + s * b;
        default: return silu_f(a) * b;
    }
}

template <typename T>
__global__ __launch_bounds__(256) void ew_kernel(EwArgs a)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < a.n16; i += stride) {
        const uint4 p = ((const uint4 *)a.x0)[i];
        uint4 q = make_uint4(0, 0, 0, 0);
        if (a.x1) q = ((const uint4 *)a.x1)[i];
        const uint32_t pw[4] = {p.x, p.y, p.z, p.w}, qw[4] = {q.x, q.y, q.z, q.w};
        uint32_t r[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if constexpr (T::ES == 4) {
                r[j] = __float_as_uint(ew_apply(a.op, __uint_as_float(pw[j]), __uint_as_float(qw[j]), a.s));
            } else {
                const float lo = ew_apply(a.op, bf16_to_f32(pw[j] & 0xffff), bf16_to_f32(qw[j] & 0xffff), a.s);
                const float hi = ew_apply(a.op, bf16_to_f32(pw[j] >> 16), bf16_to_f32(qw[j] >> 16), a.s);
                r[j] = bf16_rne(lo) | (bf16_rne(hi) << 16);
            }
        }
        ((uint4 *)a.out)[i] = make_uint4(r[0], r[1], r[2], r[3]);
    }
}

hipError_t launch_elementwise(const EwArgs &a, int dtype, hipStream_t st)
{
    if (a.n16 <= 0) return hipSuccess;
    int64_t blocks = (a.n16 + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    if (dtype == LPG_F32)
        hipLaunchKernelGGL((ew_kernel<F32>), dim3((unsigned)blocks), dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL((ew_kernel<BF16>), dim3((unsigned)blocks), dim3(256), 0, st, a);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// GEMM.  out[fl][fr] = epilogue(alpha * sum_k L[fl][k] * R[fr][k] + beta * Cin[fl][fr]),
// L = P(L; FL, K), R = P(R; FR, K), out = P(out; free = FL, contraction = FR).
//
// The MFMA computes a 32x32 tile D[i][j] = sum_k Aop[i][k] * Bop[k][j]; lane l of the
// A operand carries row i = l%32, lane l of the B operand carries column j = l%32, and
// lane l, register r of D holds D[8*(r/4) + 4*(l/32) + r%4][l%32].  With R's fragment
// in the A slot and L's fragment in the B slot, lanes run along out's free index and
// each group of four registers is four consecutive contraction indices of out: the
// accumulators already are fragments of P(out; FL, FR) and are stored as they stand.
//
// Workgroup tile: TLG x TRG 32-groups; WL x WR waves, each owning (TLG/WL) x (TRG/WR)
// 32x32 tiles.  One K block (4 fragments per group) is staged per step through a
// double-buffered LDS copy of the packed blocks; since the packed block is already in
// register-image order the LDS copy is verbatim and every ds_read_b128 is conflict free.

template <typename IN>
__device__ __forceinline__ void mma_frag(f32x16 &acc, const uint4 &r, const uint4 &l)
{
    if constexpr (IN::ES == 4) {
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(r.x), __uint_as_float(l.x), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(r.y), __uint_as_float(l.y), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(r.z), __uint_as_float(l.z), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(r.w), __uint_as_float(l.w), acc, 0, 0, 0);
    } else {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, r),
                                                      __builtin_bit_cast(bf16x8, l), acc, 0, 0, 0);
    }
}

__device__ __forceinline__ float epi_apply(int epi, float v, float g)
{
    if (epi == LPG_EPI_SILU) return silu_f(v);
    if (epi == LPG_EPI_GATE_SILU) return silu_f(g) * v;
    return v;
}

template <typename IN, typename OUT, int TLG, int TRG, int WL, int WR>
__global__ __launch_bounds__(WL *WR * 64) void gemm_kernel(GemmArgs p)
{
    constexpr int NT = WL * WR * 64;
    constexpr int WTL = TLG / WL, WTR = TRG / WR;
    constexpr int NCH = (TLG + TRG) * 256 / NT;  // 16-byte chunks per thread per stage
    constexpr int STAGE = (TLG + TRG) * kBlockBytes;
    static_assert((TLG + TRG) * 256 % NT == 0, "stage must divide over the threads");
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wl = wave % WL, wr = wave / WL;

    // ---- workgroup -> (batch, tile) with an XCD-aware remap: hardware deals workgroups
    // round-robin to the 8 XCDs, so give each XCD a contiguous range of tile ids, then
    // walk tiles in bands of GM tile-rows so that neighbours share L and R panels in L2.
    const int ntile = p.tiles_l * p.tiles_r;
    const int64_t total = (int64_t)ntile * p.batch;
    int64_t pid;
    {
        const int64_t bid = blockIdx.x;
        const int64_t per = total / 8, rem = total % 8, x = bid % 8, idx = bid / 8;
        pid = (x < rem) ? x * (per + 1) + idx : rem * (per + 1) + (x - rem) * per + idx;
    }
    const int b = (int)(pid / ntile);
    const int tp = (int)(pid % ntile);
    constexpr int GM = 8;
    const int width = GM * p.tiles_r;
    const int band = tp / width, first_l = band * GM;
    const int gsz = min(p.tiles_l - first_l, GM);
    const int tl = first_l + (tp % width) % gsz;
    const int tr = (tp % width) / gsz;

    const int gl0 = tl * TLG, gr0 = tr * TRG;
    const int nlg = min(TLG, p.FLg - gl0);
    const int nrg = max(0, min(TRG, p.FRg - gr0));
    const char *Lp = p.L + (int64_t)(b / p.l_div) * p.l_slot + (int64_t)gl0 * kBlockBytes;
    const char *Rp = p.R + (int64_t)(b / p.r_div) * p.r_slot + (int64_t)gr0 * kBlockBytes;

    uint4 pre[NCH];
    auto gload = [&](int kb) {
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int c = i * NT + tid;      // chunk id within the stage
            const int grp = c >> 8;          // block (32-group) the chunk belongs to
            const int off = (c & 255) * 16;
            if (grp < TLG) {
                if (grp < nlg)
                    pre[i] = *(const uint4 *)(Lp + (int64_t)kb * p.l_kbs + grp * kBlockBytes + off);
            } else {
                if (grp - TLG < nrg)
                    pre[i] = *(const uint4 *)(Rp + (int64_t)kb * p.r_kbs + (grp - TLG) * kBlockBytes + off);
            }
        }
    };
    auto sstore = [&](int st) {
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int c = i * NT + tid;
            *(uint4 *)(smem + st * STAGE + c * 16) = pre[i];
        }
    };

    f32x16 acc[WTL][WTR];
#pragma unroll
    for (int a = 0; a < WTL; ++a)
#pragma unroll
        for (int q = 0; q < WTR; ++q)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[a][q][e] = 0.0f;

#pragma unroll
    for (int i = 0; i < NCH; ++i) pre[i] = make_uint4(0, 0, 0, 0);

    if (p.nkb > 0) {
        gload(0);
        sstore(0);
    }
    __syncthreads();
    for (int kb = 0; kb < p.nkb; ++kb) {
        const int cur = kb & 1;
        if (kb + 1 < p.nkb) gload(kb + 1);
        const char *sL = smem + cur * STAGE + (wl * WTL) * kBlockBytes + lane * 16;
        const char *sR = smem + cur * STAGE + (TLG + wr * WTR) * kBlockBytes + lane * 16;
#pragma unroll
        for (int c = 0; c < kFragsPerBlock; ++c) {
            uint4 lf[WTL], rf[WTR];
#pragma unroll
            for (int a = 0; a < WTL; ++a) lf[a] = *(const uint4 *)(sL + a * kBlockBytes + c * kFragBytes);
#pragma unroll
            for (int q = 0; q < WTR; ++q) rf[q] = *(const uint4 *)(sR + q * kBlockBytes + c * kFragBytes);
#pragma unroll
            for (int a = 0; a < WTL; ++a)
#pragma unroll
                for (int q = 0; q < WTR; ++q) mma_frag<IN>(acc[a][q], rf[q], lf[a]);
        }
        if (kb + 1 < p.nkb) sstore(cur ^ 1);
        __syncthreads();
    }

    // ---- epilogue: registers -> fragments of P(out; FL, FR)
    const int h = lane >> 5;
    const int64_t oslot = (int64_t)b * p.o_slot;
    char *Ob = p.Out + oslot;
    const char *Cb = p.Cin ? p.Cin + oslot : nullptr;
    const char *Eb = p.Epi ? p.Epi + oslot : nullptr;
    const bool use_c = (p.beta != 0.0f) && Cb;
    const bool use_e = (p.epi == LPG_EPI_GATE_SILU) && Eb;
#pragma unroll
    for (int a = 0; a < WTL; ++a) {
        const int grL = gl0 + wl * WTL + a;
        if (grL >= p.FLg) continue;
        const int fl = grL * 32 + (lane & 31);
#pragma unroll
        for (int q = 0; q < WTR; ++q) {
            const int grR = gr0 + wr * WTR + q;
            if (grR >= p.FRg_out) continue;
            const bool have = grR < p.FRg;
            float v[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) v[e] = have ? p.alpha * acc[a][q][e] : 0.0f;
            // byte offset of this tile's first fragment inside out
            int64_t obase;
            if constexpr (OUT::ES == 4)
                obase = (int64_t)grR * p.o_kbs + (int64_t)grL * kBlockBytes + lane * 16;
            else
                obase = (int64_t)(grR >> 1) * p.o_kbs + (int64_t)grL * kBlockBytes +
                        (grR & 1) * 2 * kFragBytes + lane * 16;
            constexpr int NF = (OUT::ES == 4) ? 4 : 2;  // fragments this tile spans
            if (use_c || use_e) {
#pragma unroll
                for (int fgi = 0; fgi < NF; ++fgi) {
                    float cv[16 / NF], ev[16 / NF];
                    if constexpr (OUT::ES == 4) {
                        if (use_c) {
                            const uint4 t4 = *(const uint4 *)(Cb + obase + fgi * kFragBytes);
                            cv[0] = __uint_as_float(t4.x); cv[1] = __uint_as_float(t4.y);
                            cv[2] = __uint_as_float(t4.z); cv[3] = __uint_as_float(t4.w);
                        }
                        if (use_e) {
                            const uint4 t4 = *(const uint4 *)(Eb + obase + fgi * kFragBytes);
                            ev[0] = __uint_as_float(t4.x); ev[1] = __uint_as_float(t4.y);
                            ev[2] = __uint_as_float(t4.z); ev[3] = __uint_as_float(t4.w);
                        }
                    } else {
                        if (use_c) {
                            const uint4 t4 = *(const uint4 *)(Cb + obase + fgi * kFragBytes);
                            const uint32_t w[4] = {t4.x, t4.y, t4.z, t4.w};
#pragma unroll
                            for (int j = 0; j < 8; ++j) cv[j] = bf16_to_f32((w[j >> 1] >> (16 * (j & 1))) & 0xffff);
                        }
                        if (use_e) {
                            const uint4 t4 = *(const uint4 *)(Eb + obase + fgi * kFragBytes);
                            const uint32_t w[4] = {t4.x, t4.y, t4.z, t4.w};
#pragma unroll
                            for (int j = 0; j < 8; ++j) ev[j] = bf16_to_f32((w[j >> 1] >> (16 * (j & 1))) & 0xffff);
                        }
                    }
#pragma unroll
                    for (int j = 0; j < 16 / NF; ++j) {
                        float x = v[fgi * (16 / NF) + j];
                        if (use_c) x += p.beta * cv[j];
                        v[fgi * (16 / NF) + j] = epi_apply(p.epi, x, use_e ? ev[j] : 0.0f);
                    }
                }
            } else if (p.epi == LPG_EPI_SILU) {
#pragma unroll
                for (int e = 0; e < 16; ++e) v[e] = silu_f(v[e]);
            }
            // zero the padding of ragged edge tiles
            if (grL * 32 + 32 > p.FL || grR * 32 + 32 > p.FR) {
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int fr = grR * 32 + 8 * (e >> 2) + 4 * h + (e & 3);
                    if (fl >= p.FL || fr >= p.FR) v[e] = 0.0f;
                }
            }
            if constexpr (OUT::ES == 4) {
#pragma unroll
                for (int fgi = 0; fgi < 4; ++fgi)
                    *(uint4 *)(Ob + obase + fgi * kFragBytes) =
                        make_uint4(__float_as_uint(v[4 * fgi]), __float_as_uint(v[4 * fgi + 1]),
                                   __float_as_uint(v[4 * fgi + 2]), __float_as_uint(v[4 * fgi + 3]));
            } else {
#pragma unroll
                for (int fgi = 0; fgi < 2; ++fgi) {
                    uint32_t w[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        w[j] = bf16_rne(v[8 * fgi + 2 * j]) | (bf16_rne(v[8 * fgi + 2 * j + 1]) << 16);
                    *(uint4 *)(Ob + obase + fgi * kFragBytes) = make_uint4(w[0], w[1], w[2], w[3]);
                }
            }
        }
    }
}

template <typename IN, typename OUT, int TLG, int TRG, int WL, int WR>
static hipError_t launch_gemm_cfg(GemmArgs a, hipStream_t st)
{
    constexpr int NT = WL * WR * 64;
    constexpr size_t lds = 2 * (size_t)(TLG + TRG) * kBlockBytes;
    a.tiles_l = (a.FLg + TLG - 1) / TLG;
    a.tiles_r = (a.FRg_out + TRG - 1) / TRG;
    const int64_t total = (int64_t)a.tiles_l * a.tiles_r * a.batch;
    if (total <= 0) return hipSuccess;
    if (total > 0x7fffffff) return hipErrorInvalidValue;
    auto kern = gemm_kernel<IN, OUT, TLG, TRG, WL, WR>;
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)total), dim3(NT), lds, st, a);
    return hipGetLastError();
}

hipError_t launch_gemm(const GemmArgs &a, int in_dtype, int out_dtype, hipStream_t st)
{
    if (in_dtype == LPG_F32 && out_dtype == LPG_F32) return launch_gemm_cfg<F32, F32, 4, 4, 2, 2>(a, st);
    if (in_dtype == LPG_BF16 && out_dtype == LPG_BF16) return launch_gemm_cfg<BF16, BF16, 4, 4, 2, 2>(a, st);
    if (in_dtype == LPG_BF16 && out_dtype == LPG_F32) return launch_gemm_cfg<BF16, F32, 4, 4, 2, 2>(a, st);
    return hipErrorInvalidValue;
}

}  // namespace lpg
