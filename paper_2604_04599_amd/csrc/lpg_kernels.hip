// Device code of the GPU path for gfx950: pack / unpack / elementwise / row operations / RoPE /
// fused attention, the choice of the GEMM tile configuration, and the library's static scratch.
//
// Packed layout (see include/lpg.h): blocks of 4 KiB = 32 free indices x KB
// contraction indices, each made of four 1 KiB fragments; a fragment is the
// 64-lane x 16-byte register image of an MFMA operand.  Lane l = 32*h + fl of
// fragment c holds free index fl and k = KF*c + 8*(v/4) + 4*h + v%4, v < KV.


#include "lpg_device.h"
#include "lpg_tiles.h"

namespace lpg {

// ---------------------------------------------------------------------------------
// Process-wide state: tuning hooks, per-device facts, the static scratch.

static int g_tune[LPG_TUNE_KEYS] = {-1, -1, -1, -1, -1, -1, -1, -1};

int tune_get(int key) { return __atomic_load_n(&g_tune[key], __ATOMIC_RELAXED); }

int tune_set(int key, int value)
{
    if (key < 0 || key >= LPG_TUNE_KEYS) return -1;
    __atomic_store_n(&g_tune[key], value < 0 ? -1 : value, __ATOMIC_RELAXED);
    return 0;
}

constexpr int kMaxDevices = 128;

static int current_device()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) dev = 0;
    return dev;
}

const DeviceInfo &device_info()
{
    // filled once per device; a race between two first callers writes the same values twice
    static DeviceInfo info[kMaxDevices];
    static unsigned char known[kMaxDevices];
    const int dev = current_device();
    if (!__atomic_load_n(&known[dev], __ATOMIC_ACQUIRE)) {
        int ncu = 0, lds = 0;
        if (hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || ncu <= 0) ncu = 256;
        // the LDS of one compute unit: what a single resident workgroup can be given
        if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, dev) != hipSuccess || lds < 64 * 1024)
            lds = 64 * 1024;
        info[dev].ncu = ncu;
        info[dev].lds_bytes = lds;
        __atomic_store_n(&known[dev], 1, __ATOMIC_RELEASE);
    }
    return info[dev];
}

bool first_use_on_device(PerDeviceFlag &f)
{
    const int dev = current_device();
    return !((__atomic_load_n(&f.done[dev / 64], __ATOMIC_ACQUIRE) >> (dev % 64)) & 1ull);
}

void mark_used_on_device(PerDeviceFlag &f)
{
    const int dev = current_device();
    __atomic_fetch_or(&f.done[dev / 64], 1ull << (dev % 64), __ATOMIC_RELEASE);
}

// Device memory the library owns, for callers that may not allocate (lpg_chain_static): the
// row-major copies of the canonical control chain.  Every GPU the library runs on holds its own
// copy of this array, at its own address, until the process ends.  `scratch` is a host-side
// stand-in here, never a device address: host code uses the address hipGetSymbolAddress gives.
constexpr size_t kScratchBytes = (size_t)LPG_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

hipError_t static_scratch(void **ptr, size_t *bytes)
{
    static void *base[kMaxDevices];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    void *p = __atomic_load_n(&base[dev], __ATOMIC_ACQUIRE);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        __atomic_store_n(&base[dev], p, __ATOMIC_RELEASE);
    }
    *ptr = p;
    *bytes = kScratchBytes;
    return hipSuccess;
}

// Launch limits of HIP: a request past them is reported, never narrowed.
constexpr int64_t kMaxGridX = 0x7fffffff, kMaxGridYZ = 65535;

// ---------------------------------------------------------------------------------
// pack / unpack.  A workgroup of 256 threads moves whole blocks (32 f x KB k), KPW
// consecutive K blocks of one 32-group per workgroup.
// PACK = true: canonical -> packed (zero padding written); false: packed -> canonical.
// C = canonical element type, P = packed element type.
// KC = true: canonical is contiguous along k (sk == 1); thread t handles free index
//   t/8 and the (t%8)-th eighth of the block's k range: PER = KB/8 consecutive canonical
//   elements, moved as 16- or 32-byte vectors when VEC says every such run is 16-byte
//   aligned, so 8 neighbouring lanes touch one contiguous run of the canonical row and one
//   contiguous 128-byte run of a fragment half.
// KC = false: canonical is contiguous along f (sf == 1); thread t owns the 16 packed
//   bytes at t*16 and touches KV canonical elements, lanes running along f.
template <typename T, int N>
__device__ __forceinline__ void load_run(T (&dst)[N], const T *src, bool vec)
{
    constexpr int BYTES = N * (int)sizeof(T);
    static_assert(BYTES % 16 == 0, "runs are whole 16-byte vectors");
    if (vec) {
        uint4 q[BYTES / 16];
#pragma unroll
        for (int i = 0; i < BYTES / 16; ++i) q[i] = ((const uint4 *)src)[i];
        __builtin_memcpy(dst, q, BYTES);
    } else {
#pragma unroll
        for (int i = 0; i < N; ++i) dst[i] = src[i];
    }
}
template <typename T, int N>
__device__ __forceinline__ void store_run(T *dst, const T (&src)[N])
{
    constexpr int BYTES = N * (int)sizeof(T);
    uint4 q[BYTES / 16];
    __builtin_memcpy(q, src, BYTES);
#pragma unroll
    for (int i = 0; i < BYTES / 16; ++i) ((uint4 *)dst)[i] = q[i];
}

template <bool PACK, typename C, typename P, bool KC, bool VEC>
__global__ __launch_bounds__(256) void pack_kernel(PackArgs a)
{
    typedef typename C::raw craw;
    typedef typename P::raw praw;
    constexpr int KV = P::KV, KF = P::KF, KB = P::KB;
    const int g = blockIdx.x, b = blockIdx.z;
    const int t = threadIdx.x;
    craw *canon = (craw *)(a.canon + (int64_t)(b / a.c_div) * a.c_slot);
    char *pgroup = a.packed + (int64_t)(b / a.p_div) * a.p_slot + (int64_t)g * a.p_gs;
    const int kb_end = min(a.nkb, (int)(blockIdx.y + 1) * a.kpw);

    for (int kb = blockIdx.y * a.kpw; kb < kb_end; ++kb) {
        char *pblock = pgroup + (int64_t)kb * a.p_kbs;
        if constexpr (KC) {
            const int fl = t >> 3, piece = t & 7;
            const int64_t f = (int64_t)g * 32 + fl;
            constexpr int PER = KB / 8;  // consecutive k per thread: 4 (fp32) or 8 (bf16)
            const int64_t kbase = (int64_t)kb * KB + piece * PER;
            craw *run = canon + f * a.sf + kbase;
            const bool row_in = f < a.F;
            const bool whole = row_in && kbase + PER <= a.K;
            craw cv[PER];
            praw pv[PER];
            // packed position of the run: k = KF*c + 8*u + 4*h + j (j < 4).
            //   fp32: piece = 2c + h, one 16-byte vector.
            //   bf16: piece = 2c + u; its first four k have h = 0, the last four h = 1: two
            //   8-byte halves of neighbouring 16-byte lane vectors.
            char *dst0 = pblock + (piece >> 1) * kFragBytes + fl * 16;
            if constexpr (PACK) {
                if (whole) {
                    load_run(cv, run, VEC);
                } else {
#pragma unroll
                    for (int j = 0; j < PER; ++j) cv[j] = (row_in && kbase + j < a.K) ? run[j] : (craw)0;
                }
#pragma unroll
                for (int j = 0; j < PER; ++j) pv[j] = convert_raw<C, P>(cv[j]);
                // a view whose ragged extent ends inside its parent shares this block with the
                // parent's other elements: write only what belongs to the view
                const bool f_mine = row_in || !a.keep_f;
                if (!f_mine || (a.keep_k && kbase + PER > a.K)) {
#pragma unroll
                    for (int j = 0; j < PER; ++j) {
                        if (!f_mine || kbase + j >= a.K) continue;
                        if constexpr (P::ES == 4) *(praw *)(dst0 + (piece & 1) * 512 + j * 4) = pv[j];
                        else *(praw *)(dst0 + (j >> 2) * 512 + (piece & 1) * 8 + (j & 3) * 2) = pv[j];
                    }
                } else if constexpr (P::ES == 4) {
                    *(uint4 *)(dst0 + (piece & 1) * 512) = make_uint4(pv[0], pv[1], pv[2], pv[3]);
                } else {
#pragma unroll
                    for (int h = 0; h < 2; ++h)
                        *(uint2 *)(dst0 + h * 512 + (piece & 1) * 8) =
                            make_uint2((uint32_t)pv[4 * h] | ((uint32_t)pv[4 * h + 1] << 16),
                                       (uint32_t)pv[4 * h + 2] | ((uint32_t)pv[4 * h + 3] << 16));
                }
            } else {
                if constexpr (P::ES == 4) {
                    const uint4 q = *(const uint4 *)(dst0 + (piece & 1) * 512);
                    pv[0] = q.x; pv[1] = q.y; pv[2] = q.z; pv[3] = q.w;
                } else {
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const uint2 q = *(const uint2 *)(dst0 + h * 512 + (piece & 1) * 8);
                        pv[4 * h] = (praw)(q.x & 0xffff); pv[4 * h + 1] = (praw)(q.x >> 16);
                        pv[4 * h + 2] = (praw)(q.y & 0xffff); pv[4 * h + 3] = (praw)(q.y >> 16);
                    }
                }
#pragma unroll
                for (int j = 0; j < PER; ++j) cv[j] = convert_raw<P, C>(pv[j]);
                if (whole && VEC) {
                    store_run(run, cv);
                } else {
#pragma unroll
                    for (int j = 0; j < PER; ++j)
                        if (row_in && kbase + j < a.K) run[j] = cv[j];
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
                const int64_t k_hi = (int64_t)kb * KB + KF * c + KF - 1;  // largest k this thread holds
                const bool f_mine = f < a.F || !a.keep_f;
                if (!f_mine || (a.keep_k && k_hi >= a.K)) {
#pragma unroll
                    for (int j = 0; j < KV; ++j) {
                        const int64_t k = (int64_t)kb * KB + KF * c + 8 * (j >> 2) + 4 * h + (j & 3);
                        if (f_mine && k < a.K) dst[j] = v[j];
                    }
                } else if constexpr (P::ES == 4) {
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
}

// The same move for a view whose origin is off the 32 / KB grid (a.f_off / a.k_off into the
// block a.packed points at).  The canonical run that feeds one 16-byte lane vector is then
// neither aligned nor whole, so every element goes by itself: thread t owns the 16 packed
// bytes at t*16 of a block, maps each of its KV elements back to the view's (f, k) and moves
// it if it lies inside.  Nothing outside the view is written, padding included.
template <bool PACK, typename C, typename P>
__global__ __launch_bounds__(256) void pack_offgrid_kernel(PackArgs a)
{
    typedef typename C::raw craw;
    typedef typename P::raw praw;
    constexpr int KV = P::KV, KF = P::KF, KB = P::KB;
    const int g = blockIdx.x, kb = blockIdx.y, b = blockIdx.z;
    const int t = threadIdx.x;
    craw *canon = (craw *)(a.canon + (int64_t)(b / a.c_div) * a.c_slot);
    praw *pvec = (praw *)(a.packed + (int64_t)(b / a.p_div) * a.p_slot + (int64_t)g * a.p_gs +
                          (int64_t)kb * a.p_kbs + t * 16);
    const int c = t >> 6, lane = t & 63, h = lane >> 5, fl = lane & 31;
    const int64_t f = (int64_t)g * 32 + fl - a.f_off;
    if (f < 0 || f >= a.F) return;
#pragma unroll
    for (int v = 0; v < KV; ++v) {
        const int64_t k = (int64_t)kb * KB + KF * c + 8 * (v >> 2) + 4 * h + (v & 3) - a.k_off;
        if (k < 0 || k >= a.K) continue;
        craw *ce = canon + f * a.sf + k * a.sk;
        if constexpr (PACK) pvec[v] = convert_raw<C, P>(*ce);
        else *ce = convert_raw<P, C>(pvec[v]);
    }
}

template <bool PACK>
static hipError_t launch_pack_impl(PackArgs a, int cdt, int pdt, hipStream_t st)
{
    if (a.ngroups <= 0 || a.nkb <= 0 || a.batch <= 0) return hipSuccess;
    if (a.f_off || a.k_off) {
        if (a.nkb > kMaxGridYZ || a.batch > kMaxGridYZ) return hipErrorInvalidConfiguration;
        const dim3 grid(a.ngroups, a.nkb, a.batch), block(256);
        if (cdt == LPG_F32 && pdt == LPG_F32) hipLaunchKernelGGL((pack_offgrid_kernel<PACK, F32, F32>), grid, block, 0, st, a);
        else if (cdt == LPG_BF16 && pdt == LPG_BF16) hipLaunchKernelGGL((pack_offgrid_kernel<PACK, BF16, BF16>), grid, block, 0, st, a);
        else if (cdt == LPG_F32 && pdt == LPG_BF16) hipLaunchKernelGGL((pack_offgrid_kernel<PACK, F32, BF16>), grid, block, 0, st, a);
        else return hipErrorInvalidValue;
        return hipGetLastError();
    }
    a.kpw = a.nkb >= 16 ? 4 : 1;
    if ((a.nkb + a.kpw - 1) / a.kpw > kMaxGridYZ || a.batch > kMaxGridYZ) return hipErrorInvalidConfiguration;
    dim3 grid(a.ngroups, (a.nkb + a.kpw - 1) / a.kpw, a.batch), block(256);
    const bool kc = (a.sk == 1);
    // vector path: every PER-element run of the canonical side starts on a 16-byte boundary
    const int ces = cdt == LPG_F32 ? 4 : 2;
    const bool vec = kc && ((uintptr_t)a.canon % 16 == 0) && ((a.sf * ces) % 16 == 0) && (a.c_slot % 16 == 0);
#define LPG_PACK_CASE(CT, PT)                                                                    \
    do {                                                                                         \
        if (kc && vec)                                                                           \
            hipLaunchKernelGGL((pack_kernel<PACK, CT, PT, true, true>), grid, block, 0, st, a);  \
        else if (kc)                                                                             \
            hipLaunchKernelGGL((pack_kernel<PACK, CT, PT, true, false>), grid, block, 0, st, a); \
        else                                                                                     \
            hipLaunchKernelGGL((pack_kernel<PACK, CT, PT, false, false>), grid, block, 0, st, a); \
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
                r[j] = bf16_pack2(lo, hi);
            }
        }
        ((uint4 *)a.out)[i] = make_uint4(r[0], r[1], r[2], r[3]);
    }
    // elements past the last whole 16-byte chunk (tight canonical buffers of odd sizes only:
    // packed buffers are whole blocks)
    if (blockIdx.x == 0 && (int)threadIdx.x < a.tail) {
        const int64_t e = a.n16 * (16 / T::ES) + threadIdx.x;
        typedef typename T::raw raw;
        const raw x0 = ((const raw *)a.x0)[e];
        const raw x1 = a.x1 ? ((const raw *)a.x1)[e] : (raw)0;
        if constexpr (T::ES == 4) {
            ((raw *)a.out)[e] = __float_as_uint(ew_apply(a.op, __uint_as_float(x0), __uint_as_float(x1), a.s));
        } else {
            ((raw *)a.out)[e] = (raw)bf16_rne(ew_apply(a.op, bf16_to_f32(x0), bf16_to_f32(x1), a.s));
        }
    }
}

hipError_t launch_elementwise(const EwArgs &a, int dtype, hipStream_t st)
{
    if (a.n16 <= 0 && a.tail <= 0) return hipSuccess;
    int64_t blocks = (a.n16 + 255) / 256;
    if (blocks > (int64_t)device_info().ncu * 16) blocks = (int64_t)device_info().ncu * 16;
    if (blocks < 1) blocks = 1;
    if (dtype == LPG_F32)
        hipLaunchKernelGGL((ew_kernel<F32>), dim3((unsigned)blocks), dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL((ew_kernel<BF16>), dim3((unsigned)blocks), dim3(256), 0, st, a);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// Row operations on a packed left operand (row = free index, reduction along the
// contraction index): softmax with the attention block's scale and causal mask folded in,
// and RMS normalisation.  Both reduce a row to a pair of numbers, then rewrite the row.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr float kNegBig = -3.0e38f;  // "no element yet": finite, so differences never give NaN

// element v (< KV) of a 16-byte chunk, widened to fp32
template <typename T>
__device__ __forceinline__ float chunk_elem(const u32x4 &c, int v)
{
    if constexpr (T::ES == 4) {
        return __uint_as_float(c[v]);
    } else {
        return (v & 1) ? __uint_as_float(c[v / 2] & 0xffff0000u) : __uint_as_float(c[v / 2] << 16);
    }
}
// KV fp32 results -> one 16-byte chunk of T (bf16: round to nearest even)
template <typename T>
__device__ __forceinline__ u32x4 chunk_from(const float (&e)[T::KV])
{
    if constexpr (T::ES == 4) {
        return (u32x4){__float_as_uint(e[0]), __float_as_uint(e[1]), __float_as_uint(e[2]), __float_as_uint(e[3])};
    } else {
        return (u32x4){bf16_pack2(e[0], e[1]), bf16_pack2(e[2], e[3]), bf16_pack2(e[4], e[5]), bf16_pack2(e[6], e[7])};
    }
}
// column of chunk element v relative to the chunk's first: packed chunks hold k0 + 8*(v/4) + v%4
// (a lane's share of a fragment half), chunks cut from a row-major row (LINEAR) hold k0 + v
template <bool LINEAR>
__device__ __forceinline__ constexpr int chunk_k(int v) { return LINEAR ? v : 8 * (v / 4) + v % 4; }

// Makes the compiler treat the chunks as new values (no instruction is emitted), so that it
// re-derives widened elements from the 16-byte chunks in the next pass instead of keeping
// every element of the previous pass alive in a register of its own.
template <int N>
__device__ __forceinline__ void forget_derived(u32x4 (&buf)[N])
{
#pragma unroll
    for (int i = 0; i < N; ++i) asm volatile("" : "+v"(buf[i]));
}

// Softmax policy.  Values are v = x * sl, sl = scale * log2(e) > 0; a row part is summarised
// as (m, s) = (max v, sum 2^(v - m)).  Elements outside the kept columns are replaced by -inf
// once, when a chunk arrives (`admit`): the passes then need no masks, a masked element
// contributes 2^(-inf) = 0 to the sum and comes out as an exact 0.  The maximum is taken over
// products x*sl, the exponent's argument is one fused multiply-add fma(x, sl, -m): one
// rounding, and no product is kept between the passes.
struct SoftmaxRow {
    static constexpr bool kMasked = true;  // honours RowArgs::causal
    float sl;
    __device__ __forceinline__ explicit SoftmaxRow(const RowArgs &a) : sl(a.scalar) {}
    __device__ __forceinline__ static void init(float &m, float &s) { m = kNegBig; s = 0.0f; }
    __device__ __forceinline__ static void merge(float &m, float &s, float m2, float s2)
    {
        const float M = fmaxf(m, m2);
        s = s * __builtin_amdgcn_exp2f(m - M) + s2 * __builtin_amdgcn_exp2f(m2 - M);
        m = M;
    }
    // a chunk that is not loaded because all of it is masked: -inf in every element
    template <typename T>
    __device__ __forceinline__ static u32x4 absent()
    {
        constexpr uint32_t w = T::ES == 4 ? 0xff800000u : 0xff80ff80u;
        return (u32x4){w, w, w, w};
    }
    // element v of the chunk sits in column k0 + chunk_k(v); columns > last become -inf
    template <typename T, bool LINEAR>
    __device__ __forceinline__ static u32x4 admit(u32x4 c, int k0, int last)
    {
        if constexpr (T::ES == 4) {
#pragma unroll
            for (int v = 0; v < 4; ++v) c[v] = (k0 + chunk_k<LINEAR>(v) <= last) ? c[v] : 0xff800000u;
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t lo = (k0 + chunk_k<LINEAR>(2 * j) <= last) ? (c[j] & 0xffffu) : 0xff80u;
                const uint32_t hi = (k0 + chunk_k<LINEAR>(2 * j + 1) <= last) ? (c[j] & 0xffff0000u) : 0xff800000u;
                c[j] = lo | hi;
            }
        }
        return c;
    }
    // folds admitted chunks buf[0..N) into (m, s)
    template <typename T, int N>
    __device__ __forceinline__ void fold(u32x4 (&buf)[N], float &m, float &s) const
    {
        float bm = m;
#pragma unroll
        for (int i = 0; i < N; ++i)
#pragma unroll
            for (int v = 0; v < T::KV; ++v) bm = fmaxf(bm, chunk_elem<T>(buf[i], v) * sl);
        forget_derived(buf);
        float bs = 0.0f;
#pragma unroll
        for (int i = 0; i < N; ++i)
#pragma unroll
            for (int v = 0; v < T::KV; ++v) bs += __builtin_amdgcn_exp2f(fmaf(chunk_elem<T>(buf[i], v), sl, -bm));
        s = s * __builtin_amdgcn_exp2f(m - bm) + bs;
        m = bm;
    }
    // (m, s) of the whole row -> the two constants `emit` uses
    __device__ __forceinline__ void finish(float &m, float &s) const { s = s > 0.0f ? 1.0f / s : 0.0f; }
    template <typename T, bool LINEAR>
    __device__ __forceinline__ u32x4 emit(const u32x4 &c, int k0, int last, float m, float inv) const
    {
        float e[T::KV];
#pragma unroll
        for (int v = 0; v < T::KV; ++v) e[v] = __builtin_amdgcn_exp2f(fmaf(chunk_elem<T>(c, v), sl, -m)) * inv;
        return chunk_from<T>(e);
    }
};

// RMS normalisation policy: (sum of squares, unused) -> y = x * rsqrt(mean square + eps) * w[k].
// Padding and chunks that are not loaded are zeros: no mask is needed.
struct RmsNormRow {
    static constexpr bool kMasked = false;
    const float *w;
    float eps, inv_n;
    __device__ __forceinline__ explicit RmsNormRow(const RowArgs &a) : w(a.weight), eps(a.scalar), inv_n(1.0f / (float)a.cols) {}
    __device__ __forceinline__ static void init(float &q, float &u) { q = 0.0f; u = 0.0f; }
    __device__ __forceinline__ static void merge(float &q, float &u, float q2, float) { q += q2; }
    template <typename T>
    __device__ __forceinline__ static u32x4 absent() { return (u32x4){0u, 0u, 0u, 0u}; }
    template <typename T, bool LINEAR>
    __device__ __forceinline__ static u32x4 admit(u32x4 c, int, int) { return c; }
    template <typename T, int N>
    __device__ __forceinline__ void fold(u32x4 (&buf)[N], float &q, float &u) const
    {
        float acc = 0.0f;
#pragma unroll
        for (int i = 0; i < N; ++i)
#pragma unroll
            for (int v = 0; v < T::KV; ++v) acc = fmaf(chunk_elem<T>(buf[i], v), chunk_elem<T>(buf[i], v), acc);
        q += acc;
    }
    __device__ __forceinline__ void finish(float &q, float &u) const { q = 1.0f / sqrtf(q * inv_n + eps); }
    template <typename T, bool LINEAR>
    __device__ __forceinline__ u32x4 emit(const u32x4 &c, int k0, int last, float r, float) const
    {
        float e[T::KV];
#pragma unroll
        for (int v = 0; v < T::KV; ++v) {
            const int k = k0 + chunk_k<LINEAR>(v);
            e[v] = k <= last ? chunk_elem<T>(c, v) * r * w[k] : 0.0f;
        }
        return chunk_from<T>(e);
    }
};

// A workgroup of NW waves owns R (32, 16 or 8) consecutive rows of one 32-row group over
// the whole contraction range.  In every fragment half those rows are one contiguous run of
// R*16 bytes; runs are numbered q = 8*kb + 2*c + h, a wave load covers 64/R consecutive runs
// (lane l: row l%R of run l/R), and consecutive waves take consecutive loads, so the
// workgroup streams whole blocks in address order.  NW*64/R is a multiple of 8, so a lane
// stays on one (c, h) and only its K block advances, by NW*8/R per load: addresses and k
// indices are affine in the load counter.  Lane-local k of chunk element v:
// k0 + 8*(v/4) + v%4 with k0 = KB*kb + KF*c + 4*h.
// CACHED: the R rows fit in 16 chunks per lane; they are read once, kept in registers
// across the reduction and written once.  Otherwise the rows are streamed twice.
template <typename T, typename OP, int R, int NW, bool CACHED>
__global__ __launch_bounds__(NW * 64) void row_packed_kernel(RowArgs a)
{
    constexpr int RPW = 64 / R, NCH = 16;
    constexpr int KBSTEP = NW * RPW / 8;  // K blocks a lane advances per load
    constexpr int KINC = KBSTEP * T::KB;
    static_assert((NW * RPW) % 8 == 0, "a lane must stay on one fragment half");
    __shared__ float red_a[NW][32], red_b[NW][32];
    OP op(a);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int rl = lane % R, rsel = lane / R;
    uint32_t wg = blockIdx.x;
    const int sub = wg % (32 / R);
    wg /= (32 / R);
    const int g = wg % a.ngroups, b = wg / a.ngroups;
    const int row = 32 * g + sub * R + rl;
    int last = (OP::kMasked && a.causal) ? row + (a.cols - a.rows) : a.cols - 1;  // last kept column of this row
    last = last < a.cols - 1 ? last : a.cols - 1;
    if (row >= a.rows) last = -1;
    const int q0 = w * RPW + rsel;  // this lane's run in load 0
    const int kfirst = T::KB * (q0 >> 3) + T::KF * ((q0 >> 1) & 3) + 4 * (q0 & 1);
    const int kend = T::KB * a.nkb;  // runs exist for k0 < kend
    const int64_t base = (int64_t)b * a.slot + (int64_t)g * kBlockBytes + (sub * R + rl) * 16 +
                         (int64_t)(q0 >> 3) * a.kbs + (q0 & 7) * 512;
    const char *xp = a.x + base;
    char *outp = a.out + base;
    const int64_t step = (int64_t)KBSTEP * a.kbs;
    const int nbatches = CACHED ? 1 : (a.nkb + NCH * KBSTEP - 1) / (NCH * KBSTEP);

    u32x4 buf[NCH];
    float ra, rb;
    OP::init(ra, rb);
    for (int bt = 0; bt < nbatches; ++bt) {
        const int k0b = kfirst + bt * NCH * KINC;
        const char *xb = xp + (int64_t)bt * NCH * step;
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            buf[i] = OP::template absent<T>();
            if (k0b + i * KINC <= last) buf[i] = *(const u32x4 *)(xb + i * step);  // last < kend
        }
#pragma unroll
        for (int i = 0; i < NCH; ++i) buf[i] = OP::template admit<T, false>(buf[i], k0b + i * KINC, last);
        forget_derived(buf);
        op.template fold<T>(buf, ra, rb);
    }
    // lanes l, l^R, l^2R, ... hold parts of the same row; then the NW waves
#pragma unroll
    for (int off = R; off < 64; off <<= 1) OP::merge(ra, rb, __shfl_xor(ra, off, 64), __shfl_xor(rb, off, 64));
    if (lane < R) {
        red_a[w][lane] = ra;
        red_b[w][lane] = rb;
    }
    __syncthreads();
    ra = red_a[0][rl];
    rb = red_b[0][rl];
#pragma unroll
    for (int ww = 1; ww < NW; ++ww) OP::merge(ra, rb, red_a[ww][rl], red_b[ww][rl]);
    op.finish(ra, rb);
    forget_derived(buf);

    for (int bt = 0; bt < nbatches; ++bt) {
        const int k0b = kfirst + bt * NCH * KINC;
        const char *xb = xp + (int64_t)bt * NCH * step;
        char *ob = outp + (int64_t)bt * NCH * step;
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int k0 = k0b + i * KINC;
            if constexpr (!CACHED) {
                buf[i] = OP::template absent<T>();
                if (k0 <= last) buf[i] = *(const u32x4 *)(xb + i * step);
                buf[i] = OP::template admit<T, false>(buf[i], k0, last);
            }
            const u32x4 o = op.template emit<T, false>(buf[i], k0, last, ra, rb);
            if (k0 < kend) *(u32x4 *)(ob + i * step) = o;
        }
    }
}

// KV consecutive elements of a row-major row starting at column j, as one chunk (columns
// >= cols read as zero); VEC: one 16-byte access.
template <typename T, bool VEC>
__device__ __forceinline__ u32x4 row_chunk_load(const typename T::raw *xp, int j, int cols)
{
    if constexpr (VEC) {
        return *(const u32x4 *)(xp + j);
    } else {
        typename T::raw r[T::KV];
#pragma unroll
        for (int v = 0; v < T::KV; ++v) r[v] = j + v < cols ? xp[j + v] : (typename T::raw)0;
        u32x4 c;
        __builtin_memcpy(&c, r, 16);
        return c;
    }
}
template <typename T, bool VEC>
__device__ __forceinline__ void row_chunk_store(typename T::raw *op, int j, int cols, const u32x4 &c)
{
    if constexpr (VEC) {
        *(u32x4 *)(op + j) = c;
    } else {
        typename T::raw r[T::KV];
        __builtin_memcpy(r, &c, 16);
#pragma unroll
        for (int v = 0; v < T::KV; ++v)
            if (j + v < cols) op[j + v] = r[v];
    }
}

// The same operations on a row-major matrix, for the canonical-layout control: one
// workgroup per row, lanes along the row in chunks of KV elements (one 16-byte access when
// VEC says rows start and end on 16-byte boundaries).  The row is read twice; the second
// read comes from cache for rows of ordinary length.
template <typename T, typename OP, bool VEC>
__global__ __launch_bounds__(256) void row_major_kernel(RowArgs a)
{
    typedef typename T::raw raw;
    constexpr int KV = T::KV;
    __shared__ float red_a[4], red_b[4];
    const OP op(a);
    const int row = blockIdx.x % a.rows, b = blockIdx.x / a.rows;
    int last = (OP::kMasked && a.causal) ? row + (a.cols - a.rows) : a.cols - 1;
    last = last < a.cols - 1 ? last : a.cols - 1;
    const int64_t base = (int64_t)b * a.slot + (int64_t)row * a.row_stride;
    const raw *xp = (const raw *)(a.x + base);
    raw *outp = (raw *)(a.out + base);

    float ra, rb;
    OP::init(ra, rb);
    for (int j = threadIdx.x * KV; j <= last; j += 256 * KV) {
        u32x4 c[1] = {OP::template admit<T, true>(row_chunk_load<T, VEC>(xp, j, a.cols), j, last)};
        op.template fold<T>(c, ra, rb);
    }
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) OP::merge(ra, rb, __shfl_xor(ra, off, 64), __shfl_xor(rb, off, 64));
    if ((threadIdx.x & 63) == 0) {
        red_a[threadIdx.x >> 6] = ra;
        red_b[threadIdx.x >> 6] = rb;
    }
    __syncthreads();
    ra = red_a[0];
    rb = red_b[0];
#pragma unroll
    for (int ww = 1; ww < 4; ++ww) OP::merge(ra, rb, red_a[ww], red_b[ww]);
    op.finish(ra, rb);

    for (int j = threadIdx.x * KV; j < a.cols; j += 256 * KV) {
        u32x4 c = OP::template absent<T>();
        if (j <= last) c = OP::template admit<T, true>(row_chunk_load<T, VEC>(xp, j, a.cols), j, last);
        row_chunk_store<T, VEC>(outp, j, a.cols, op.template emit<T, true>(c, j, last, ra, rb));
    }
}

template <typename T, typename OP>
static hipError_t launch_row_dtype(const RowArgs &a, bool packed, hipStream_t st)
{
    if (!packed) {
        const int64_t grid = (int64_t)a.batch * a.rows;
        if (grid > kMaxGridX) return hipErrorInvalidConfiguration;
        const bool vec = ((uintptr_t)a.x | (uintptr_t)a.out | (uint64_t)a.row_stride | (uint64_t)a.slot |
                          (uint64_t)((int64_t)a.cols * T::ES)) % 16 == 0;
        if (vec)
            hipLaunchKernelGGL((row_major_kernel<T, OP, true>), dim3((unsigned)grid), dim3(256), 0, st, a);
        else
            hipLaunchKernelGGL((row_major_kernel<T, OP, false>), dim3((unsigned)grid), dim3(256), 0, st, a);
        return hipGetLastError();
    }
    // Variants: rows per workgroup, waves, cached.  A cached variant holds rows of up to
    // 128 * waves / R K blocks (16 chunks a lane).  The tuning hook LPG_TUNE_ROW_VARIANT pins the
    // choice if that variant can hold the rows.
    struct Variant { int r, nw; bool cached; };
    static const Variant kVariants[] = {{32, 8, true}, {16, 8, true}, {8, 8, true}, {8, 16, true},
                                        {8, 8, false}, {32, 4, true}};
    auto fits = [&](int v) { return !kVariants[v].cached || kVariants[v].r * a.nkb <= 128 * kVariants[v].nw; };
    int variant = fits(5) ? 5 : fits(0) ? 0 : fits(1) ? 1 : fits(2) ? 2 : fits(3) ? 3 : 4;  // short rows: 4 waves
    // few row groups (a 4096-row activation matrix has 128): fewer rows per workgroup, so that
    // the launch still has a couple of workgroups per compute unit
    const int64_t groups = (int64_t)a.batch * a.ngroups;
    while ((variant == 5 || variant == 0 || variant == 1) && groups * (32 / kVariants[variant].r) < 512)
        variant = variant == 5 ? 0 : variant + 1;
    {
        const int v = tune_get(LPG_TUNE_ROW_VARIANT);
        if (v >= 0 && v < 6 && fits(v)) variant = v;
    }
    if ((int64_t)a.batch * a.ngroups * (32 / kVariants[variant].r) > kMaxGridX) return hipErrorInvalidConfiguration;
    const unsigned grid = (unsigned)((int64_t)a.batch * a.ngroups * (32 / kVariants[variant].r));
    const dim3 block(kVariants[variant].nw * 64);
    switch (variant) {
        case 0: hipLaunchKernelGGL((row_packed_kernel<T, OP, 32, 8, true>), dim3(grid), block, 0, st, a); break;
        case 1: hipLaunchKernelGGL((row_packed_kernel<T, OP, 16, 8, true>), dim3(grid), block, 0, st, a); break;
        case 2: hipLaunchKernelGGL((row_packed_kernel<T, OP, 8, 8, true>), dim3(grid), block, 0, st, a); break;
        case 3: hipLaunchKernelGGL((row_packed_kernel<T, OP, 8, 16, true>), dim3(grid), block, 0, st, a); break;
        case 4: hipLaunchKernelGGL((row_packed_kernel<T, OP, 8, 8, false>), dim3(grid), block, 0, st, a); break;
        default: hipLaunchKernelGGL((row_packed_kernel<T, OP, 32, 4, true>), dim3(grid), block, 0, st, a); break;
    }
    return hipGetLastError();
}

hipError_t launch_row_op(const RowArgs &a, int op, int dtype, bool packed, hipStream_t st)
{
    if (a.batch <= 0 || a.rows <= 0 || a.cols <= 0) return hipSuccess;
    if (op == kRowSoftmax)
        return dtype == LPG_F32 ? launch_row_dtype<F32, SoftmaxRow>(a, packed, st) : launch_row_dtype<BF16, SoftmaxRow>(a, packed, st);
    return dtype == LPG_F32 ? launch_row_dtype<F32, RmsNormRow>(a, packed, st) : launch_row_dtype<BF16, RmsNormRow>(a, packed, st);
}

// ---------------------------------------------------------------------------------
// Rotary position embedding.  Tables: angle(t, i) = (pos0 + t) * base^(-2i/head_dim) in
// fp64, cos and sin rounded to fp32, row-major [rows][head_dim/2].
__global__ __launch_bounds__(256) void rope_tables_kernel(float *cos_t, float *sin_t, int64_t n, int half, double base,
                                                          double pos0)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= n) return;
    const int64_t t = idx / half;
    const int i = (int)(idx % half);
    const double ang = (pos0 + (double)t) * pow(base, -(double)i / (double)half);
    cos_t[idx] = (float)cos(ang);
    sin_t[idx] = (float)sin(ang);
}

hipError_t launch_rope_tables(float *cos_t, float *sin_t, int64_t rows, int head_dim, double base, double pos0,
                              hipStream_t st)
{
    const int64_t n = rows * (head_dim / 2);
    if (n <= 0) return hipSuccess;
    if ((n + 255) / 256 > kMaxGridX) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(rope_tables_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, cos_t, sin_t, n,
                       head_dim / 2, base, pos0);
    return hipGetLastError();
}

// On a packed left operand (row = position, columns = heads x head_dim).  Element i of a
// head's first half pairs with element i of its second half, head_dim/2 columns further:
// a whole number of fragments (the host checks head_dim % (2*KF) == 0), so the partner of
// a lane's chunk is the same lane's chunk of another fragment, and one wave rotates a
// fragment pair with four coalesced 1 KiB accesses.  Rows are the interleaved dimension
// of the layout: 32 positions rotate at once, each lane with its own row of the tables.
// Fragments numbered fk = k / KF over the whole row; a task is (slot, 32-row group, j):
// j < nlo rotates a pair, larger j zero-fills a fragment of column padding (out != x only).
template <typename T>
__global__ __launch_bounds__(256) void rope_packed_kernel(RopeArgs a)
{
    constexpr int KV = T::KV;
    const int lane = threadIdx.x & 63;
    const int h = lane >> 5, fl = lane & 31;
    const int64_t per_group = a.nlo + a.npad;
    const int64_t ntasks = (int64_t)a.batch * a.ngroups * per_group;
    for (int64_t task = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); task < ntasks; task += (int64_t)gridDim.x * 4) {
        const int j = (int)(task % per_group);
        const int64_t gb = task / per_group;
        const int g = (int)(gb % a.ngroups), b = (int)(gb / a.ngroups);
        const int64_t base = (int64_t)b * a.slot + (int64_t)g * kBlockBytes + lane * 16;
        if (j >= a.nlo) {
            const int fk = 2 * a.nlo + (j - a.nlo);
            *(u32x4 *)(a.out + base + (int64_t)(fk >> 2) * a.kbs + (fk & 3) * kFragBytes) = (u32x4){0u, 0u, 0u, 0u};
            continue;
        }
        const int head = j / a.fph, wi = j % a.fph;
        const int fk_lo = head * 2 * a.fph + wi, fk_hi = fk_lo + a.fph;
        const int64_t off_lo = base + (int64_t)(fk_lo >> 2) * a.kbs + (fk_lo & 3) * kFragBytes;
        const int64_t off_hi = base + (int64_t)(fk_hi >> 2) * a.kbs + (fk_hi & 3) * kFragBytes;
        const u32x4 lo = *(const u32x4 *)(a.x + off_lo), hi = *(const u32x4 *)(a.x + off_hi);
        const int row = 32 * g + fl;
        const int trow = row < a.rows ? row : a.rows - 1;  // padding rows: any valid table row, result unused
        const int i0 = wi * T::KF + 4 * h;
        const float *cp = a.cos_t + (int64_t)trow * a.half + i0, *sp = a.sin_t + (int64_t)trow * a.half + i0;
        float c[KV], s[KV];
#pragma unroll
        for (int q = 0; q < KV / 4; ++q) {
            const f32x4 cq = *(const f32x4 *)(cp + 8 * q), sq = *(const f32x4 *)(sp + 8 * q);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                c[4 * q + v] = cq[v];
                s[4 * q + v] = sq[v];
            }
        }
        float elo[KV], ehi[KV];
#pragma unroll
        for (int v = 0; v < KV; ++v) {
            const float x0 = chunk_elem<T>(lo, v), x1 = chunk_elem<T>(hi, v);
            elo[v] = row < a.rows ? fmaf(x0, c[v], -(x1 * s[v])) : 0.0f;
            ehi[v] = row < a.rows ? fmaf(x1, c[v], x0 * s[v]) : 0.0f;
        }
        *(u32x4 *)(a.out + off_lo) = chunk_from<T>(elo);
        *(u32x4 *)(a.out + off_hi) = chunk_from<T>(ehi);
    }
}

// Row-major twin for the control chain: one thread per pair, lanes along a head's half.
template <typename T>
__global__ __launch_bounds__(256) void rope_rows_kernel(RopeArgs a)
{
    typedef typename T::raw raw;
    const int64_t per_row = (int64_t)a.nheads * a.half;
    const int64_t n = (int64_t)a.batch * a.rows * per_row;
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < n; idx += (int64_t)gridDim.x * 256) {
        const int64_t p = idx % per_row, rb = idx / per_row;
        const int i = (int)(p % a.half), head = (int)(p / a.half);
        const int row = (int)(rb % a.rows), b = (int)(rb / a.rows);
        const int64_t base = (int64_t)b * a.slot + (int64_t)row * a.row_stride;
        const raw *xp = (const raw *)(a.x + base) + head * 2 * a.half + i;
        raw *outp = (raw *)(a.out + base) + head * 2 * a.half + i;
        float x0, x1;
        if constexpr (T::ES == 4) {
            x0 = __uint_as_float(xp[0]);
            x1 = __uint_as_float(xp[a.half]);
        } else {
            x0 = bf16_to_f32(xp[0]);
            x1 = bf16_to_f32(xp[a.half]);
        }
        const float c = a.cos_t[(int64_t)row * a.half + i], s = a.sin_t[(int64_t)row * a.half + i];
        const float y0 = fmaf(x0, c, -(x1 * s)), y1 = fmaf(x1, c, x0 * s);
        if constexpr (T::ES == 4) {
            outp[0] = __float_as_uint(y0);
            outp[a.half] = __float_as_uint(y1);
        } else {
            outp[0] = (raw)(bf16_pack2(y0, 0.0f) & 0xffffu);
            outp[a.half] = (raw)(bf16_pack2(y1, 0.0f) & 0xffffu);
        }
    }
}

hipError_t launch_rope(const RopeArgs &a, int dtype, bool packed, hipStream_t st)
{
    if (a.batch <= 0 || a.rows <= 0 || a.nheads <= 0) return hipSuccess;
    int64_t work = packed ? ((int64_t)a.batch * a.ngroups * (a.nlo + a.npad) + 3) / 4
                          : ((int64_t)a.batch * a.rows * a.nheads * a.half + 255) / 256;
    if (work > 256 * 32) work = 256 * 32;
    const dim3 grid((unsigned)work), block(256);
    if (packed) {
        if (dtype == LPG_F32) hipLaunchKernelGGL(rope_packed_kernel<F32>, grid, block, 0, st, a);
        else hipLaunchKernelGGL(rope_packed_kernel<BF16>, grid, block, 0, st, a);
    } else {
        if (dtype == LPG_F32) hipLaunchKernelGGL(rope_rows_kernel<F32>, grid, block, 0, st, a);
        else hipLaunchKernelGGL(rope_rows_kernel<BF16>, grid, block, 0, st, a);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// Fused attention on packed operands: O = softmax(scale * Q K^T [causal]) V per (batch, head),
// with the scores kept in registers.  This is layout propagation at register level: with K's
// fragment in the A slot and Q's in the B slot the MFMA leaves S^T tiles with lanes on the
// query index and registers on the key index, which (after exp and, for bf16, pairwise
// rounding) already are the fragments of P as a left operand of P V, so nothing is
// transposed or staged between the two products.  The row maximum and sum are per lane (one
// query) over registers, plus one exchange between the two half waves.
//
// Operands: Q = P(Q; tq, DH), K = P(K; tk, DH) (a left-operand image of K, i.e. the
// right-operand image of K^T), V = P(V; DH, tk) (right operand), O = P(O; tq, DH).
// A workgroup of four waves owns 128 queries (one 32-group per wave) of one (batch, head)
// and walks the keys 64 at a time; the 64 keys' fragments of K and V go through a two-stage
// LDS ring with the direct global->LDS transfer, one barrier per step.  Groups or K blocks
// that do not exist (ragged tk) are replaced by the last existing one; their keys are masked.
struct AttnFrag {
    // source of stage fragment f (0 <= f < NF) of key step j, for this lane
    template <typename T, int DH>
    __device__ __forceinline__ static const char *src(const AttnArgs &a, const char *Kb, const char *Vb, int f, int j,
                                                      int lane)
    {
        constexpr int FD = DH / T::KF, FK = 32 / T::KF, NFK = 2 * FD;
        if (f < NFK) {
            const int kg = f / FD, fd = f % FD;
            int grp = 2 * j + kg;
            grp = grp < a.k_groups ? grp : a.k_groups - 1;
            return Kb + (int64_t)(fd / 4) * a.k_kbs + (int64_t)grp * kBlockBytes + (fd % 4) * kFragBytes + lane * 16;
        }
        const int fv = f - NFK;
        const int dg = fv / (2 * FK), st = fv % (2 * FK);
        const int kidx = 64 * j + T::KF * st;
        int vkb = kidx / T::KB;
        vkb = vkb < a.v_nkb ? vkb : a.v_nkb - 1;
        return Vb + (int64_t)vkb * a.v_kbs + (int64_t)dg * kBlockBytes + ((kidx % T::KB) / T::KF) * kFragBytes + lane * 16;
    }
};

// SOFTMAX = false is the same walk without the softmax, O = (scale * Q K^T [causal]) V: the two
// chained GEMMs of the GEMM-only attention workloads with their intermediate in registers
// (bf16: rounded to bf16 exactly where the first GEMM's epilogue would have stored it).
// QG = 32-query groups per wave (a workgroup owns 128*QG queries): with two groups every K and
// V fragment read from LDS feeds two MFMAs instead of one, at twice the accumulator registers.
template <typename T, int DH, bool SOFTMAX, int QG>
__global__ __launch_bounds__(256) void attention_kernel(AttnArgs a)
{
    constexpr int NW = 4;
    constexpr int FD = DH / T::KF;  // fragments along d of a 32-row group of Q or K
    constexpr int FK = 32 / T::KF;  // fragments along the keys of a 32-key group (P and V)
    constexpr int DG = DH / 32;     // 32-groups of d
    constexpr int NFK = 2 * FD, NFV = DG * 2 * FK, NF = NFK + NFV, FPW = NF / NW;
    constexpr int STAGE = NF * kFragBytes;
    constexpr int GPB = NW * QG;    // query groups per block
    static_assert(NF % NW == 0, "stage must divide over the waves");
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const uint32_t sbase = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)smem;

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int h = lane >> 5;
    // Under a causal mask a query block's work grows with its position, so a workgroup takes
    // a pair: block p from the end, then block p from the start (the middle one alone when the
    // count is odd); every workgroup then walks the same number of key steps.
    const int nqb = (a.q_groups + GPB - 1) / GPB;
    const int pair = (int)(blockIdx.x / (uint32_t)a.batch);
    const int b = (int)(blockIdx.x % (uint32_t)a.batch);
    const int nparts = (a.causal && pair != nqb - 1 - pair) ? 2 : 1;
    const int shift = a.tk - a.tq;
    const float sl = a.sl;
    const char *Kb = a.K + (int64_t)(b / a.k_div) * a.k_slot;
    const char *Vb = a.V + (int64_t)(b / a.v_div) * a.v_slot;
    int ring = 0;  // steps issued so far: the ring stage alternates across the parts too
    auto issue = [&](int j, int stage) {
#pragma unroll
        for (int i = 0; i < FPW; ++i) {
            const int f = i * NW + w;
            lds_dma16(AttnFrag::src<T, DH>(a, Kb, Vb, f, j, lane), sbase + stage * STAGE + f * kFragBytes);
        }
    };

    for (int part = 0; part < nparts; ++part) {
        const int qb = a.causal ? (part == 0 ? nqb - 1 - pair : pair) : pair;
        const int g0 = (qb * NW + w) * QG;  // this wave's first query group
        // keys the workgroup has to walk
        int wg_last = a.causal ? 32 * (qb * GPB + GPB) - 1 + shift : a.tk - 1;
        wg_last = wg_last < a.tk - 1 ? wg_last : a.tk - 1;
        const int nsteps = wg_last < 0 ? 0 : wg_last / 64 + 1;
        // smallest `last` among this wave's lanes: steps wholly below it need no masking
        int wave_min_last = a.causal ? 32 * g0 + shift : a.tk - 1;
        wave_min_last = wave_min_last < a.tk - 1 ? wave_min_last : a.tk - 1;
        if (32 * (g0 + QG) - 1 >= a.tq) wave_min_last = -1;

        int last[QG];  // last key this lane's query of group x sees
        uint4 qf[QG][FD];
        f32x16 o[QG][DG];
        float m[QG], lsum[QG];  // reference maximum (shared by the half waves), this lane's part of the sum
#pragma unroll
        for (int x = 0; x < QG; ++x) {
            const int g = g0 + x, q = 32 * g + (lane & 31);
            last[x] = a.causal ? q + shift : a.tk - 1;
            last[x] = last[x] < a.tk - 1 ? last[x] : a.tk - 1;
            if (q >= a.tq) last[x] = -1;
#pragma unroll
            for (int fd = 0; fd < FD; ++fd) {
                qf[x][fd] = make_uint4(0u, 0u, 0u, 0u);
                if (g < a.q_groups)
                    qf[x][fd] = *(const uint4 *)(a.Q + (int64_t)b * a.q_slot + (int64_t)(fd / 4) * a.q_kbs +
                                                 (int64_t)g * kBlockBytes + (fd % 4) * kFragBytes + lane * 16);
            }
#pragma unroll
            for (int dg = 0; dg < DG; ++dg)
#pragma unroll
                for (int e = 0; e < 16; ++e) o[x][dg][e] = 0.0f;
            m[x] = kNegBig;
            lsum[x] = 0.0f;
        }

        // The stage written here was last read two steps ago (possibly by the previous part),
        // and every wave has passed the barrier of the step in between.
        if (nsteps > 0) issue(0, ring & 1);
        for (int j = 0; j < nsteps; ++j, ++ring) {
            wait_vmcnt<0>();
            __syncthreads();  // step j's fragments are in LDS; everyone is done reading the other stage
            if (j + 1 < nsteps) issue(j + 1, (ring + 1) & 1);
            const char *sb = smem + (ring & 1) * STAGE + lane * 16;

            // S^T tiles: registers run along 32 keys, lanes along 32 queries
            f32x16 s[QG][2];
#pragma unroll
            for (int kg = 0; kg < 2; ++kg) {
#pragma unroll
                for (int x = 0; x < QG; ++x)
#pragma unroll
                    for (int e = 0; e < 16; ++e) s[x][kg][e] = 0.0f;
#pragma unroll
                for (int fd = 0; fd < FD; ++fd) {
                    const uint4 kf = *(const uint4 *)(sb + (kg * FD + fd) * kFragBytes);
#pragma unroll
                    for (int x = 0; x < QG; ++x) mma_frag<T>(s[x][kg], kf, qf[x][fd]);
                }
            }
            // key of register e of tile kg: 64j + 32kg + 8(e/4) + 4h + e%4
            const int key0 = 64 * j + 4 * h;
            const bool masked = 64 * j + 63 > wave_min_last;  // wave-uniform
#pragma unroll
            for (int x = 0; x < QG; ++x) {
                if (masked) {
                    const float gone = SOFTMAX ? -__builtin_inff() : 0.0f;
#pragma unroll
                    for (int kg = 0; kg < 2; ++kg)
#pragma unroll
                        for (int e = 0; e < 16; ++e)
                            s[x][kg][e] = (key0 + 32 * kg + 8 * (e >> 2) + (e & 3) <= last[x]) ? s[x][kg][e] : gone;
                }
                if constexpr (SOFTMAX) {
                    float bmx = -__builtin_inff();
#pragma unroll
                    for (int kg = 0; kg < 2; ++kg)
#pragma unroll
                        for (int e = 0; e < 16; ++e) bmx = fmaxf(bmx, s[x][kg][e]);
                    bmx = fmaxf(bmx, __shfl_xor(bmx, 32, 64));
                    // The reference point m of the exponentials only has to stay within 2^8 of the
                    // true running maximum (the final division cancels it), so O and the sum are
                    // rescaled only in the steps where some query of the wave moved further than that.
                    const float bm = bmx * sl;
                    if (__any(bm > m[x] + 8.0f)) {
                        const float mn = fmaxf(m[x], bm);
                        const float alpha = __builtin_amdgcn_exp2f(m[x] - mn);
                        m[x] = mn;
                        lsum[x] *= alpha;
#pragma unroll
                        for (int dg = 0; dg < DG; ++dg)
#pragma unroll
                            for (int e = 0; e < 16; ++e) o[x][dg][e] *= alpha;
                    }
                    float psum = 0.0f;
#pragma unroll
                    for (int kg = 0; kg < 2; ++kg)
#pragma unroll
                        for (int e = 0; e < 16; ++e) {
                            s[x][kg][e] = __builtin_amdgcn_exp2f(fmaf(s[x][kg][e], sl, -m[x]));
                            psum += s[x][kg][e];
                        }
                    lsum[x] += psum;
                } else if (a.scale != 1.0f) {
#pragma unroll
                    for (int kg = 0; kg < 2; ++kg)
#pragma unroll
                        for (int e = 0; e < 16; ++e) s[x][kg][e] *= a.scale;
                }
            }
            // P's fragments are the registers as they stand (bf16: rounded in pairs); O^T += V^T P^T
#pragma unroll
            for (int kg = 0; kg < 2; ++kg)
#pragma unroll
                for (int c = 0; c < FK; ++c) {
                    uint4 pf[QG];
#pragma unroll
                    for (int x = 0; x < QG; ++x) {
                        const f32x16 &t = s[x][kg];
                        if constexpr (T::ES == 4) {
                            pf[x] = make_uint4(__float_as_uint(t[4 * c]), __float_as_uint(t[4 * c + 1]),
                                               __float_as_uint(t[4 * c + 2]), __float_as_uint(t[4 * c + 3]));
                        } else {
                            pf[x] = make_uint4(bf16_pack2(t[8 * c], t[8 * c + 1]), bf16_pack2(t[8 * c + 2], t[8 * c + 3]),
                                               bf16_pack2(t[8 * c + 4], t[8 * c + 5]), bf16_pack2(t[8 * c + 6], t[8 * c + 7]));
                        }
                    }
#pragma unroll
                    for (int dg = 0; dg < DG; ++dg) {
                        const uint4 vf = *(const uint4 *)(sb + (NFK + dg * 2 * FK + kg * FK + c) * kFragBytes);
#pragma unroll
                        for (int x = 0; x < QG; ++x) mma_frag<T>(o[x][dg], vf, pf[x]);
                    }
                }
        }
#pragma unroll
        for (int x = 0; x < QG; ++x) {
            const int g = g0 + x, q = 32 * g + (lane & 31);
            if (g >= a.q_groups) continue;
            const float l = SOFTMAX ? lsum[x] + __shfl_xor(lsum[x], 32, 64) : 1.0f;
            const float inv = (l > 0.0f && q < a.tq) ? 1.0f / l : 0.0f;  // padding rows and rows without keys: zeros
            char *Ob = a.O + (int64_t)b * a.o_slot + (int64_t)g * kBlockBytes + lane * 16;
#pragma unroll
            for (int dg = 0; dg < DG; ++dg) {
                float v[16];
#pragma unroll
                for (int e = 0; e < 16; ++e) v[e] = o[x][dg][e] * inv;
                if constexpr (T::ES == 4) {
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        *(uint4 *)(Ob + (int64_t)dg * a.o_kbs + c * kFragBytes) =
                            make_uint4(__float_as_uint(v[4 * c]), __float_as_uint(v[4 * c + 1]), __float_as_uint(v[4 * c + 2]),
                                       __float_as_uint(v[4 * c + 3]));
                } else {
#pragma unroll
                    for (int c = 0; c < 2; ++c)
                        *(uint4 *)(Ob + (int64_t)(dg >> 1) * a.o_kbs + (2 * (dg & 1) + c) * kFragBytes) =
                            make_uint4(bf16_pack2(v[8 * c], v[8 * c + 1]), bf16_pack2(v[8 * c + 2], v[8 * c + 3]),
                                       bf16_pack2(v[8 * c + 4], v[8 * c + 5]), bf16_pack2(v[8 * c + 6], v[8 * c + 7]));
                }
            }
        }
    }
    wait_vmcnt<0>();  // no transfer into this workgroup's LDS may outlive the wave
}

template <typename T, int DH, bool SOFTMAX, int QG>
static hipError_t launch_attention_dh(const AttnArgs &a, hipStream_t st)
{
    constexpr int NF = 2 * (DH / T::KF) + (DH / 32) * 2 * (32 / T::KF);
    constexpr size_t lds = 2 * (size_t)NF * kFragBytes;
    static_assert(lds <= 160 * 1024, "ring does not fit the LDS");
    auto kern = attention_kernel<T, DH, SOFTMAX, QG>;
    if (lds > (size_t)device_info().lds_bytes) return hipErrorInvalidConfiguration;
    if (lds > 64 * 1024) {
        static PerDeviceFlag raised;
        if (first_use_on_device(raised)) {
            hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            mark_used_on_device(raised);
        }
    }
    const int nqb = (a.q_groups + 4 * QG - 1) / (4 * QG);
    const int64_t grid = (int64_t)(a.causal ? (nqb + 1) / 2 : nqb) * a.batch;  // causal: query blocks in pairs
    if (grid > kMaxGridX) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), lds, st, a);
    return hipGetLastError();
}

// Two query groups per wave pay only where a launch keeps several workgroups per compute
// unit even so and all of them do the same work: bf16, head_dim 64, no causal mask, at least
// 512 workgroups (measured 113 against 123 us on 32 heads x 4096 x 4096; under a causal mask the
// larger blocks lose more to imbalance than the reuse gives).  The tuning hook LPG_TUNE_ATTN_QUERY_GROUPS (1 or 2)
// pins the choice for head_dim 64.
template <typename T, int DH>
static hipError_t launch_attention_mode(const AttnArgs &a, hipStream_t st)
{
    if constexpr (DH == 64) {
        const int64_t wgs2 = (int64_t)((a.q_groups + 7) / 8) * a.batch;
        int qg = (T::ES == 2 && !a.causal && wgs2 >= 512) ? 2 : 1;
        const int force = tune_get(LPG_TUNE_ATTN_QUERY_GROUPS);
        if (force == 1 || force == 2) qg = force;
        if (qg == 2)
            return a.softmax ? launch_attention_dh<T, DH, true, 2>(a, st) : launch_attention_dh<T, DH, false, 2>(a, st);
    }
    return a.softmax ? launch_attention_dh<T, DH, true, 1>(a, st) : launch_attention_dh<T, DH, false, 1>(a, st);
}

hipError_t launch_attention(const AttnArgs &a, int dtype, int head_dim, hipStream_t st)
{
    if (a.batch <= 0 || a.tq <= 0) return hipSuccess;
    if (head_dim == 64)
        return dtype == LPG_F32 ? launch_attention_mode<F32, 64>(a, st) : launch_attention_mode<BF16, 64>(a, st);
    if (head_dim == 128)
        return dtype == LPG_F32 ? launch_attention_mode<F32, 128>(a, st) : launch_attention_mode<BF16, 128>(a, st);
    return hipErrorInvalidValue;
}

// Estimated run time (cycles of the busiest compute unit) of one GEMM with a tile
// configuration.  Three terms: MFMA time, derated when only one wave feeds a SIMD or when a
// wave's tile is so small that LDS reads per MFMA dominate; the L2->LDS transfer time that
// does not hide behind the MFMAs; and a fixed cost per tile (epilogue, pipeline refill).
// The constants were fitted to measured timings of the benchmark shapes on MI355X.
static double estimate_cost(const GemmArgs &a, const TileCfg &c, bool bf16)
{
    const int64_t tl = (a.FLg + c.tlg - 1) / c.tlg, tr = (a.FRg_out + c.trg - 1) / c.trg;
    const int64_t tiles = tl * tr * a.batch;
    const int ncu = device_info().ncu;
    const int occ = workgroups_per_cu(c, bf16);
    const int64_t per_cu = (tiles + ncu - 1) / ncu;  // tiles the busiest CU runs
    const int wtl = c.tlg / c.wl, wtr = c.trg / c.wr;
    const double waves_per_simd = (double)(c.wl * c.wr) / 4.0;
    const int nkb = a.nkb > 0 ? a.nkb : 1;
    const double cy_block = bf16 ? 128.0 : 1024.0;  // MFMA cycles of one 32x32 tile over one K block
    const int resident = (int)((per_cu < occ ? per_cu : occ) * waves_per_simd);  // waves per SIMD
    // one bf16 wave per SIMD stalls at every barrier of its short steps, unless the launch
    // qualifies for two K blocks per step (launch_gemm_cfg)
    const bool two_block = tiles <= ncu && c.tlg * c.trg <= 8 && nkb % 2 == 0 && nkb >= 4;
    double eff = resident >= 2 ? 1.0 : (bf16 ? (two_block ? 0.9 : 0.6) : 1.0);
    const double reads_per_mma = (double)(wtl + wtr) / (wtl * wtr);
    eff /= 1.0 + (bf16 ? 0.217 : 0.0525) * reads_per_mma;
    const double mfma = (double)per_cu * (c.tlg * c.trg / 4.0) * nkb * cy_block / eff;
    const double traffic = (double)per_cu * nkb * (c.tlg + c.trg) * 205.0 * (bf16 ? 0.141 : 0.0805);
    const double fixed = (double)per_cu * (c.tlg * c.trg * (bf16 ? 60.0 : 32.0) + 2228.0);
    return mfma + traffic + fixed;
}

int choose_gemm_config(const GemmArgs &a, int in_dtype)
{
    const bool bf16 = in_dtype == LPG_BF16;
    // A contraction of at most 256 (attention scores, whatever the head_dim) with at least two
    // tiles per compute unit makes the launch a stream of epilogues bound by the stores; the
    // cost model has no term for that.  Measured on 32 heads of 2048^2 / 4096^2 scores: two
    // workgroups per compute unit, so that one stores while the other multiplies, with 256 x 128
    // tiles in bf16 (192-205 us on 4096^2 against 201-215 for 128 x 256 and 197-222 for the
    // others) and 128 x 128 in fp32 (174-185 against 180-199).
    {
        const int pick = bf16 ? 4 : 3;
        const TileCfg &c = kCfgs[pick];
        const int64_t tiles = (int64_t)((a.FLg + c.tlg - 1) / c.tlg) * ((a.FRg_out + c.trg - 1) / c.trg) * a.batch;
        if (a.nkb * (bf16 ? 64 : 32) <= 256 && tiles >= 512) return pick;
    }
    int best = 3;
    double best_cost = 1e300;
    for (int i = 0; i < kNumCfgs; ++i) {
        const double c = estimate_cost(a, kCfgs[i], bf16);
        if (c < best_cost * 0.9995) {  // later (larger) configurations must win clearly
            best_cost = c;
            best = i;
        }
    }
    return best;
}

hipError_t launch_gemm(const GemmArgs &a, int in_dtype, int out_dtype, int cfg, hipStream_t st)
{
    if (cfg < 0 || cfg >= kNumCfgs) cfg = choose_gemm_config(a, in_dtype);
    if (tune_get(LPG_TUNE_TRACE) > 0)
        fprintf(stderr, "lpg gemm: FL %d FR %d nkb %d batch %d -> tile configuration %d\n", a.FL, a.FR, a.nkb, a.batch, cfg);
    if (in_dtype == LPG_F32 && out_dtype == LPG_F32) return launch_gemm_f32(a, cfg, st);
    if (in_dtype == LPG_BF16 && out_dtype == LPG_BF16) return launch_gemm_bf16(a, cfg, st);
    if (in_dtype == LPG_BF16 && out_dtype == LPG_F32) return launch_gemm_bf16_f32(a, cfg, st);
    return hipErrorInvalidValue;
}

hipError_t launch_gemm_gather(const GatherArgs &a, int in_dtype, int out_dtype, hipStream_t st)
{
    if (in_dtype == LPG_F32 && out_dtype == LPG_F32) return launch_gemm_gather_f32(a, st);
    if (in_dtype == LPG_BF16 && out_dtype == LPG_BF16) return launch_gemm_gather_bf16(a, st);
    if (in_dtype == LPG_BF16 && out_dtype == LPG_F32) return launch_gemm_gather_bf16_f32(a, st);
    return hipErrorInvalidValue;
}

}  // namespace lpg
