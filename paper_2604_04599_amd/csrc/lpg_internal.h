// Internal declarations shared by the host API (lpg_api.cpp) and the device
// code (lpg_kernels.hip) of the GPU path.  Nothing here is used by the CPU checker.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/lpg.h"
#include "lpg_addr.h"

namespace lpg {

// Packed-layout constants.  A fragment is 64 lanes x 16 bytes = 1 KiB, a block is
// four fragments = 32 free indices x KB contraction indices = 4 KiB, for both dtypes.
constexpr int kFragBytes = 1024;
constexpr int kBlockBytes = 4096;
constexpr int kFragsPerBlock = 4;

// Tuning and test hooks (lpg_tune_set): process-wide, -1 = the library's own choice.
int tune_get(int key);
int tune_set(int key, int value);  // 0, or -1 for an unknown key

// What the library needs to know of the device a launch goes to, queried once per device.
struct DeviceInfo {
    int ncu;        // compute units
    int lds_bytes;  // LDS a workgroup may use
};
const DeviceInfo &device_info();

// True the first time it is called for (flag, current device): guards per-device, per-kernel
// set-up such as hipFuncSetAttribute.  Safe to call from several threads (the set-up it guards is
// idempotent, so two threads doing it once each is harmless).
struct PerDeviceFlag {
    unsigned long long done[2] = {0, 0};  // one bit per device ordinal (up to 128)
};
bool first_use_on_device(PerDeviceFlag &f);
void mark_used_on_device(PerDeviceFlag &f);

inline int elem_size(int dtype) { return dtype == LPG_F32 ? 4 : 2; }
inline int kb_of(int dtype) { return dtype == LPG_F32 ? 32 : 64; }  // K extent of a block

// A packed descriptor reduced to what kernels need (all in bytes unless noted).
struct PView {
    int dtype, es;
    int64_t F, K;          // logical extents of one view (free, contraction)
    int64_t PF, PK;        // logical extents of the parent
    int64_t PFp, PKp;      // padded extents of the parent
    int64_t f0, k0;        // origin of slot 0's view (elements)
    int64_t fstep, kstep;  // origin shift per slot (elements)
    int batch, bdiv;
    int64_t bstride;       // elements between parents of consecutive slots
    int64_t kb_stride;     // bytes between consecutive K blocks of the parent
    int64_t g_stride;      // bytes between consecutive 32-groups of the free dimension
    bool default_order;    // the strides are the default ones (groups back to back, K blocks back to back)
    int64_t origin;        // bytes from buffer start to slot 0's first block
    int64_t slot_step;     // bytes added per slot
    bool transposed;       // kind == PACKED_B (free = cols)
    bool keep_f, keep_k;   // ragged extent ending inside the parent: its last block is shared
    int f_off, k_off;      // origin's distance from the 32 / KB grid (origin points at the block that holds it)
};

// A canonical descriptor reduced to strides over (free, contraction) indices.
struct CView {
    int dtype, es;
    int64_t rows, cols;
    int64_t row_stride, col_stride;  // elements
    int64_t origin;                  // elements
    int64_t slot_step;               // elements
    int batch, bdiv;
};

struct PackArgs {
    const char *canon;   // canonical buffer + origin (bytes applied)
    char *packed;        // packed buffer + origin
    int64_t sf, sk;      // canonical strides (elements) along free / contraction index
    int64_t c_slot;      // canonical bytes per slot
    int64_t p_kbs;       // packed bytes between K blocks
    int64_t p_gs;        // packed bytes between 32-groups
    int64_t p_slot;      // packed bytes per slot
    int32_t c_div, p_div;
    int32_t F, K;        // logical extents
    int32_t ngroups;     // ceil(F/32)
    int32_t nkb;         // ceil(K/KB)
    int32_t batch;
    int32_t kpw;         // K blocks per workgroup (set by the launcher)
    int32_t keep_f, keep_k;  // pack: leave packed elements past F / past K untouched
    int32_t f_off, k_off;    // view origin inside its first block (off the 32 / KB grid when non-zero)
};

struct GemmArgs {
    const char *L;       // operand whose free index lands on lanes (out's free dimension)
    const char *R;       // operand whose free index lands on registers (out's contraction dim)
    const char *Cin;     // may be null (beta == 0)
    const char *Epi;     // may be null
    char *Out;
    int64_t l_kbs, r_kbs, o_kbs;     // bytes between K blocks (packed operands)
    int64_t l_gs, r_gs, o_gs;        // bytes between 32-groups of the free dimension (packed operands)
    int64_t l_slot, r_slot, o_slot;  // bytes per slot
    // Canonical (row/column-major) operands read or written directly, without a pack or
    // unpack pass: the fused Initial / Ending kernels.  Inputs: fp32, contiguous along k;
    // l_ld / r_ld = bytes between consecutive free indices.  Output: o_sf / o_sk = bytes per
    // step of out's lane index (free) and register index (contraction).
    int32_t l_canon, r_canon, o_canon;
    int64_t l_ld, r_ld;
    int64_t o_sf, o_sk;
    int32_t l_div, r_div;
    int32_t l_foff, r_foff;          // packed inputs: rows between the view's origin and the 32-grid (read views)
    int32_t FL, FR;                  // logical extents of out: free dim, contraction dim
    int32_t FLg, FRg;                // 32-groups present in L and R
    int32_t FRg_out;                 // 32-groups of out's contraction dim incl. block padding
    int32_t nkb;                     // contraction blocks of the product
    int32_t batch;
    int32_t epi;
    float alpha, beta;
    int32_t o_keep_l, o_keep_r;      // packed out: leave elements past FL / past FR untouched
    // o_canon == 2: packed out whose origin is off the 32 / KB grid; Out points at the block holding
    // the origin, the view starts o_foff free indices and o_koff contraction indices into it
    int32_t o_foff, o_koff;
    TileWalk walk;                   // order in which the launch's tiles are walked (set by the launcher)
    DivBy by_ldiv, by_rdiv;          // division by l_div / r_div (set by the launcher)
    int32_t o_stream;                // plain packed output written with streaming (non-temporal) stores
};

// One input of the general (gathering) GEMM kernel: any canonical matrix (any strides, fp32 or
// bf16 elements) or any view of a packed parent, read element by element.
struct GatherOperand {
    const char *base;     // canonical: element (0, 0) of slot 0's view; packed: the block that holds the view's origin
    int64_t slot;         // bytes per slot
    int64_t sf, sk;       // canonical: byte strides along the free and the contraction index
    int64_t kbs, gs;      // packed: bytes between K blocks / between 32-groups
    int32_t div;          // matrix b uses slot b / div
    int32_t packed;       // 0: canonical, 1: view of a packed parent
    int32_t mode;         // how its lane vectors are fetched (kGather* in lpg_gemm.h), chosen on the host
    int32_t es;           // bytes of a source element (4: fp32, converted if the GEMM multiplies bf16; 2: bf16)
    int32_t foff, koff;   // packed: the origin's distance from the 32 / KB grid
    int32_t F, K;         // logical extents; what lies outside reads as zero
};

struct GatherArgs {
    GemmArgs g;           // output side, extents, alpha / beta / epilogue, tile walk (L, R and their strides unused)
    GatherOperand l, r;   // the operand on lanes (out's free dimension) and the one on registers
};

struct EwArgs {
    const char *x0, *x1;
    char *out;
    int64_t n16;  // number of whole 16-byte chunks
    int32_t tail; // elements after the last whole chunk (tight canonical buffers of odd sizes)
    int32_t op;
    float s;
};

// Row operations (softmax, RMS normalisation) on a packed left operand or a row-major matrix.
enum { kRowSoftmax = 0, kRowRmsNorm = 1 };
struct RowArgs {
    const char *x;       // buffer + origin (bytes applied)
    char *out;
    const float *weight; // RMS normalisation: per-column weights
    int64_t kbs;         // packed: bytes between K blocks
    int64_t row_stride;  // canonical: bytes between rows
    int64_t slot;        // bytes per slot
    int32_t rows, cols;  // logical extents (packed: free, contraction)
    int32_t ngroups;     // packed: ceil(rows/32)
    int32_t nkb;         // packed: ceil(cols/KB)
    int32_t batch;
    int32_t causal;      // softmax
    float scalar;        // softmax: scale * log2(e); RMS normalisation: eps
};

struct RopeArgs {
    const char *x;       // buffer + origin (bytes applied)
    char *out;
    const float *cos_t, *sin_t;  // [rows][half]
    int64_t kbs, row_stride, slot;
    int32_t rows, nheads, half;  // half = head_dim / 2
    int32_t ngroups, batch;
    int32_t fph;         // packed: fragments per half head
    int32_t nlo;         // packed: fragment pairs per 32-row group = nheads * fph
    int32_t npad;        // packed: fragments of column padding to zero-fill (0 when in place)
};

struct AttnArgs {
    const char *Q, *K, *V;  // buffers + origins (bytes applied)
    char *O;
    int64_t q_kbs, k_kbs, v_kbs, o_kbs;      // bytes between K blocks
    int64_t q_slot, k_slot, v_slot, o_slot;  // bytes per slot
    int32_t k_div, v_div;                    // query heads per key / value head
    int32_t tq, tk;                          // queries, keys
    int32_t q_groups, k_groups;              // ceil(tq/32), ceil(tk/32)
    int32_t v_nkb;                           // ceil(tk/KB): contraction blocks of V
    int32_t batch, causal, softmax;
    float sl;                                // scale * log2(e) (softmax)
    float scale;                             // scale (no softmax)
};

// Launchers (lpg_kernels.hip).  Return hipError_t of the launch.
hipError_t launch_pack(const PackArgs &a, int src_dtype, int dst_dtype, hipStream_t st);
hipError_t launch_unpack(const PackArgs &a, int src_dtype, int dst_dtype, hipStream_t st);
// cfg < 0 lets the library choose the tile configuration.
hipError_t launch_gemm(const GemmArgs &a, int in_dtype, int out_dtype, int cfg, hipStream_t st);
// One translation unit per dtype pair (lpg_gemm_*.hip); cfg is a valid tile configuration index.
hipError_t launch_gemm_f32(const GemmArgs &a, int cfg, hipStream_t st);
hipError_t launch_gemm_bf16(const GemmArgs &a, int cfg, hipStream_t st);
hipError_t launch_gemm_bf16_f32(const GemmArgs &a, int cfg, hipStream_t st);
// The general kernel: operands gathered element by element (any layout, view, conversion).
hipError_t launch_gemm_gather(const GatherArgs &a, int in_dtype, int out_dtype, hipStream_t st);
hipError_t launch_gemm_gather_f32(const GatherArgs &a, hipStream_t st);
hipError_t launch_gemm_gather_bf16(const GatherArgs &a, hipStream_t st);
hipError_t launch_gemm_gather_bf16_f32(const GatherArgs &a, hipStream_t st);
int choose_gemm_config(const GemmArgs &a, int in_dtype);
hipError_t launch_elementwise(const EwArgs &a, int dtype, hipStream_t st);
hipError_t launch_row_op(const RowArgs &a, int op, int dtype, bool packed, hipStream_t st);
hipError_t launch_rope_tables(float *cos_t, float *sin_t, int64_t rows, int head_dim, double base, double pos0,
                              hipStream_t st);
hipError_t launch_rope(const RopeArgs &a, int dtype, bool packed, hipStream_t st);
hipError_t launch_attention(const AttnArgs &a, int dtype, int head_dim, hipStream_t st);

// The library's own device scratch (lpg_chain_static): address of the current device's copy and
// its size.  Allocates nothing.
hipError_t static_scratch(void **ptr, size_t *bytes);

}  // namespace lpg
