/*
 * lpg.h - layout-propagating GEMM chains on one MI355X (gfx950).  C ABI.
 *
 * A chain of dependent GEMMs  C_i = alpha_i * A_i * B_i + beta_i * C_i  (paper
 * Eq. 1, chained as in Eq. 2) in which every intermediate stays in the packed,
 * MFMA-fragment-ordered layout that the next GEMM's loads consume: matrices are
 * packed once at the chain's entry and unpacked once at its exit (the paper's
 * Initial / Intermediate / Ending decomposition, section III-A), so row/column
 * major semantics hold only at the boundaries.
 *
 * General rules for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller; descriptors and
 *     stage arrays are HOST memory read during the call only.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is enqueued asynchronously; no call synchronises or allocates.
 *   - Return value: LPG_OK (0) or a negative lpg_status.  Errors are detected on
 *     the host before anything is launched; lpg_last_error() gives a message.
 *   - Packed buffers must be 16-byte aligned (LPG_EALIGN otherwise).
 *   - Sizes: rows and cols up to 2^31-1 each (LPG_EINVAL past that); every byte
 *     offset is formed in 64 bits, so buffers, slots and leading dimensions may
 *     pass 4 GiB.  A request whose launch would exceed the device's grid limits
 *     (lpg_pack / lpg_unpack: more than 65535 batches or K blocks; any call: more
 *     than 2^31-1 workgroups or output tiles) returns LPG_EUNSUPPORTED or LPG_EHIP
 *     and launches nothing.
 *
 * The packed layout P(X; F, K) (this library's re-design, for 64-lane MFMA
 * operand registers, of the tile order of Eq. 3).  X has a free dimension F and
 * a contraction dimension K.  With es = element size, KV = 16/es, KF = 2*KV,
 * KB = 4*KF (fp32: 4, 8, 32; bf16: 8, 16, 64), F padded to 32 and K to KB with
 * zeros, the nested dimensions are, outermost to innermost,
 *        [K/KB] [F/32] [4 fragments] [2 lane halves h] [32 lanes fl] [KV v]
 * and  k = KB*kb + KF*c + 8*(v/4) + 4*h + v%4,  f = 32*g + fl.
 * One fragment (1 KiB) is exactly one 128-bit-per-lane wave load and is the
 * operand register image of v_mfma_f32_32x32x2_f32 (four of them per fragment)
 * or v_mfma_f32_32x32x16_bf16 (one).  A 32x32 accumulator tile, as the MFMA
 * leaves it in registers, is already a run of fragments of the output's packed
 * layout, so the epilogue stores it with plain 128-bit stores.
 *   LPG_PACKED_A = P(X; F = rows, K = cols): X will be a LEFT operand.
 *   LPG_PACKED_B = P(X; F = cols, K = rows): X will be a RIGHT operand.
 * PACKED_A of X and PACKED_B of X^T are the same bytes.
 */
#ifndef LPG_H
#define LPG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LPG_OK = 0,
    LPG_EINVAL = -1,       /* bad argument (NULL, negative size, shape mismatch)        */
    LPG_ELAYOUT = -2,      /* descriptor kinds / packed geometry do not fit together    */
    LPG_EUNSUPPORTED = -3, /* dtype combination or option not implemented               */
    LPG_EALIGN = -4,       /* pointer or view origin not aligned as the layout needs    */
    LPG_EHIP = -5,         /* a HIP runtime call failed                                 */
    LPG_EWORKSPACE = -6    /* lpg_chain: workspace too small                            */
} lpg_status;

typedef enum { LPG_F32 = 0, LPG_BF16 = 1 } lpg_dtype;

typedef enum {
    LPG_ROW_MAJOR = 0, /* canonical, boundaries only */
    LPG_COL_MAJOR = 1, /* canonical, boundaries only */
    LPG_PACKED_A = 2,
    LPG_PACKED_B = 3
} lpg_kind;

/*
 * Descriptor of a (batched) matrix or of a view into a larger parent.
 *
 * rows, cols          logical extent of one matrix.
 * ld                  canonical kinds: leading dimension in elements (0 = tight:
 *                     parent_cols for row-major, parent_rows for column-major).
 * parent_rows/cols    extent of the parent this view lives in (0,0 = the view is
 *                     the whole parent).  For packed kinds the parent fixes the
 *                     padded geometry (block strides).
 * row0, col0          origin of the view inside the parent.  Packed kinds: the row,
 *                     elementwise and attention entry points and batched views with a
 *                     per-slot origin step need the free-dimension origin to be a
 *                     multiple of 32 and the contraction-dimension origin a multiple of
 *                     KB (LPG_EALIGN otherwise), and a view extent that is not such a
 *                     multiple must end at the parent's edge (its padding is then the
 *                     parent's own zero padding).  A and B of lpg_gemm_packed take any
 *                     origin and any extent inside the parent: what lies outside the
 *                     view never enters a sum.
 *                     WRITTEN views - the destination of lpg_pack, the source of
 *                     lpg_unpack, and C / C_in / epi_arg of lpg_gemm_packed - may
 *                     have any origin and any extent inside the parent: the call
 *                     touches the view's own elements only, as if the rectangle had
 *                     been replaced in the canonical parent and the parent packed
 *                     again.  With an origin on the 32 / KB grid whole 16-byte lane
 *                     vectors are moved (edge blocks element by element); with an
 *                     origin off the grid every element is addressed by itself and
 *                     the parent's padding is never written, so the parent must
 *                     have been zero-filled or packed once before.  This is the
 *                     general form of the paper's "store stride / block order"
 *                     parameters (section III-C): per-head slices of Q, K, V, O
 *                     (section IV-A), and appends of any number of rows or columns
 *                     at any position of a growing operand (a key / value cache).
 * batch               number of matrices (0 is read as 1).
 * batch_div           matrix b uses slot b / batch_div (0 is read as 1); lets
 *                     several query heads share one key/value head instead of
 *                     replicating it (Alg. 2, head-wise replication step).
 * batch_stride        elements between the parents of consecutive slots (0 = all
 *                     slots share one parent).
 * batch_row_step,
 * batch_col_step      shift of the view origin per slot inside the parent.
 * group_stride,
 * kblock_stride       packed kinds: the paper's "block order" and "store stride" parameters
 *                     (section III-C).  The packed parent is a grid of blocks, [K/KB] K blocks
 *                     by [F/32] groups of the free dimension, each block 32 x KB elements
 *                     (4 KiB) in the fragment order above.  group_stride = elements from one
 *                     group's block to the next group's, kblock_stride = elements from one K
 *                     block to the next; 0 = the default order, groups back to back inside a
 *                     K block (group_stride = 32*KB) and K blocks back to back (kblock_stride
 *                     = padded F * KB).  Other values change the order in which the blocks lie
 *                     in memory (groups outermost: group_stride = padded K * 32, kblock_stride
 *                     = 32*KB, which makes a row range of a left operand one contiguous run)
 *                     or leave room between them (a stride larger than what the blocks need:
 *                     the room is never read or written).  Both must be multiples of one block
 *                     (32*KB elements) and must not make blocks overlap (LPG_EINVAL).  lpg_pack,
 *                     lpg_unpack, lpg_gemm_packed (A, B, C, C_in, epi_arg), lpg_chain and
 *                     lpg_layout_offset take them; the elementwise, row and attention entry
 *                     points work on default-ordered buffers only (LPG_EUNSUPPORTED).
 */
typedef struct lpg_desc {
    int32_t kind;
    int32_t dtype;
    int64_t rows, cols;
    int64_t ld;
    int64_t parent_rows, parent_cols;
    int64_t row0, col0;
    int32_t batch;
    int32_t batch_div;
    int64_t batch_stride;
    int64_t batch_row_step, batch_col_step;
    int64_t group_stride, kblock_stride;
} lpg_desc;

/* Elementwise operations on packed buffers (layout-oblivious; paper II-C, IV-A). */
typedef enum {
    LPG_EW_SCALE = 0,   /* out = s * x0            (x1 ignored)                          */
    LPG_EW_ADD = 1,     /* out = x0 + s * x1                                             */
    LPG_EW_SILU_MUL = 2 /* out = x0 * sigmoid(x0) * x1   (SiLU(gate) * up)               */
} lpg_ew_op;

/* Operations fused into the GEMM epilogue, applied to v = alpha*acc + beta*C_in. */
typedef enum {
    LPG_EPI_NONE = 0,      /* out = v                                                    */
    LPG_EPI_SILU = 1,      /* out = v * sigmoid(v)                                       */
    LPG_EPI_GATE_SILU = 2  /* out = g * sigmoid(g) * v, g = epi_arg at the same position
                              (epi_arg: device buffer laid out and typed exactly as C_out) */
} lpg_epilogue_op;

/* Bytes of the allocation a descriptor addresses (all slots, padding included
 * for packed kinds).  Returns 0 if the descriptor is invalid. */
size_t lpg_packed_bytes(const lpg_desc *d);

/* Host-side index function of the layout: element offset (in elements, from the
 * buffer start) of logical element (row, col) of matrix b.  Works for canonical
 * and packed kinds.  Returns LPG_OK or LPG_EINVAL. */
int lpg_layout_offset(const lpg_desc *d, int64_t b, int64_t row, int64_t col, int64_t *offset);

/*
 * lpg_pack - canonical -> packed, once at the chain's entry (the packing step of
 * the GotoBLAS loop nest, Fig. 2c, done for the whole matrix; paper II-A).
 * src_d: ROW_MAJOR or COL_MAJOR; dst_d: PACKED_A or PACKED_B, same rows/cols/batch.
 * Writes every block the matrix touches, zero-filling padding; a destination that is
 * a view inside a larger parent is written as lpg_desc describes (its own elements
 * only where a block is shared with the parent's other elements).  dtype pairs:
 * f32->f32, bf16->bf16 (bit-exact copies), f32->bf16 (round to nearest even).
 */
int lpg_pack(const void *src, const lpg_desc *src_d, void *dst, const lpg_desc *dst_d,
             void *stream);

/*
 * lpg_unpack - packed -> canonical, once at the chain's exit (the reordering the
 * paper's Default micro-kernel performs, III-B).  Padding is dropped.  dtype
 * pairs: f32->f32, bf16->bf16 (bit-exact), bf16->f32 (exact widening).
 */
int lpg_unpack(const void *src, const lpg_desc *src_d, void *dst, const lpg_desc *dst_d,
               void *stream);

/*
 * lpg_gemm_packed - the Intermediate kernel (III-A.2) with the Propagate-Layout
 * micro-kernel (III-B):  C_out = epilogue(alpha * A * B + beta * C_in), all
 * operands packed, C written directly as operand fragments of the next GEMM.
 *   a_d.kind == LPG_PACKED_A, b_d.kind == LPG_PACKED_B, a_d.cols == b_d.rows.
 *   c_d.kind == LPG_PACKED_A (C will be a left operand) or LPG_PACKED_B (right).
 *   dtypes: (f32, f32 -> f32), (bf16, bf16 -> bf16 or f32); accumulation is fp32.
 *   C_in: laid out and typed as c_d; may be NULL iff beta == 0, and is never read
 *   when beta == 0 (the packed-C requirement of III-B, which this library
 *   supports).  C_in == C_out (in place) is allowed; C_out must not alias A or B.
 *   Batches: c_d.batch matrices; A, B use slot b / batch_div of their descriptors.
 *   Padding of C_out is written as zeros (C as a view inside a parent: see lpg_desc).
 * The same call is also the paper's Initial and Ending kernels (III-A.1, III-A.3):
 *   Initial: a_d and / or b_d may be LPG_ROW_MAJOR or LPG_COL_MAJOR, fp32 or bf16, with any
 *   leading dimension, origin and element alignment, and the contraction extent may be any
 *   length: the kernel builds the MFMA fragments from the canonical matrix itself, no pack
 *   pass.  The product multiplies in the dtype of the packed operand; with two canonical
 *   operands in bf16 if either of them or the result is bf16, else in fp32; an fp32 canonical
 *   operand of a bf16 product is rounded to nearest even as it is read, as lpg_pack would
 *   have rounded it.  (A bf16 canonical operand beside an fp32 packed one: LPG_EUNSUPPORTED.)
 *   An fp32 operand that is contiguous along the contraction index, 16-byte aligned and a
 *   multiple of 32 long is copied verbatim by the main kernel (full speed); every other form
 *   is gathered element by element by the general kernel.
 *   Packed inputs may be views with any origin and any extent inside their parent (lpg_desc):
 *   the main kernel takes any free-dimension origin at full speed; a contraction-dimension
 *   origin off the KB grid, or a contraction extent that ends inside the parent, goes through
 *   the general kernel.
 *   Ending: c_d may be LPG_ROW_MAJOR or LPG_COL_MAJOR (any dtype pair above, any
 *   ld): C_out, and C_in / epi_arg if used, are then canonical, elements outside the
 *   logical extent are left untouched, and no unpack pass is needed.
 * Both give bit-identical values to lpg_pack / lpg_unpack around the packed call.
 */
int lpg_gemm_packed(float alpha, const void *A, const lpg_desc *a_d, const void *B,
                    const lpg_desc *b_d, float beta, const void *C_in, void *C_out,
                    const lpg_desc *c_d, int epilogue_op, const void *epi_arg, void *stream);

/*
 * lpg_elementwise_packed - layout-oblivious elementwise op over whole packed (or
 * canonical, tightly stored) buffers sharing one descriptor `d` (no sub-views).
 * Every supported op maps zero padding to zero.  Math in fp32; bf16 results are
 * rounded to nearest even.  x1 may be NULL for LPG_EW_SCALE.  In place is allowed.
 */
int lpg_elementwise_packed(int op, const void *x0, const void *x1, float s, void *out,
                           const lpg_desc *d, void *stream);

/*
 * lpg_softmax_packed - the steps between the two attention GEMMs (Alg. 2: scale,
 * optional mask, softmax), done on the packed layout so that the scores never leave
 * it (section IV-A: operations that are not layout-oblivious are re-written for the
 * propagated layout instead of unpacking around them):
 *     out[i][j] = exp(scale*x[i][j] - m_i) / sum_j' exp(scale*x[i][j'] - m_i),
 * m_i = max_j scale*x[i][j], over the logical columns of every row of every slot.
 * causal != 0 keeps only columns j <= i + (cols - rows) of row i; masked positions,
 * and rows with no kept column, get 0.  scale must be positive and finite (LPG_EINVAL).
 *   d->kind == LPG_PACKED_A (the row index is the free index, the softmax runs along
 *   the contraction index of the GEMM that will consume the result as its left
 *   operand; views as in lpg_desc, batch_div must be 1) or LPG_ROW_MAJOR (any ld /
 *   view; what the canonical control chain calls).  Other kinds: LPG_EUNSUPPORTED.
 *   x and out share the descriptor; in place (out == x) is allowed, partial overlap
 *   is not.  Math in fp32; bf16 results are rounded to nearest even.  Packed kinds:
 *   every block the view touches is written, padding as zeros.
 */
int lpg_softmax_packed(const void *x, void *out, const lpg_desc *d, float scale, int causal,
                       void *stream);

/*
 * lpg_rmsnorm_packed - RMS normalisation on the packed layout (the RMSNorm the paper lists
 * among the operations re-implemented for the propagated layout; it gives no formula, so
 * the usual one is taken):  out[i][j] = x[i][j] / sqrt(mean_j x[i][j]^2 + eps) * weight[j].
 *   d, x, out: as for lpg_softmax_packed (LPG_PACKED_A or LPG_ROW_MAJOR, shared descriptor,
 *   in place allowed).  weight: device, d->cols fp32 values.  eps >= 0.
 */
int lpg_rmsnorm_packed(const void *x, const float *weight, void *out, const lpg_desc *d, float eps,
                       void *stream);

/*
 * lpg_rope_tables - cosine / sine tables for lpg_rope_packed: device fp32, row-major
 * [rows][head_dim/2], cos_t[t][i] = cos((pos0 + t) * base^(-2i/head_dim)), sin_t likewise.
 * Angles, cosines and sines are computed in fp64 and rounded once.
 */
int lpg_rope_tables(float *cos_t, float *sin_t, int64_t rows, int32_t head_dim, double base,
                    int64_t pos0, void *stream);

/*
 * lpg_rope_packed - rotary position embedding of Q or K on the packed layout (Alg. 2, the
 * step before the score GEMM; section IV-A: rows rotate independently, which is how the
 * layout interleaves them, so 32 positions are rotated per wave access).  d->cols must be
 * heads * head_dim; in every head, element i of the first half pairs with element i of the
 * second half (the paper fixes no pairing; this is the one Llama checkpoints are stored
 * for), and row t's pair (a, b) becomes (a*cos - b*sin, b*cos + a*sin) with cos_t[t][i],
 * sin_t[t][i] (device fp32 tables with at least d->rows rows, 16-byte aligned; every slot
 * of a batch uses the same tables).
 *   d, x, out: as for lpg_softmax_packed.  Packed kinds need head_dim to be a multiple of
 *   16 (fp32) or 32 (bf16), so that a head's halves are whole fragments apart
 *   (LPG_EUNSUPPORTED otherwise).  Math in fp32; bf16 results rounded to nearest even.
 */
int lpg_rope_packed(const void *x, void *out, const lpg_desc *d, const float *cos_t,
                    const float *sin_t, int32_t head_dim, void *stream);

/*
 * lpg_attention_packed - the attention block of Alg. 2 (score GEMM, scale, optional causal
 * mask, softmax, weighted sum) as one kernel in which the scores stay in registers:
 *     O = softmax(scale * Q K^T [causal]) V        per matrix of the batch (head).
 * The paper keeps the scores as a matrix in the propagated layout between two GEMMs; on this
 * hardware the accumulator tile the score MFMA leaves is already the operand fragment the
 * second MFMA consumes, so the propagated intermediate need not be stored at all.  Same
 * values as lpg_gemm_packed + lpg_softmax_packed + lpg_gemm_packed up to rounding (the
 * probabilities are not rounded to the storage type before the row sum).
 *   q_d, o_d: LPG_PACKED_A, queries x head_dim (views of the projections' outputs are fine).
 *   k_d: the keys as a left-operand image, LPG_PACKED_A keys x head_dim, or the same bytes
 *        described as LPG_PACKED_B head_dim x keys (K^T as a right operand).
 *   v_d: LPG_PACKED_B keys x head_dim (or LPG_PACKED_A head_dim x keys).
 *   One dtype for all four (f32 or bf16; fp32 accumulation and softmax); head_dim 64 or 128;
 *   batch counts equal; batch_div on k_d / v_d shares a key/value head among query heads.
 *   flags: LPG_ATTN_CAUSAL - query i sees keys j <= i + (keys - queries);
 *          LPG_ATTN_NO_SOFTMAX - O = (scale * Q K^T [causal]) V, the two chained GEMMs of the
 *          GEMM-only attention workloads with the intermediate kept in registers (bf16: it is
 *          rounded to bf16 where the first GEMM would have stored it; any finite scale).
 *   With the softmax scale must be positive.  O must not alias an input.  Padding rows of O
 *   are written as zeros.
 */
typedef enum { LPG_ATTN_CAUSAL = 1, LPG_ATTN_NO_SOFTMAX = 2 } lpg_attention_flags;
int lpg_attention_packed(const void *Q, const lpg_desc *q_d, const void *K, const lpg_desc *k_d,
                         const void *V, const lpg_desc *v_d, void *O, const lpg_desc *o_d,
                         float scale, int flags, void *stream);

/* One stage of a chain. */
typedef enum {
    LPG_STAGE_PACK = 0,
    LPG_STAGE_GEMM = 1,
    LPG_STAGE_ELEMENTWISE = 2,
    LPG_STAGE_UNPACK = 3,
    LPG_STAGE_SOFTMAX = 4,
    LPG_STAGE_RMSNORM = 5,
    LPG_STAGE_ROPE = 6,
    LPG_STAGE_ATTENTION = 7
} lpg_stage_type;

typedef struct lpg_stage {
    int32_t type;       /* lpg_stage_type                                               */
    int32_t op;         /* GEMM: lpg_epilogue_op; ELEMENTWISE: lpg_ew_op; SOFTMAX: causal;
                           ATTENTION: lpg_attention_flags; ROPE: head_dim                */
    float alpha, beta;  /* GEMM                                                         */
    float scalar;       /* ELEMENTWISE: s; SOFTMAX, ATTENTION: scale; RMSNORM: eps      */
    int32_t reserved;
    const void *in0;    /* PACK/UNPACK: src; GEMM: A; ELEMENTWISE: x0; SOFTMAX, RMSNORM,
                           ROPE: x; ATTENTION: Q                                         */
    const void *in1;    /* GEMM: B; ELEMENTWISE: x1; RMSNORM: weight; ROPE: cos table;
                           ATTENTION: K                                                  */
    const void *in2;    /* GEMM: C_in (or NULL); ROPE: sin table; ATTENTION: V          */
    const void *epi_arg;/* GEMM: epilogue argument (or NULL)                            */
    void *out;
    lpg_desc in0_d;     /* descriptor of in0                                            */
    lpg_desc in1_d;     /* GEMM: descriptor of B                                        */
    lpg_desc out_d;     /* descriptor of out (and of in2, epi_arg, and of the x inputs of
                           ELEMENTWISE / SOFTMAX / RMSNORM / ROPE)                       */
    lpg_desc in2_d;     /* ATTENTION: descriptor of V                                   */
} lpg_stage;

typedef enum {
    LPG_CHAIN_PROPAGATED = 0, /* intermediates stay packed (LP-GEMM, Fig. 1b)           */
    LPG_CHAIN_CANONICAL = 1   /* control: every intermediate is unpacked to row-major
                                 by its producer and re-packed for its consumer, as a
                                 BLAS-API chain does (Fig. 1a); same kernels, same result */
} lpg_chain_mode;

/* Workspace bytes lpg_chain needs (0 in propagated mode).  SIZE_MAX on error. */
size_t lpg_chain_workspace_bytes(const lpg_stage *stages, int n, int mode);

/*
 * lpg_chain - enqueue a whole chain (Eq. 2) on one stream.  Checks that each
 * packed input that an earlier stage produced is read with the packed geometry
 * it was written in (LPG_ELAYOUT otherwise), then launches the stages in order.
 * In LPG_CHAIN_CANONICAL mode `workspace` (device, 256-byte aligned, at least
 * lpg_chain_workspace_bytes) holds the row-major copies of the intermediates.
 */
int lpg_chain(const lpg_stage *stages, int n, int mode, void *workspace,
              size_t workspace_bytes, void *stream);

/*
 * lpg_chain_static - lpg_chain for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same stages, same modes, same kernels and same results as lpg_chain; the
 * row-major copies of LPG_CHAIN_CANONICAL live in a static device array of the library
 * (LPG_STATIC_SCRATCH_BYTES, one copy per GPU the library runs on, held until the process
 * ends) instead of a caller's workspace.  The call allocates nothing and frees nothing.
 *   A chain whose lpg_chain_workspace_bytes exceeds LPG_STATIC_SCRATCH_BYTES is refused with
 *   LPG_EWORKSPACE before anything is launched.  LPG_CHAIN_PROPAGATED needs no scratch at all.
 *   The device that is current at the call must be the stream's device; the address of that
 *   device's copy of the array is looked up on the first call per device (the one call that
 *   should not be made while a capture is in progress) and kept.
 *   All calls on one GPU share that GPU's array, and nothing in it needs to start at zero
 *   (every byte a stage reads there was written by an earlier stage of the same call), so
 *   calls on one stream may follow each other freely, but calls that overlap in time on one
 *   GPU (different streams, or graphs replayed concurrently) race on it.
 */
#define LPG_STATIC_SCRATCH_BYTES (64u << 20)
int lpg_chain_static(const lpg_stage *stages, int n, int mode, void *stream);

/*
 * Tuning and test hooks.  Every choice the library makes per launch (tile configuration, band
 * height of the tile walk, staging-ring variants, row-kernel variant) can be pinned for
 * measurements and for tests that must reach every variant; -1 (LPG_TUNE_AUTO) gives the choice
 * back to the library.  Process-wide, read at every launch, not meant for production use.
 * Table I of the paper lists such parameters per architecture; these are this library's.
 */
typedef enum {
    LPG_TUNE_TILE = 0,                    /* GEMM tile configuration index 0..7                      */
    LPG_TUNE_BAND = 1,                    /* tile rows per band of the XCD-local tile walk          */
    LPG_TUNE_TWO_BLOCK_STEPS = 2,         /* 0: lone small tiles take one K block per step          */
    LPG_TUNE_BF16_WHOLE_BLOCK_STEPS = 3,  /* 0: bf16 4-wave tiles use the half-block ring           */
    LPG_TUNE_ROW_VARIANT = 4,             /* softmax / RMSNorm kernel variant 0..5                  */
    LPG_TUNE_ATTN_QUERY_GROUPS = 5,       /* fused attention: 1 or 2 query groups per wave          */
    LPG_TUNE_TRACE = 6,                   /* 1: print the tile configuration of every GEMM launch   */
    LPG_TUNE_STREAM_STORES = 7,           /* 0 / 1: GEMM epilogue stores plain / streaming (non-temporal)   */
    LPG_TUNE_KEYS = 8
} lpg_tune_key;
#define LPG_TUNE_AUTO (-1)
int lpg_tune_set(int key, int value);
int lpg_tune_get(int key, int *value);

/* Message for the last error on this thread ("" if none). */
const char *lpg_last_error(void);

/* Library version string. */
const char *lpg_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LPG_H */
