// Host side of the C ABI: descriptor validation, view arithmetic, kernel argument
// marshalling, and the chain executor (propagated and canonical-control modes).
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "lpg_internal.h"

namespace lpg {

static thread_local char g_err[512] = "";

static int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

static inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }
static inline bool is_packed(int kind) { return kind == LPG_PACKED_A || kind == LPG_PACKED_B; }
static inline bool is_canon(int kind) { return kind == LPG_ROW_MAJOR || kind == LPG_COL_MAJOR; }

static int check_common(const lpg_desc *d, const char *what)
{
    if (!d) return fail(LPG_EINVAL, "%s: descriptor is NULL", what);
    if (d->kind < LPG_ROW_MAJOR || d->kind > LPG_PACKED_B) return fail(LPG_EINVAL, "%s: bad kind %d", what, d->kind);
    if (d->dtype != LPG_F32 && d->dtype != LPG_BF16) return fail(LPG_EUNSUPPORTED, "%s: bad dtype %d", what, d->dtype);
    if (d->rows < 0 || d->cols < 0) return fail(LPG_EINVAL, "%s: negative extent", what);
    if (d->rows > 0x7fffffff || d->cols > 0x7fffffff) return fail(LPG_EINVAL, "%s: extent over 2^31-1", what);
    if (d->batch < 0 || d->batch_div < 0) return fail(LPG_EINVAL, "%s: negative batch", what);
    if (d->row0 < 0 || d->col0 < 0 || d->batch_stride < 0 || d->batch_row_step < 0 || d->batch_col_step < 0 ||
        d->group_stride < 0 || d->kblock_stride < 0)
        return fail(LPG_EINVAL, "%s: negative origin, step or stride", what);
    if ((d->parent_rows == 0) != (d->parent_cols == 0))
        return fail(LPG_EINVAL, "%s: parent_rows and parent_cols must both be set or both be 0", what);
    return LPG_OK;
}

static inline int nbatch(const lpg_desc *d) { return d->batch > 0 ? d->batch : 1; }
static inline int bdiv(const lpg_desc *d) { return d->batch_div > 0 ? d->batch_div : 1; }
static inline int nslots(const lpg_desc *d) { return (nbatch(d) + bdiv(d) - 1) / bdiv(d); }

// Reduce a packed descriptor to a PView and validate its geometry.  A ragged extent (not a
// multiple of 32 along the free index, of KB along the contraction index) normally has to end
// at the parent's edge, where its padding is the parent's own.  `inner` names the dimensions
// in which the caller can also take a ragged extent that ends inside the parent: the view's
// last block is then shared with neighbouring elements of the parent, keep_f / keep_k are set,
// and a writer must leave those neighbours alone.  kOffGrid: the caller also takes an origin
// that is not a multiple of 32 / KB (f_off / k_off are then non-zero, the origin points at the
// block that holds the first element, and nothing outside the view may be written).  kRaggedSteps:
// the caller only reads, so the views of a stepped batch may have ragged extents (a writer's ragged
// view would spill its padding into the next slot's elements).
enum { kInnerF = 1, kInnerK = 2, kOffGrid = 4, kRaggedSteps = 8 };
static int make_pview(const lpg_desc *d, const char *what, PView *v, unsigned inner = 0)
{
    int rc = check_common(d, what);
    if (rc) return rc;
    if (!is_packed(d->kind)) return fail(LPG_ELAYOUT, "%s: expected a packed kind, got %d", what, d->kind);
    const bool tr = d->kind == LPG_PACKED_B;
    v->dtype = d->dtype;
    v->es = elem_size(d->dtype);
    const int64_t KB = kb_of(d->dtype);
    const int64_t prow = d->parent_rows ? d->parent_rows : d->rows;
    const int64_t pcol = d->parent_cols ? d->parent_cols : d->cols;
    v->transposed = tr;
    v->F = tr ? d->cols : d->rows;
    v->K = tr ? d->rows : d->cols;
    v->PF = tr ? pcol : prow;
    v->PK = tr ? prow : pcol;
    v->f0 = tr ? d->col0 : d->row0;
    v->k0 = tr ? d->row0 : d->col0;
    v->fstep = tr ? d->batch_col_step : d->batch_row_step;
    v->kstep = tr ? d->batch_row_step : d->batch_col_step;
    v->batch = nbatch(d);
    v->bdiv = bdiv(d);
    v->bstride = d->batch_stride;
    v->PFp = round_up(v->PF, 32);
    v->PKp = round_up(v->PK, KB);
    const int ns = nslots(d);
    v->f_off = (int)(v->f0 % 32);
    v->k_off = (int)(v->k0 % KB);
    const bool off_grid = v->f_off || v->k_off;
    if ((v->f_off && !(inner & kOffGrid)) || v->fstep % 32)
        return fail(LPG_EALIGN, "%s: free-dimension origin/step must be a multiple of 32", what);
    if ((v->k_off && !(inner & kOffGrid)) || v->kstep % KB)
        return fail(LPG_EALIGN, "%s: contraction-dimension origin/step must be a multiple of %d", what, (int)KB);
    const int64_t f_last = v->f0 + (ns - 1) * v->fstep, k_last = v->k0 + (ns - 1) * v->kstep;
    if (f_last + v->F > v->PF || k_last + v->K > v->PK)
        return fail(LPG_EINVAL, "%s: view exceeds its parent", what);
    // a ragged extent may only sit at the parent's edge, where its padding is the parent's
    if (!(inner & kRaggedSteps) && v->F % 32 && (ns > 1 ? v->fstep != 0 : false))
        return fail(LPG_EALIGN, "%s: stepped views need a free extent that is a multiple of 32", what);
    if (!(inner & kRaggedSteps) && v->K % KB && (ns > 1 ? v->kstep != 0 : false))
        return fail(LPG_EALIGN, "%s: stepped views need a contraction extent that is a multiple of %d", what, (int)KB);
    v->keep_f = !off_grid && v->F % 32 && v->f0 + v->F != v->PF;
    v->keep_k = !off_grid && v->K % KB && v->k0 + v->K != v->PK;
    if (v->keep_f && !(inner & kInnerF))
        return fail(LPG_EALIGN, "%s: a free extent that is not a multiple of 32 must end at the parent's edge", what);
    if (v->keep_k && !(inner & kInnerK))
        return fail(LPG_EALIGN, "%s: a contraction extent that is not a multiple of %d must end at the parent's edge", what, (int)KB);
    if ((v->bstride * v->es) % 16)
        return fail(LPG_EALIGN, "%s: batch_stride must keep 16-byte alignment", what);
    // block order / store stride: bytes from group to group and from K block to K block
    const int64_t blk = 32 * KB;  // elements of one block
    if (d->group_stride % blk || d->kblock_stride % blk)
        return fail(LPG_EINVAL, "%s: group_stride and kblock_stride must be multiples of one block (%lld elements)", what, (long long)blk);
    const int64_t ng = v->PFp / 32, nk = v->PKp / KB;
    int64_t gs = d->group_stride, ks = d->kblock_stride;
    if (!gs && !ks) { gs = blk; ks = ng * blk; }
    else if (!gs) gs = blk;                 // kblock_stride alone: K blocks spread out, groups back to back
    else if (!ks) ks = blk;                 // group_stride alone: groups outermost, K blocks back to back
    const bool k_outer = ks >= ng * gs, f_outer = gs >= nk * ks;
    if (!k_outer && !f_outer && ng > 1 && nk > 1)
        return fail(LPG_EINVAL, "%s: group_stride %lld and kblock_stride %lld make blocks overlap", what, (long long)gs, (long long)ks);
    v->default_order = gs == blk && ks == ng * blk;
    v->g_stride = gs * v->es;
    v->kb_stride = ks * v->es;
    v->origin = (v->k0 / KB) * v->kb_stride + (v->f0 / 32) * v->g_stride;
    v->slot_step = v->bstride * v->es + (v->kstep / KB) * v->kb_stride + (v->fstep / 32) * v->g_stride;
    if (ns > 1 && v->bstride != 0 && v->bstride * v->es < (ng - 1) * v->g_stride + (nk - 1) * v->kb_stride + kBlockBytes)
        return fail(LPG_EINVAL, "%s: batch_stride smaller than one packed parent", what);
    return LPG_OK;
}

static int make_cview(const lpg_desc *d, const char *what, CView *v)
{
    int rc = check_common(d, what);
    if (rc) return rc;
    if (!is_canon(d->kind)) return fail(LPG_ELAYOUT, "%s: expected ROW_MAJOR or COL_MAJOR, got kind %d", what, d->kind);
    const int64_t prow = d->parent_rows ? d->parent_rows : d->rows;
    const int64_t pcol = d->parent_cols ? d->parent_cols : d->cols;
    const bool rm = d->kind == LPG_ROW_MAJOR;
    const int64_t tight = rm ? pcol : prow;
    const int64_t ld = d->ld ? d->ld : tight;
    if (ld < tight) return fail(LPG_EINVAL, "%s: ld %lld smaller than the parent's extent %lld", what, (long long)ld, (long long)tight);
    v->dtype = d->dtype;
    v->es = elem_size(d->dtype);
    v->rows = d->rows;
    v->cols = d->cols;
    v->row_stride = rm ? ld : 1;
    v->col_stride = rm ? 1 : ld;
    v->batch = nbatch(d);
    v->bdiv = bdiv(d);
    const int ns = nslots(d);
    if (d->row0 + (ns - 1) * d->batch_row_step + d->rows > prow ||
        d->col0 + (ns - 1) * d->batch_col_step + d->cols > pcol)
        return fail(LPG_EINVAL, "%s: view exceeds its parent", what);
    v->origin = d->row0 * v->row_stride + d->col0 * v->col_stride;
    v->slot_step = d->batch_stride + d->batch_row_step * v->row_stride + d->batch_col_step * v->col_stride;
    return LPG_OK;
}

static size_t desc_bytes(const lpg_desc *d)
{
    if (check_common(d, "desc")) return 0;
    const int ns = nslots(d);
    const int es = elem_size(d->dtype);
    const int64_t prow = d->parent_rows ? d->parent_rows : d->rows;
    const int64_t pcol = d->parent_cols ? d->parent_cols : d->cols;
    int64_t one;
    if (is_packed(d->kind)) {
        PView pv;
        if (make_pview(d, "desc", &pv, kInnerF | kInnerK | kOffGrid)) return 0;
        const bool tr = d->kind == LPG_PACKED_B;
        const int64_t PF = tr ? pcol : prow, PK = tr ? prow : pcol;
        const int64_t KB = kb_of(d->dtype), blk = 32 * KB;
        const int64_t ng = round_up(PF, 32) / 32, nk = round_up(PK, KB) / KB;
        int64_t gs = d->group_stride, ks = d->kblock_stride;
        if (!gs && !ks) { gs = blk; ks = ng * blk; }
        else if (!gs) gs = blk;
        else if (!ks) ks = blk;
        one = (ng && nk) ? (ng - 1) * gs + (nk - 1) * ks + blk : 0;
    } else {
        const bool rm = d->kind == LPG_ROW_MAJOR;
        const int64_t tight = rm ? pcol : prow;
        const int64_t ld = d->ld ? d->ld : tight;
        one = ld * (rm ? prow : pcol);
    }
    const int64_t total = (d->batch_stride ? (int64_t)(ns - 1) * d->batch_stride : 0) + one;
    return (size_t)total * es;
}

static int check_ptr16(const void *p, const char *what)
{
    if (!p) return fail(LPG_EINVAL, "%s: NULL pointer", what);
    if ((uintptr_t)p % 16) return fail(LPG_EALIGN, "%s: packed buffers must be 16-byte aligned", what);
    return LPG_OK;
}

// ------------------------------------------------------------------------ pack / unpack

static int do_pack_unpack(bool pack, const void *canon, const lpg_desc *cd, const void *packed,
                          const lpg_desc *pd, hipStream_t st)
{
    const char *name = pack ? "lpg_pack" : "lpg_unpack";
    PView pv;
    CView cv;
    int rc = make_pview(pd, pack ? "lpg_pack dst" : "lpg_unpack src", &pv, kInnerF | kInnerK | kOffGrid);
    if (rc) return rc;
    rc = make_cview(cd, pack ? "lpg_pack src" : "lpg_unpack dst", &cv);
    if (rc) return rc;
    if (cd->rows != pd->rows || cd->cols != pd->cols)
        return fail(LPG_EINVAL, "%s: source and destination extents differ", name);
    if (nbatch(cd) != nbatch(pd)) return fail(LPG_EINVAL, "%s: batch counts differ", name);
    const bool conv_ok = pack ? (cv.dtype == pv.dtype || (cv.dtype == LPG_F32 && pv.dtype == LPG_BF16))
                              : (cv.dtype == pv.dtype || (pv.dtype == LPG_BF16 && cv.dtype == LPG_F32));
    if (!conv_ok) return fail(LPG_EUNSUPPORTED, "%s: dtype conversion not supported", name);
    if (!canon) return fail(LPG_EINVAL, "%s: NULL canonical pointer", name);
    rc = check_ptr16(packed, name);
    if (rc) return rc;
    if ((uintptr_t)canon % cv.es) return fail(LPG_EALIGN, "%s: canonical pointer not element aligned", name);
    if (pv.F == 0 || pv.K == 0) return LPG_OK;

    PackArgs a;
    a.canon = (const char *)canon + cv.origin * cv.es;
    a.packed = (char *)packed + pv.origin;
    a.sf = pv.transposed ? cv.col_stride : cv.row_stride;
    a.sk = pv.transposed ? cv.row_stride : cv.col_stride;
    a.c_slot = cv.slot_step * cv.es;
    a.p_kbs = pv.kb_stride;
    a.p_gs = pv.g_stride;
    a.p_slot = pv.slot_step;
    a.c_div = cv.bdiv;
    a.p_div = pv.bdiv;
    a.F = (int32_t)pv.F;
    a.K = (int32_t)pv.K;
    // blocks the view touches, counted from the block that holds its origin
    a.ngroups = (int32_t)((pv.f_off + pv.F + 31) / 32);
    a.nkb = (int32_t)((pv.k_off + pv.K + kb_of(pv.dtype) - 1) / kb_of(pv.dtype));
    a.batch = pv.batch;
    a.kpw = 1;
    a.keep_f = pv.keep_f;
    a.keep_k = pv.keep_k;
    a.f_off = pv.f_off;
    a.k_off = pv.k_off;
    if (a.nkb > 65535 || a.batch > 65535) return fail(LPG_EUNSUPPORTED, "%s: more than 65535 K blocks or batches", name);
    hipError_t e = pack ? launch_pack(a, cv.dtype, pv.dtype, st) : launch_unpack(a, pv.dtype, cv.dtype, st);
    if (e != hipSuccess) return fail(LPG_EHIP, "%s: %s", name, hipGetErrorString(e));
    return LPG_OK;
}

// ------------------------------------------------------------------------------- GEMM

// An input of the product in (free, contraction) terms, packed or canonical.
struct Operand {
    bool canon;                 // canonical (row- or column-major) rather than packed
    bool copyable_f32;          // canonical: fp32, contiguous along k, K a multiple of 32, 16-byte aligned rows
    bool copyable_packed;       // packed: origin on the K-block grid, contraction extent whole or ending at the parent's edge
    int dtype;                  // of the stored elements
    int64_t F, K;
    int batch, bdiv;
    int64_t origin, slot_step;  // bytes
    int64_t kb_stride;          // packed: bytes between K blocks
    int64_t ld_bytes;           // canonical: bytes between consecutive free indices
    int64_t g_stride;           // packed: bytes between 32-groups
    int f_off;                  // packed: rows between the view's origin and the 32-grid
    GatherOperand go;           // the same operand for the general (gathering) kernel
};

// is_a: the left operand (free = rows; PACKED_A or canonical); else the right operand (free =
// cols; PACKED_B or canonical).  What the main kernel can copy verbatim is marked copyable;
// every other operand is read by the general kernel (the Initial kernel for any layout).
static int make_operand(const lpg_desc *d, const void *ptr, bool is_a, Operand *o)
{
    const char *what = is_a ? "lpg_gemm_packed A" : "lpg_gemm_packed B";
    int rc = check_common(d, what);
    if (rc) return rc;
    if (!ptr) return fail(LPG_EINVAL, "%s: NULL pointer", what);
    *o = Operand{};
    if (is_packed(d->kind)) {
        if ((uintptr_t)ptr % 16) return fail(LPG_EALIGN, "%s: packed buffers must be 16-byte aligned", what);
        if (d->kind != (is_a ? LPG_PACKED_A : LPG_PACKED_B))
            return fail(LPG_ELAYOUT, "%s: must be %s", what, is_a ? "LPG_PACKED_A" : "LPG_PACKED_B");
        PView v;
        rc = make_pview(d, what, &v, kInnerF | kInnerK | kOffGrid | kRaggedSteps);
        if (rc) return rc;
        // a contraction extent that ends inside the parent's last touched block would add the
        // neighbours to every sum if that block were copied whole
        const bool k_tail_inside = v.K % kb_of(v.dtype) && v.k0 + v.K != v.PK;
        o->canon = false;
        o->copyable_packed = v.k_off == 0 && !k_tail_inside;
        o->dtype = v.dtype;
        o->F = v.F; o->K = v.K; o->batch = v.batch; o->bdiv = v.bdiv;
        o->origin = v.origin; o->slot_step = v.slot_step; o->kb_stride = v.kb_stride; o->g_stride = v.g_stride;
        o->f_off = v.f_off;
        o->go = GatherOperand{(const char *)ptr + v.origin, v.batch == 1 ? 0 : v.slot_step, 0, 0, v.kb_stride, v.g_stride,
                              v.bdiv, 1, 3 /* element by element through the packed position */, v.es, v.f_off, v.k_off,
                              (int32_t)v.F, (int32_t)v.K};
        return LPG_OK;
    }
    CView v;
    rc = make_cview(d, what, &v);
    if (rc) return rc;
    if ((uintptr_t)ptr % v.es) return fail(LPG_EALIGN, "%s: buffer not element aligned", what);
    const int64_t K = is_a ? d->cols : d->rows, F = is_a ? d->rows : d->cols;
    const int64_t sf = is_a ? v.row_stride : v.col_stride, sk = is_a ? v.col_stride : v.row_stride;  // elements
    o->canon = true;
    o->copyable_f32 = v.dtype == LPG_F32 && sk == 1 && K % 32 == 0 && (uintptr_t)ptr % 16 == 0 && (sf * 4) % 16 == 0 &&
                      (v.origin * 4) % 16 == 0 && (v.slot_step * 4) % 16 == 0;
    o->dtype = v.dtype;
    o->F = F; o->K = K; o->batch = v.batch; o->bdiv = v.bdiv;
    o->origin = v.origin * v.es; o->slot_step = v.slot_step * v.es; o->ld_bytes = sf * v.es;
    // vector loads where rows are contiguous along k, start on 16-byte (fp32) / 8-byte (bf16) boundaries and the
    // contraction extent is a multiple of 4 (a run of four k is then inside or outside as a whole)
    const int64_t vec = v.es == 4 ? 16 : 8;
    const bool vec_ok = sk == 1 && K % 4 == 0 && ((uintptr_t)ptr + v.origin * v.es) % vec == 0 && (sf * v.es) % vec == 0 &&
                        (v.slot_step * v.es) % vec == 0;
    const int mode = vec_ok ? (v.es == 4 ? 1 : 2) : 0;
    o->go = GatherOperand{(const char *)ptr + v.origin * v.es, v.batch == 1 ? 0 : v.slot_step * v.es, sf * v.es, sk * v.es, 0, 0,
                          v.bdiv, 0, mode, v.es, 0, 0, (int32_t)F, (int32_t)K};
    return LPG_OK;
}

static int do_gemm(float alpha, const void *A, const lpg_desc *a_d, const void *B, const lpg_desc *b_d,
                   float beta, const void *C_in, void *C_out, const lpg_desc *c_d, int epi,
                   const void *epi_arg, hipStream_t st, bool launch)
{
    Operand ao, bo;
    int rc = make_operand(a_d, A, true, &ao);
    if (rc) return rc;
    rc = make_operand(b_d, B, false, &bo);
    if (rc) return rc;
    rc = check_common(c_d, "lpg_gemm_packed C");
    if (rc) return rc;
    const bool c_canon = is_canon(c_d->kind);
    PView cv{};
    CView ccv{};
    rc = c_canon ? make_cview(c_d, "lpg_gemm_packed C", &ccv) : make_pview(c_d, "lpg_gemm_packed C", &cv, kInnerF | kInnerK | kOffGrid);
    if (rc) return rc;
    const int c_dtype = c_d->dtype, c_batch = nbatch(c_d);
    if (ao.K != bo.K)
        return fail(LPG_EINVAL, "lpg_gemm_packed: inner dimensions differ (A cols %lld, B rows %lld)",
                    (long long)a_d->cols, (long long)b_d->rows);
    if (c_d->rows != a_d->rows || c_d->cols != b_d->cols)
        return fail(LPG_EINVAL, "lpg_gemm_packed: C is %lldx%lld but A*B is %lldx%lld", (long long)c_d->rows,
                    (long long)c_d->cols, (long long)a_d->rows, (long long)b_d->cols);
    // The type the MFMAs multiply: that of the packed operands; an fp32 canonical operand beside a
    // bf16 one is rounded to bf16 as it is read (as lpg_pack would have done).
    int in_dtype;
    if (!ao.canon && !bo.canon) {
        if (ao.dtype != bo.dtype) return fail(LPG_EUNSUPPORTED, "lpg_gemm_packed: A and B dtypes differ");
        in_dtype = ao.dtype;
    } else if (ao.canon && bo.canon) {
        // two canonical operands: bf16 if either is, or if the result is to be stored as bf16
        in_dtype = (ao.dtype == LPG_BF16 || bo.dtype == LPG_BF16 || c_dtype == LPG_BF16) ? LPG_BF16 : LPG_F32;
    } else {
        in_dtype = ao.canon ? bo.dtype : ao.dtype;
        if (in_dtype == LPG_F32 && (ao.canon ? ao.dtype : bo.dtype) != LPG_F32)
            return fail(LPG_EUNSUPPORTED, "lpg_gemm_packed: a bf16 canonical operand beside an fp32 packed one");
    }
    if (in_dtype == LPG_F32 && c_dtype != LPG_F32)
        return fail(LPG_EUNSUPPORTED, "lpg_gemm_packed: f32 inputs need an f32 output");
    auto copyable = [&](const Operand &o) { return o.canon ? (o.copyable_f32 && in_dtype == LPG_F32) : o.copyable_packed; };
    const bool general = !(copyable(ao) && copyable(bo));
    if (epi < LPG_EPI_NONE || epi > LPG_EPI_GATE_SILU) return fail(LPG_EINVAL, "lpg_gemm_packed: bad epilogue op %d", epi);
    if (epi == LPG_EPI_GATE_SILU && !epi_arg) return fail(LPG_EINVAL, "lpg_gemm_packed: LPG_EPI_GATE_SILU needs epi_arg");
    if (beta != 0.0f && !C_in) return fail(LPG_EINVAL, "lpg_gemm_packed: beta != 0 needs C_in");
    if (bdiv(c_d) != 1) return fail(LPG_EINVAL, "lpg_gemm_packed: C batch_div must be 1");
    const int nb = c_batch;
    if ((nb + ao.bdiv - 1) / ao.bdiv > (ao.batch + ao.bdiv - 1) / ao.bdiv && ao.batch != 1)
        return fail(LPG_EINVAL, "lpg_gemm_packed: A has too few batch slots");
    if ((nb + bo.bdiv - 1) / bo.bdiv > (bo.batch + bo.bdiv - 1) / bo.bdiv && bo.batch != 1)
        return fail(LPG_EINVAL, "lpg_gemm_packed: B has too few batch slots");
    if (!C_out) return fail(LPG_EINVAL, "lpg_gemm_packed C_out: NULL pointer");
    const int c_align = c_canon ? elem_size(c_dtype) : 16;
    if ((uintptr_t)C_out % c_align) return fail(LPG_EALIGN, "lpg_gemm_packed: C_out not aligned");
    if (C_in && (uintptr_t)C_in % c_align) return fail(LPG_EALIGN, "lpg_gemm_packed: C_in not aligned");
    if (epi_arg && (uintptr_t)epi_arg % c_align) return fail(LPG_EALIGN, "lpg_gemm_packed: epi_arg not aligned");
    if (C_out == A || C_out == B) return fail(LPG_EINVAL, "lpg_gemm_packed: C_out must not alias A or B");
    if (!launch) return LPG_OK;

    // Which operand rides on lanes decides the role C is written in: lanes become the free
    // dimension of a packed C, and the contiguous dimension of a canonical C.
    const bool l_is_a = c_canon ? c_d->kind == LPG_COL_MAJOR : c_d->kind == LPG_PACKED_A;
    const Operand &L = l_is_a ? ao : bo;
    const Operand &R = l_is_a ? bo : ao;
    GemmArgs g;
    g.o_keep_l = g.o_keep_r = 0;
    g.o_foff = g.o_koff = 0;
    g.o_stream = 0;
    g.L = (const char *)(l_is_a ? A : B) + L.origin;
    g.R = (const char *)(l_is_a ? B : A) + R.origin;
    g.l_canon = L.canon;
    g.r_canon = R.canon;
    g.l_ld = L.ld_bytes;
    g.r_ld = R.ld_bytes;
    g.l_kbs = L.kb_stride;
    g.r_kbs = R.kb_stride;
    g.l_gs = L.g_stride;
    g.r_gs = R.g_stride;
    g.l_foff = L.f_off;
    g.r_foff = R.f_off;
    g.o_gs = kBlockBytes;
    g.l_slot = L.batch == 1 ? 0 : L.slot_step;
    g.r_slot = R.batch == 1 ? 0 : R.slot_step;
    g.l_div = L.bdiv;
    g.r_div = R.bdiv;
    int64_t c_origin;
    if (c_canon) {
        const int es = elem_size(c_dtype);
        c_origin = ccv.origin * es;
        g.o_canon = 1;
        g.o_kbs = 0;
        g.o_slot = ccv.slot_step * es;
        // lanes <-> L's free index: rows of C if L is A, columns if L is B
        g.o_sf = (l_is_a ? ccv.row_stride : ccv.col_stride) * es;
        g.o_sk = (l_is_a ? ccv.col_stride : ccv.row_stride) * es;
        g.FRg_out = (int32_t)((R.F + 31) / 32);
    } else {
        c_origin = cv.origin;
        g.o_canon = 0;
        g.o_kbs = cv.kb_stride;
        g.o_gs = cv.g_stride;
        g.o_slot = cv.slot_step;
        g.o_sf = g.o_sk = 0;
        g.FRg_out = (int32_t)(round_up(R.F, kb_of(c_dtype)) / 32);
        g.o_keep_l = cv.keep_f;
        g.o_keep_r = cv.keep_k;
        if (cv.f_off || cv.k_off) {
            // origin off the grid: element-wise stores at shifted packed positions, nothing
            // outside the view (padding included) is written
            g.o_canon = 2;
            g.o_foff = cv.f_off;
            g.o_koff = cv.k_off;
            g.FRg_out = (int32_t)((R.F + 31) / 32);
        }
    }
    g.Cin = (beta != 0.0f) ? (const char *)C_in + c_origin : nullptr;
    g.Epi = epi_arg ? (const char *)epi_arg + c_origin : nullptr;
    g.Out = (char *)C_out + c_origin;
    g.FL = (int32_t)L.F;
    g.FR = (int32_t)R.F;
    g.FLg = (int32_t)((L.F + 31) / 32);
    g.FRg = (int32_t)((R.F + 31) / 32);
    g.nkb = (int32_t)((ao.K + kb_of(in_dtype) - 1) / kb_of(in_dtype));
    g.walk = TileWalk{};
    g.batch = nb;
    g.epi = epi;
    g.alpha = alpha;
    g.beta = beta;
    if (g.FL == 0 || g.FR == 0) return LPG_OK;
    if (general) {
        GatherArgs ga;
        ga.g = g;
        ga.g.L = ga.g.R = nullptr;
        ga.g.l_canon = ga.g.r_canon = 1;
        ga.l = L.go;
        ga.r = R.go;
        hipError_t e = launch_gemm_gather(ga, in_dtype, c_dtype, st);
        if (e != hipSuccess) return fail(LPG_EHIP, "lpg_gemm_packed: %s", hipGetErrorString(e));
        return LPG_OK;
    }
    // the tuning hook LPG_TUNE_TILE pins the tile configuration (-1 = automatic)
    hipError_t e = launch_gemm(g, in_dtype, c_dtype, tune_get(LPG_TUNE_TILE), st);
    if (e != hipSuccess) return fail(LPG_EHIP, "lpg_gemm_packed: %s", hipGetErrorString(e));
    return LPG_OK;
}

// ------------------------------------------------------------------------ elementwise

static int do_elementwise(int op, const void *x0, const void *x1, float s, void *out, const lpg_desc *d,
                          hipStream_t st, bool launch)
{
    int rc = check_common(d, "lpg_elementwise_packed");
    if (rc) return rc;
    if (op < LPG_EW_SCALE || op > LPG_EW_SILU_MUL) return fail(LPG_EINVAL, "lpg_elementwise_packed: bad op %d", op);
    if (d->row0 || d->col0 || d->batch_row_step || d->batch_col_step ||
        (d->parent_rows && (d->parent_rows != d->rows || d->parent_cols != d->cols)))
        return fail(LPG_EUNSUPPORTED, "lpg_elementwise_packed: sub-views are not supported");
    if (is_canon(d->kind)) {
        const int64_t tight = d->kind == LPG_ROW_MAJOR ? d->cols : d->rows;
        if (d->ld && d->ld != tight) return fail(LPG_EUNSUPPORTED, "lpg_elementwise_packed: canonical buffers must be tight");
    } else {
        PView v;
        rc = make_pview(d, "lpg_elementwise_packed", &v);
        if (rc) return rc;
        if (!v.default_order) return fail(LPG_EUNSUPPORTED, "lpg_elementwise_packed: packed buffers must have the default block order");
    }
    if (!x0 || !out) return fail(LPG_EINVAL, "lpg_elementwise_packed: NULL pointer");
    if (op != LPG_EW_SCALE && !x1) return fail(LPG_EINVAL, "lpg_elementwise_packed: op needs x1");
    const size_t bytes = desc_bytes(d);
    if ((uintptr_t)x0 % 16 || (uintptr_t)out % 16 || (x1 && (uintptr_t)x1 % 16))
        return fail(LPG_EALIGN, "lpg_elementwise_packed: buffers must be 16-byte aligned");
    if (!launch) return LPG_OK;
    EwArgs a;
    a.x0 = (const char *)x0;
    a.x1 = (op == LPG_EW_SCALE) ? nullptr : (const char *)x1;
    a.out = (char *)out;
    a.n16 = (int64_t)(bytes / 16);
    a.tail = (int32_t)((bytes % 16) / elem_size(d->dtype));
    a.op = op;
    a.s = s;
    hipError_t e = launch_elementwise(a, d->dtype, st);
    if (e != hipSuccess) return fail(LPG_EHIP, "lpg_elementwise_packed: %s", hipGetErrorString(e));
    return LPG_OK;
}

// ------------------------------------------------- softmax / RMS normalisation / RoPE

// Shared by the row operations: resolve x/out under descriptor d (PACKED_A or ROW_MAJOR).
struct RowTarget {
    bool packed;
    const char *x;
    char *out;
    int64_t kbs, row_stride, slot;
    int32_t ngroups, nkb;
};
static int make_row_target(const char *what, const void *x, void *out, const lpg_desc *d, RowTarget *t)
{
    int rc = check_common(d, what);
    if (rc) return rc;
    if (d->kind != LPG_PACKED_A && d->kind != LPG_ROW_MAJOR)
        return fail(LPG_EUNSUPPORTED, "%s: kind %d (rows must be the free index: PACKED_A, or ROW_MAJOR)", what, d->kind);
    if (bdiv(d) != 1) return fail(LPG_EUNSUPPORTED, "%s: batch_div must be 1", what);
    if (!x || !out) return fail(LPG_EINVAL, "%s: NULL pointer", what);
    *t = RowTarget{};
    t->packed = d->kind == LPG_PACKED_A;
    if (t->packed) {
        PView v;
        rc = make_pview(d, what, &v);
        if (rc) return rc;
        if (!v.default_order) return fail(LPG_EUNSUPPORTED, "%s: packed buffers must have the default block order", what);
        if ((uintptr_t)x % 16 || (uintptr_t)out % 16) return fail(LPG_EALIGN, "%s: packed buffers must be 16-byte aligned", what);
        t->x = (const char *)x + v.origin;
        t->out = (char *)out + v.origin;
        t->kbs = v.kb_stride;
        t->slot = v.slot_step;
        t->ngroups = (int32_t)((v.F + 31) / 32);
        t->nkb = (int32_t)((v.K + kb_of(v.dtype) - 1) / kb_of(v.dtype));
        if ((int64_t)v.batch * t->ngroups * 4 > 0x7fffffff) return fail(LPG_EUNSUPPORTED, "%s: too many row groups", what);
    } else {
        CView v;
        rc = make_cview(d, what, &v);
        if (rc) return rc;
        if ((uintptr_t)x % v.es || (uintptr_t)out % v.es) return fail(LPG_EALIGN, "%s: misaligned buffer", what);
        t->x = (const char *)x + v.origin * v.es;
        t->out = (char *)out + v.origin * v.es;
        t->row_stride = v.row_stride * v.es;
        t->slot = v.slot_step * v.es;
        if ((int64_t)v.batch * d->rows > 0x7fffffff) return fail(LPG_EUNSUPPORTED, "%s: too many rows", what);
    }
    return LPG_OK;
}

static int do_row_op(int op, const void *x, const void *weight, void *out, const lpg_desc *d, float scalar, int causal,
                     hipStream_t st, bool launch)
{
    const char *what = op == kRowSoftmax ? "lpg_softmax_packed" : "lpg_rmsnorm_packed";
    RowTarget t;
    int rc = make_row_target(what, x, out, d, &t);
    if (rc) return rc;
    if (op == kRowSoftmax && !(scalar > 0.0f && scalar <= 3.0e38f))
        return fail(LPG_EINVAL, "%s: scale must be positive and finite", what);
    if (op == kRowRmsNorm) {
        if (!weight) return fail(LPG_EINVAL, "%s: NULL weight", what);
        if ((uintptr_t)weight % 4) return fail(LPG_EALIGN, "%s: misaligned weight", what);
        if (!(scalar >= 0.0f)) return fail(LPG_EINVAL, "%s: eps must be >= 0", what);
    }
    RowArgs a{};
    a.x = t.x;
    a.out = t.out;
    a.weight = (const float *)weight;
    a.kbs = t.kbs;
    a.row_stride = t.row_stride;
    a.slot = t.slot;
    a.rows = (int32_t)d->rows;
    a.cols = (int32_t)d->cols;
    a.ngroups = t.ngroups;
    a.nkb = t.nkb;
    a.batch = nbatch(d);
    a.causal = causal != 0;
    a.scalar = op == kRowSoftmax ? (float)((double)scalar * 1.4426950408889634) : scalar;
    if (!launch) return LPG_OK;
    hipError_t e = launch_row_op(a, op, d->dtype, t.packed, st);
    if (e != hipSuccess) return fail(LPG_EHIP, "%s: %s", what, hipGetErrorString(e));
    return LPG_OK;
}

static int do_rope(const void *x, void *out, const lpg_desc *d, const void *cos_t, const void *sin_t, int head_dim,
                   hipStream_t st, bool launch)
{
    const char *what = "lpg_rope_packed";
    RowTarget t;
    int rc = make_row_target(what, x, out, d, &t);
    if (rc) return rc;
    if (!cos_t || !sin_t) return fail(LPG_EINVAL, "%s: NULL table", what);
    if ((uintptr_t)cos_t % 16 || (uintptr_t)sin_t % 16) return fail(LPG_EALIGN, "%s: tables must be 16-byte aligned", what);
    if (head_dim <= 0 || head_dim % 2) return fail(LPG_EINVAL, "%s: head_dim must be a positive even number", what);
    if (d->cols % head_dim) return fail(LPG_EINVAL, "%s: cols %lld is not a multiple of head_dim %d", what, (long long)d->cols, head_dim);
    RopeArgs a{};
    a.x = t.x;
    a.out = t.out;
    a.cos_t = (const float *)cos_t;
    a.sin_t = (const float *)sin_t;
    a.kbs = t.kbs;
    a.row_stride = t.row_stride;
    a.slot = t.slot;
    a.rows = (int32_t)d->rows;
    a.nheads = (int32_t)(d->cols / head_dim);
    a.half = head_dim / 2;
    a.ngroups = t.ngroups;
    a.batch = nbatch(d);
    if (t.packed) {
        // a head's two halves must be whole fragments apart
        const int kf = d->dtype == LPG_F32 ? 8 : 16;
        if (head_dim % (2 * kf))
            return fail(LPG_EUNSUPPORTED, "%s: packed %s needs head_dim to be a multiple of %d", what,
                        d->dtype == LPG_F32 ? "fp32" : "bf16", 2 * kf);
        a.fph = head_dim / (2 * kf);
        a.nlo = a.nheads * a.fph;
        a.npad = out == x ? 0 : t.nkb * kFragsPerBlock - 2 * a.nlo;
    }
    if (!launch) return LPG_OK;
    hipError_t e = launch_rope(a, d->dtype, t.packed, st);
    if (e != hipSuccess) return fail(LPG_EHIP, "%s: %s", what, hipGetErrorString(e));
    return LPG_OK;
}

// -------------------------------------------------------------------------- attention

static int do_attention(const void *Q, const lpg_desc *q_d, const void *K, const lpg_desc *k_d, const void *V,
                        const lpg_desc *v_d, void *O, const lpg_desc *o_d, float scale, int flags, hipStream_t st,
                        bool launch)
{
    const char *what = "lpg_attention_packed";
    if (flags & ~(LPG_ATTN_CAUSAL | LPG_ATTN_NO_SOFTMAX)) return fail(LPG_EINVAL, "%s: unknown flag bits in %d", what, flags);
    const bool softmax = !(flags & LPG_ATTN_NO_SOFTMAX);
    PView q, k, v, o;
    int rc = make_pview(q_d, what, &q);
    if (rc) return rc;
    if ((rc = make_pview(k_d, what, &k))) return rc;
    if ((rc = make_pview(v_d, what, &v))) return rc;
    if ((rc = make_pview(o_d, what, &o))) return rc;
    if (q_d->kind != LPG_PACKED_A || o_d->kind != LPG_PACKED_A)
        return fail(LPG_ELAYOUT, "%s: Q and O must be PACKED_A (queries x head_dim)", what);
    if (!q.default_order || !k.default_order || !v.default_order || !o.default_order)
        return fail(LPG_EUNSUPPORTED, "%s: packed buffers must have the default block order", what);
    if (q.dtype != k.dtype || q.dtype != v.dtype || q.dtype != o.dtype)
        return fail(LPG_EUNSUPPORTED, "%s: Q, K, V, O must share one dtype", what);
    const int64_t dh = q.K, tq = q.F, tk = k.F;
    if (dh != 64 && dh != 128) return fail(LPG_EUNSUPPORTED, "%s: head_dim %lld (64 and 128 are built)", what, (long long)dh);
    // K: free index = key, contraction = head_dim (PACKED_A of K, or PACKED_B of K^T: same bytes);
    // V: free index = head_dim, contraction = key (PACKED_B of V, or PACKED_A of V^T)
    if (k.K != dh || v.F != dh || v.K != tk || o.F != tq || o.K != dh)
        return fail(LPG_EINVAL, "%s: shapes do not fit (Q %lldx%lld, K keys %lld x %lld, V %lld keys x %lld, O %lldx%lld)", what,
                    (long long)tq, (long long)dh, (long long)tk, (long long)k.K, (long long)v.K, (long long)v.F,
                    (long long)o.F, (long long)o.K);
    if (q.batch != o.batch || k.batch != q.batch || v.batch != q.batch)
        return fail(LPG_EINVAL, "%s: batch counts differ", what);
    if (q.bdiv != 1 || o.bdiv != 1) return fail(LPG_EUNSUPPORTED, "%s: batch_div applies to K and V only", what);
    if (softmax && !(scale > 0.0f && scale <= 3.0e38f)) return fail(LPG_EINVAL, "%s: scale must be positive and finite", what);
    if (!softmax && !(scale >= -3.0e38f && scale <= 3.0e38f)) return fail(LPG_EINVAL, "%s: scale must be finite", what);
    if (tq > 0 && tk <= 0) return fail(LPG_EINVAL, "%s: no keys", what);
    if ((rc = check_ptr16(Q, what)) || (rc = check_ptr16(K, what)) || (rc = check_ptr16(V, what)) || (rc = check_ptr16(O, what)))
        return rc;
    if (O == Q || O == K || O == V) return fail(LPG_EINVAL, "%s: O must not alias an input", what);
    if ((int64_t)q.batch * ((tq + 127) / 128) > 0x7fffffff) return fail(LPG_EUNSUPPORTED, "%s: too many query blocks", what);
    if (!launch) return LPG_OK;
    AttnArgs a{};
    a.Q = (const char *)Q + q.origin;
    a.K = (const char *)K + k.origin;
    a.V = (const char *)V + v.origin;
    a.O = (char *)O + o.origin;
    a.q_kbs = q.kb_stride; a.k_kbs = k.kb_stride; a.v_kbs = v.kb_stride; a.o_kbs = o.kb_stride;
    a.q_slot = q.slot_step; a.k_slot = k.slot_step; a.v_slot = v.slot_step; a.o_slot = o.slot_step;
    a.k_div = k.bdiv;
    a.v_div = v.bdiv;
    a.tq = (int32_t)tq;
    a.tk = (int32_t)tk;
    a.q_groups = (int32_t)((tq + 31) / 32);
    a.k_groups = (int32_t)((tk + 31) / 32);
    a.v_nkb = (int32_t)((tk + kb_of(q.dtype) - 1) / kb_of(q.dtype));
    a.batch = q.batch;
    a.causal = (flags & LPG_ATTN_CAUSAL) != 0;
    a.softmax = softmax;
    a.sl = (float)((double)scale * 1.4426950408889634);
    a.scale = scale;
    hipError_t e = launch_attention(a, q.dtype, (int)dh, st);
    if (e != hipSuccess) return fail(LPG_EHIP, "%s: %s", what, hipGetErrorString(e));
    return LPG_OK;
}

// ------------------------------------------------------------------------------ chain

// Packed geometry two descriptors must share to address the same bytes the same way.
struct Geometry {
    int dtype;
    int64_t PF, PK, bstride, gs, ks;
};
static bool geometry_of(const lpg_desc *d, Geometry *g)
{
    if (!is_packed(d->kind)) return false;
    const bool tr = d->kind == LPG_PACKED_B;
    const int64_t prow = d->parent_rows ? d->parent_rows : d->rows;
    const int64_t pcol = d->parent_cols ? d->parent_cols : d->cols;
    g->dtype = d->dtype;
    g->PF = tr ? pcol : prow;
    g->PK = tr ? prow : pcol;
    g->bstride = d->batch_stride;
    g->gs = d->group_stride;
    g->ks = d->kblock_stride;
    return true;
}

// Row-major twin of a packed descriptor: the same logical views (rows, cols, origin,
// per-slot steps) over a tight row-major parent.
static lpg_desc canonical_twin(const lpg_desc *p)
{
    lpg_desc c = *p;
    const int64_t prow = p->parent_rows ? p->parent_rows : p->rows;
    const int64_t pcol = p->parent_cols ? p->parent_cols : p->cols;
    c.kind = LPG_ROW_MAJOR;
    c.ld = pcol;
    c.parent_rows = prow;
    c.parent_cols = pcol;
    c.batch_stride = p->batch_stride ? prow * pcol : 0;
    c.group_stride = c.kblock_stride = 0;
    return c;
}

struct Slot {
    const void *packed;   // packed buffer this slot mirrors
    char *canon;          // row-major copy in the workspace
    size_t bytes;
    bool canonical_live;  // the up-to-date copy is the canonical one
};

static size_t twin_bytes(const lpg_desc *p)
{
    lpg_desc c = canonical_twin(p);
    return (desc_bytes(&c) + 255) / 256 * 256;
}

static inline bool is_row_stage(int type)
{
    return type == LPG_STAGE_SOFTMAX || type == LPG_STAGE_RMSNORM || type == LPG_STAGE_ROPE;
}

// A softmax / RMS normalisation / RoPE stage on buffers x, out under descriptor d (the
// stage's own, or their row-major twins in the canonical control).
static int run_row_stage(const lpg_stage &s, const void *x, void *out, const lpg_desc *d, hipStream_t hs, bool launch)
{
    switch (s.type) {
        case LPG_STAGE_SOFTMAX: return do_row_op(kRowSoftmax, x, nullptr, out, d, s.scalar, s.op, hs, launch);
        case LPG_STAGE_RMSNORM: return do_row_op(kRowRmsNorm, x, s.in1, out, d, s.scalar, 0, hs, launch);
        default: return do_rope(x, out, d, s.in1, s.in2, s.op, hs, launch);
    }
}

static bool later_reads(const lpg_stage *st, int n, int from, const void *buf, bool *by_compute)
{
    bool any = false;
    *by_compute = false;
    for (int i = from; i < n; ++i) {
        const lpg_stage &s = st[i];
        const bool reads = s.in0 == buf || (s.type == LPG_STAGE_GEMM && (s.in1 == buf || s.in2 == buf || s.epi_arg == buf)) ||
                           (s.type == LPG_STAGE_ATTENTION && (s.in1 == buf || s.in2 == buf)) ||
                           (s.type == LPG_STAGE_ELEMENTWISE && s.in1 == buf);
        if (reads) {
            any = true;
            if (s.type != LPG_STAGE_PACK && s.type != LPG_STAGE_UNPACK) *by_compute = true;
        }
        if (s.out == buf) break;  // overwritten from here on
    }
    return any;
}

static int validate_stage(const lpg_stage &s, int i)
{
    switch (s.type) {
        case LPG_STAGE_PACK:
        case LPG_STAGE_UNPACK: {
            PView pv;
            CView cv;
            const bool pk = s.type == LPG_STAGE_PACK;
            int rc = make_pview(pk ? &s.out_d : &s.in0_d, "lpg_chain pack/unpack", &pv, kInnerF | kInnerK | kOffGrid);
            if (rc) return rc;
            rc = make_cview(pk ? &s.in0_d : &s.out_d, "lpg_chain pack/unpack", &cv);
            if (rc) return rc;
            if (!s.in0 || !s.out) return fail(LPG_EINVAL, "lpg_chain: stage %d has a NULL buffer", i);
            return LPG_OK;
        }
        case LPG_STAGE_GEMM:
            return do_gemm(s.alpha, s.in0, &s.in0_d, s.in1, &s.in1_d, s.beta, s.in2, s.out, &s.out_d, s.op,
                           s.epi_arg, nullptr, false);
        case LPG_STAGE_ELEMENTWISE:
            return do_elementwise(s.op, s.in0, s.in1, s.scalar, s.out, &s.out_d, nullptr, false);
        case LPG_STAGE_SOFTMAX:
        case LPG_STAGE_RMSNORM:
        case LPG_STAGE_ROPE:
            return run_row_stage(s, s.in0, s.out, &s.out_d, nullptr, false);
        case LPG_STAGE_ATTENTION:
            return do_attention(s.in0, &s.in0_d, s.in1, &s.in1_d, s.in2, &s.in2_d, s.out, &s.out_d, s.scalar, s.op,
                                nullptr, false);
        default:
            return fail(LPG_EINVAL, "lpg_chain: stage %d has unknown type %d", i, s.type);
    }
}

// Every packed input that an earlier stage wrote must be read with the geometry it
// was written in (the consumer's loads assume the producer's block strides).
static int check_links(const lpg_stage *st, int n)
{
    for (int i = 0; i < n; ++i) {
        const lpg_stage &s = st[i];
        struct In { const void *p; const lpg_desc *d; } ins[4];
        int ni = 0;
        if (s.type == LPG_STAGE_GEMM) {
            ins[ni++] = {s.in0, &s.in0_d};
            ins[ni++] = {s.in1, &s.in1_d};
            if (s.in2) ins[ni++] = {s.in2, &s.out_d};
            if (s.epi_arg) ins[ni++] = {s.epi_arg, &s.out_d};
        } else if (s.type == LPG_STAGE_ELEMENTWISE) {
            ins[ni++] = {s.in0, &s.out_d};
            if (s.in1) ins[ni++] = {s.in1, &s.out_d};
        } else if (s.type == LPG_STAGE_ATTENTION) {
            ins[ni++] = {s.in0, &s.in0_d};
            ins[ni++] = {s.in1, &s.in1_d};
            ins[ni++] = {s.in2, &s.in2_d};
        } else if (is_row_stage(s.type)) {
            ins[ni++] = {s.in0, &s.out_d};
        } else if (s.type == LPG_STAGE_UNPACK) {
            ins[ni++] = {s.in0, &s.in0_d};
        }
        for (int k = 0; k < ni; ++k) {
            Geometry gi;
            if (!geometry_of(ins[k].d, &gi)) continue;
            for (int j = i - 1; j >= 0; --j) {
                if (st[j].out != ins[k].p) continue;
                Geometry gj;
                if (!geometry_of(&st[j].out_d, &gj))
                    return fail(LPG_ELAYOUT, "lpg_chain: stage %d reads as packed a buffer stage %d wrote canonical", i, j);
                if (gi.dtype != gj.dtype || gi.PF != gj.PF || gi.PK != gj.PK || gi.bstride != gj.bstride || gi.gs != gj.gs ||
                    gi.ks != gj.ks)
                    return fail(LPG_ELAYOUT,
                                "lpg_chain: stage %d reads a buffer with packed geometry (free %lld, k %lld, dtype %d) "
                                "but stage %d wrote it as (free %lld, k %lld, dtype %d)",
                                i, (long long)gi.PF, (long long)gi.PK, gi.dtype, j, (long long)gj.PF,
                                (long long)gj.PK, gj.dtype);
                break;
            }
        }
    }
    return LPG_OK;
}

static int run_stage(const lpg_stage &s, hipStream_t hs)
{
    switch (s.type) {
        case LPG_STAGE_PACK: return do_pack_unpack(true, s.in0, &s.in0_d, s.out, &s.out_d, hs);
        case LPG_STAGE_UNPACK: return do_pack_unpack(false, s.out, &s.out_d, s.in0, &s.in0_d, hs);
        case LPG_STAGE_GEMM:
            return do_gemm(s.alpha, s.in0, &s.in0_d, s.in1, &s.in1_d, s.beta, s.in2, s.out, &s.out_d, s.op, s.epi_arg,
                           hs, true);
        case LPG_STAGE_SOFTMAX:
        case LPG_STAGE_RMSNORM:
        case LPG_STAGE_ROPE: return run_row_stage(s, s.in0, s.out, &s.out_d, hs, true);
        case LPG_STAGE_ATTENTION:
            return do_attention(s.in0, &s.in0_d, s.in1, &s.in1_d, s.in2, &s.in2_d, s.out, &s.out_d, s.scalar, s.op, hs,
                                true);
        default: return do_elementwise(s.op, s.in0, s.in1, s.scalar, s.out, &s.out_d, hs, true);
    }
}

// Canonical control.  After each computing stage whose packed result a later computing
// stage reads, the result is unpacked to a row-major copy in the workspace; before a
// GEMM reads such a buffer it is packed again from that copy (once).  An elementwise
// stage whose inputs are all held canonically runs on the row-major copies and leaves a
// row-major result, as a BLAS-API program would.  Outputs are bit-identical to the
// propagated mode because pack and unpack are permutations.
static int chain_canonical(const lpg_stage *st, int n, char *ws, size_t ws_bytes, hipStream_t hs, bool dry,
                           size_t *need)
{
    std::vector<Slot> slots;
    size_t used = 0;
    // the dry pass validates the control's own stages too: it hands them addresses that have the
    // workspace's alignment and are never dereferenced
    if (!ws) ws = (char *)(uintptr_t)4096;
    auto find = [&](const void *p) -> Slot * {
        for (auto &s : slots)
            if (s.packed == p) return &s;
        return nullptr;
    };
    // descriptors under which stages wrote a buffer since it was last re-packed
    struct Wrote { const void *p; lpg_desc d; bool pending; };
    std::vector<Wrote> wrote;
    auto note_write = [&](const void *p, const lpg_desc &d) {
        for (auto &w : wrote)
            if (w.p == p && w.pending && !memcmp(&w.d, &d, sizeof(d))) return;  // already due for the same re-pack
        wrote.push_back({p, d, true});
    };
    auto get_slot = [&](const void *p, const lpg_desc *pd) -> Slot * {
        Slot *s = find(p);
        const size_t bytes = twin_bytes(pd);
        if (s && s->bytes >= bytes) return s;
        Slot ns{p, ws + used, bytes, false};
        used += bytes;
        if (s) { *s = ns; return s; }
        slots.push_back(ns);
        return &slots.back();
    };
    // Pack again, from the row-major copy, everything stages wrote into `p`.
    auto repack = [&](const void *p) -> int {
        Slot *s = find(p);
        if (!s || !s->canonical_live) return LPG_OK;
        for (auto &w : wrote) {
            if (w.p != p || !w.pending) continue;
            if (!dry) {
                lpg_desc c = canonical_twin(&w.d);
                int rc = do_pack_unpack(true, s->canon, &c, p, &w.d, hs);
                if (rc) return rc;
            }
            w.pending = false;
        }
        s->canonical_live = false;
        return LPG_OK;
    };

    for (int i = 0; i < n; ++i) {
        const lpg_stage &s = st[i];
        if (s.type == LPG_STAGE_ELEMENTWISE || is_row_stage(s.type)) {
            const bool sm = is_row_stage(s.type);  // one layout-bound input (tables, weights are plain arrays)
            Slot *s0 = find(s.in0), *s1 = (!sm && s.in1) ? find(s.in1) : nullptr;
            const size_t tb = is_packed(s.out_d.kind) ? twin_bytes(&s.out_d) : 0;
            const bool canon_in = s0 && s0->canonical_live && s0->bytes == tb &&
                                  (sm || !s.in1 || (s1 && s1->canonical_live && s1->bytes == tb));
            bool by_compute = false;
            later_reads(st, n, i + 1, s.out, &by_compute);
            if (canon_in && is_packed(s.out_d.kind)) {
                // run on the row-major copies; result stays row-major in the workspace
                lpg_desc c = canonical_twin(&s.out_d);
                Slot *so = get_slot(s.out, &s.out_d);
                // get_slot may have moved the vector: look the inputs up again
                s0 = find(s.in0);
                s1 = (!sm && s.in1) ? find(s.in1) : nullptr;
                {
                    int rc;
                    if (sm) {
                        rc = run_row_stage(s, s0->canon, so->canon, &c, hs, !dry);
                    } else {
                        c.ld = 0;
                        rc = do_elementwise(s.op, s0->canon, s1 ? s1->canon : nullptr, s.scalar, so->canon, &c, hs, !dry);
                    }
                    if (rc) return rc;
                }
                so->canonical_live = true;
                note_write(s.out, s.out_d);
                continue;
            }
            int rc = repack(s.in0);
            if (rc) return rc;
            if (!sm && s.in1) { rc = repack(s.in1); if (rc) return rc; }
        } else if (s.type == LPG_STAGE_GEMM || s.type == LPG_STAGE_ATTENTION) {
            int rc = repack(s.in0);
            if (rc) return rc;
            rc = repack(s.in1);
            if (rc) return rc;
            if (s.in2) { rc = repack(s.in2); if (rc) return rc; }
            if (s.epi_arg) { rc = repack(s.epi_arg); if (rc) return rc; }
        } else if (s.type == LPG_STAGE_UNPACK) {
            int rc = repack(s.in0);
            if (rc) return rc;
        }
        if (!dry) {
            int rc = run_stage(s, hs);
            if (rc) return rc;
        }
        if (s.type != LPG_STAGE_PACK && s.type != LPG_STAGE_UNPACK && is_packed(s.out_d.kind)) {
            bool by_compute = false;
            later_reads(st, n, i + 1, s.out, &by_compute);
            if (by_compute) {
                note_write(s.out, s.out_d);
                Slot *so = get_slot(s.out, &s.out_d);
                if (!dry) {
                    lpg_desc c = canonical_twin(&s.out_d);
                    int rc = do_pack_unpack(false, so->canon, &c, s.out, &s.out_d, hs);
                    if (rc) return rc;
                }
                so->canonical_live = true;
            }
        } else if (s.type == LPG_STAGE_PACK) {
            Slot *so = find(s.out);
            if (so) so->canonical_live = false;
        }
        if (!dry && used > ws_bytes) return fail(LPG_EWORKSPACE, "lpg_chain: workspace too small (%zu needed so far, %zu given)", used, ws_bytes);
    }
    if (need) *need = used;
    return LPG_OK;
}

}  // namespace lpg

// ================================================================================ C ABI

using namespace lpg;

extern "C" {

size_t lpg_packed_bytes(const lpg_desc *d) { return desc_bytes(d); }

int lpg_layout_offset(const lpg_desc *d, int64_t b, int64_t row, int64_t col, int64_t *offset)
{
    int rc = check_common(d, "lpg_layout_offset");
    if (rc) return rc;
    if (!offset) return fail(LPG_EINVAL, "lpg_layout_offset: NULL offset");
    if (b < 0 || b >= nbatch(d) || row < 0 || row >= d->rows || col < 0 || col >= d->cols)
        return fail(LPG_EINVAL, "lpg_layout_offset: index out of range");
    const int64_t slot = b / bdiv(d);
    if (is_canon(d->kind)) {
        CView v;
        rc = make_cview(d, "lpg_layout_offset", &v);
        if (rc) return rc;
        *offset = v.origin + slot * v.slot_step + row * v.row_stride + col * v.col_stride;
        return LPG_OK;
    }
    PView v;
    rc = make_pview(d, "lpg_layout_offset", &v, kInnerF | kInnerK | kOffGrid);
    if (rc) return rc;
    // v.origin is the block that holds the view's first element
    const int64_t f = (v.transposed ? col : row) + v.f_off, k = (v.transposed ? row : col) + v.k_off;
    const int64_t KB = kb_of(v.dtype), KV = 16 / v.es, KF = 2 * KV;
    const int64_t kin = k % KB, c = kin / KF, r = kin % KF;
    const int64_t h = (r >> 2) & 1, vv = 4 * (r >> 3) + (r & 3);
    const int64_t bytes = v.origin + slot * v.slot_step + (k / KB) * v.kb_stride + (f / 32) * v.g_stride +
                          c * kFragBytes + h * 512 + (f % 32) * 16 + vv * v.es;
    *offset = bytes / v.es;
    return LPG_OK;
}

int lpg_pack(const void *src, const lpg_desc *src_d, void *dst, const lpg_desc *dst_d, void *stream)
{
    return do_pack_unpack(true, src, src_d, dst, dst_d, (hipStream_t)stream);
}

int lpg_unpack(const void *src, const lpg_desc *src_d, void *dst, const lpg_desc *dst_d, void *stream)
{
    return do_pack_unpack(false, dst, dst_d, src, src_d, (hipStream_t)stream);
}

int lpg_gemm_packed(float alpha, const void *A, const lpg_desc *a_d, const void *B, const lpg_desc *b_d, float beta,
                    const void *C_in, void *C_out, const lpg_desc *c_d, int epilogue_op, const void *epi_arg,
                    void *stream)
{
    return do_gemm(alpha, A, a_d, B, b_d, beta, C_in, C_out, c_d, epilogue_op, epi_arg, (hipStream_t)stream, true);
}

int lpg_elementwise_packed(int op, const void *x0, const void *x1, float s, void *out, const lpg_desc *d,
                           void *stream)
{
    return do_elementwise(op, x0, x1, s, out, d, (hipStream_t)stream, true);
}

int lpg_softmax_packed(const void *x, void *out, const lpg_desc *d, float scale, int causal, void *stream)
{
    return do_row_op(kRowSoftmax, x, nullptr, out, d, scale, causal, (hipStream_t)stream, true);
}

int lpg_attention_packed(const void *Q, const lpg_desc *q_d, const void *K, const lpg_desc *k_d, const void *V,
                         const lpg_desc *v_d, void *O, const lpg_desc *o_d, float scale, int flags, void *stream)
{
    return do_attention(Q, q_d, K, k_d, V, v_d, O, o_d, scale, flags, (hipStream_t)stream, true);
}

int lpg_rmsnorm_packed(const void *x, const float *weight, void *out, const lpg_desc *d, float eps, void *stream)
{
    return do_row_op(kRowRmsNorm, x, weight, out, d, eps, 0, (hipStream_t)stream, true);
}

int lpg_rope_tables(float *cos_t, float *sin_t, int64_t rows, int32_t head_dim, double base, int64_t pos0, void *stream)
{
    if (rows < 0 || head_dim <= 0 || head_dim % 2 || !(base > 0.0))
        return fail(LPG_EINVAL, "lpg_rope_tables: need rows >= 0, an even positive head_dim and base > 0");
    if (rows == 0) return LPG_OK;
    if (!cos_t || !sin_t) return fail(LPG_EINVAL, "lpg_rope_tables: NULL table");
    if ((uintptr_t)cos_t % 4 || (uintptr_t)sin_t % 4) return fail(LPG_EALIGN, "lpg_rope_tables: misaligned table");
    if (rows * (head_dim / 2) > ((int64_t)1 << 38)) return fail(LPG_EUNSUPPORTED, "lpg_rope_tables: table too large");
    hipError_t e = launch_rope_tables(cos_t, sin_t, rows, head_dim, base, (double)pos0, (hipStream_t)stream);
    if (e != hipSuccess) return fail(LPG_EHIP, "lpg_rope_tables: %s", hipGetErrorString(e));
    return LPG_OK;
}

int lpg_rope_packed(const void *x, void *out, const lpg_desc *d, const float *cos_t, const float *sin_t,
                    int32_t head_dim, void *stream)
{
    return do_rope(x, out, d, cos_t, sin_t, head_dim, (hipStream_t)stream, true);
}

size_t lpg_chain_workspace_bytes(const lpg_stage *stages, int n, int mode)
{
    if (!stages || n < 0) return (size_t)-1;
    if (mode == LPG_CHAIN_PROPAGATED) return 0;
    if (mode != LPG_CHAIN_CANONICAL) return (size_t)-1;
    for (int i = 0; i < n; ++i)
        if (validate_stage(stages[i], i)) return (size_t)-1;
    size_t need = 0;
    if (chain_canonical(stages, n, nullptr, 0, nullptr, true, &need)) return (size_t)-1;
    return need;
}

int lpg_chain(const lpg_stage *stages, int n, int mode, void *workspace, size_t workspace_bytes, void *stream)
{
    if (n < 0 || (n > 0 && !stages)) return fail(LPG_EINVAL, "lpg_chain: bad stage array");
    if (mode != LPG_CHAIN_PROPAGATED && mode != LPG_CHAIN_CANONICAL) return fail(LPG_EINVAL, "lpg_chain: bad mode %d", mode);
    for (int i = 0; i < n; ++i) {
        int rc = validate_stage(stages[i], i);
        if (rc) return rc;
    }
    int rc = check_links(stages, n);
    if (rc) return rc;
    hipStream_t hs = (hipStream_t)stream;
    if (mode == LPG_CHAIN_PROPAGATED) {
        for (int i = 0; i < n; ++i) {
            rc = run_stage(stages[i], hs);
            if (rc) return rc;
        }
        return LPG_OK;
    }
    size_t need = 0;
    rc = chain_canonical(stages, n, nullptr, 0, nullptr, true, &need);
    if (rc) return rc;
    if (need > workspace_bytes || (need && !workspace))
        return fail(LPG_EWORKSPACE, "lpg_chain: workspace too small (%zu needed, %zu given)", need, workspace_bytes);
    if (need && (uintptr_t)workspace % 256) return fail(LPG_EALIGN, "lpg_chain: workspace must be 256-byte aligned");
    return chain_canonical(stages, n, (char *)workspace, workspace_bytes, hs, false, nullptr);
}

int lpg_chain_static(const lpg_stage *stages, int n, int mode, void *stream)
{
    if (mode == LPG_CHAIN_PROPAGATED) return lpg_chain(stages, n, mode, nullptr, 0, stream);
    void *ws = nullptr;
    size_t ws_bytes = 0;
    hipError_t e = static_scratch(&ws, &ws_bytes);
    if (e != hipSuccess) return fail(LPG_EHIP, "lpg_chain_static: %s", hipGetErrorString(e));
    int rc = lpg_chain(stages, n, mode, ws, ws_bytes, stream);
    if (rc == LPG_EWORKSPACE) {
        char msg[sizeof(g_err)];
        snprintf(msg, sizeof(msg), "%s", g_err);
        return fail(LPG_EWORKSPACE, "lpg_chain_static: the chain's row-major copies do not fit the library's %zu-byte static scratch (%s)", ws_bytes, msg);
    }
    return rc;
}

int lpg_tune_set(int key, int value)
{
    if (tune_set(key, value)) return fail(LPG_EINVAL, "lpg_tune_set: unknown key %d", key);
    return LPG_OK;
}

int lpg_tune_get(int key, int *value)
{
    if (key < 0 || key >= LPG_TUNE_KEYS || !value) return fail(LPG_EINVAL, "lpg_tune_get: unknown key %d or NULL value", key);
    *value = tune_get(key);
    return LPG_OK;
}

const char *lpg_last_error(void) { return g_err; }

const char *lpg_version(void) { return "lpg 0.1 (gfx950)"; }

}  // extern "C"
