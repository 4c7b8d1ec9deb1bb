/*
 * CPU oracle for layout-propagating GEMM chains.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain reference the GPU library is judged against.  It
 * shares no code, header, table or constant with the HIP path and must never be
 * linked or called from it; only tests, the smoke check and the benchmark's
 * CPU-baseline leg may use it.
 *
 * What it holds
 *   orc_gemm        C = alpha*A*B + beta*C      (paper Eq. 1), fp64, row-major
 *   orc_round_f32 / orc_round_bf16   storage rounding of an fp64 array
 *   orc_bf16_bits   fp32 bit pattern -> bf16 bit pattern, round-nearest-even
 *   orc_silu_mul    g*sigmoid(g)*u in fp64 (the activation F_i of Eq. 2 used by
 *                   the Llama-shaped workload)
 *   orc_softmax_rows  scale, optional causal mask, row softmax (Alg. 2, the steps
 *                   between the two attention GEMMs)
 *   orc_pack / orc_unpack            canonical <-> packed layout, by walking the
 *                   layout's nested dimensions outermost to innermost (the GPU
 *                   re-design of the dimension order of Eq. 3); the _strided forms
 *                   take the block order / store stride of section III-C
 *
 * The packed layout P(X; F, K) of a matrix with free dimension F (index f) and
 * contraction dimension K (index k), element size es in {4, 2} bytes:
 *   KV = 16/es            elements one lane holds in a 128-bit register
 *   KF = 2*KV             k-extent of one fragment (32 f  x KF k  = 1 KiB)
 *   KB = 4*KF             k-extent of one block    (32 f  x KB k  = 4 KiB)
 *   Fp = F rounded up to 32,  Kp = K rounded up to KB  (padding holds zeros)
 * nested dimensions, outermost to innermost:
 *   [kb : Kp/KB] [g : Fp/32] [c : 4] [h : 2] [fl : 32] [v : KV]
 * with  f = 32*g + fl  and  k = KB*kb + KF*c + 8*(v/4) + 4*h + (v%4).
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#include <stdlib.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Threads orc_gemm will use (reported beside timings). */
int orc_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ GEMM */

/* Eq. 1 on row-major fp64 arrays.  For each output row the k-sum is taken in
 * ascending l with a plain multiply and add per term; alpha multiplies the
 * finished sum once; beta == 0 means C_in is never read (it may be NULL or
 * hold NaN).  Rows are independent, so they are spread over OpenMP threads. */
void orc_gemm(int64_t m, int64_t n, int64_t k, double alpha,
              const double *A, int64_t lda, const double *B, int64_t ldb,
              double beta, const double *Cin, int64_t ldcin,
              double *Cout, int64_t ldc)
{
#pragma omp parallel
    {
        double *acc = (double *)malloc((size_t)(n > 0 ? n : 1) * sizeof(double));
#pragma omp for schedule(static)
        for (int64_t i = 0; i < m; ++i) {
            for (int64_t j = 0; j < n; ++j) acc[j] = 0.0;
            for (int64_t l = 0; l < k; ++l) {
                const double a = A[i * lda + l];
                const double *brow = B + l * ldb;
                for (int64_t j = 0; j < n; ++j) acc[j] += a * brow[j];
            }
            for (int64_t j = 0; j < n; ++j) {
                double v = alpha * acc[j];
                if (beta != 0.0) v += beta * Cin[i * ldcin + j];
                Cout[i * ldc + j] = v;
            }
        }
        free(acc);
    }
}

/* ------------------------------------------------------- storage rounding */

/* bf16 = upper 16 bits of an fp32, rounded to nearest, ties to even; NaN stays
 * NaN (quiet bit forced so that truncation cannot turn it into infinity). */
uint16_t orc_bf16_bits(uint32_t u)
{
    if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu) != 0u)
        return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

void orc_bf16_bits_array(const uint32_t *u, uint16_t *out, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) out[i] = orc_bf16_bits(u[i]);
}

void orc_round_f32(double *x, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) x[i] = (double)(float)x[i];
}

void orc_round_bf16(double *x, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) {
        float f = (float)x[i];
        uint32_t u;
        memcpy(&u, &f, 4);
        u = (uint32_t)orc_bf16_bits(u) << 16;
        memcpy(&f, &u, 4);
        x[i] = (double)f;
    }
}

/* --------------------------------------------------------------- activation */

void orc_silu_mul(const double *g, const double *u, double *out, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) out[i] = g[i] / (1.0 + exp(-g[i])) * u[i];
}

/* Row softmax of scale*x (Alg. 2: scale, optional mask, softmax), fp64, row-major.
 * causal != 0 applies the usual attention mask: row i keeps columns j <= i + shift
 * (shift = cols - rows aligns the last row with the last column); masked positions get
 * probability 0.  Each row: subtract the maximum of the kept entries, exponentiate, divide
 * by the sum. */
void orc_softmax_rows(const double *x, double *out, int64_t rows, int64_t cols, double scale, int causal)
{
    const int64_t shift = cols - rows;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i) {
        int64_t last = causal ? i + shift : cols - 1;
        if (last > cols - 1) last = cols - 1;
        const double *xr = x + i * cols;
        double *o = out + i * cols;
        for (int64_t j = 0; j < cols; ++j) o[j] = 0.0;
        if (last < 0) continue;
        double m = scale * xr[0];
        for (int64_t j = 1; j <= last; ++j)
            if (scale * xr[j] > m) m = scale * xr[j];
        double sum = 0.0;
        for (int64_t j = 0; j <= last; ++j) {
            o[j] = exp(scale * xr[j] - m);
            sum += o[j];
        }
        for (int64_t j = 0; j <= last; ++j) o[j] = o[j] / sum;
    }
}

/* ----------------------------------------------------------- packed layout */

/* Canonical element (f, k) of the matrix being packed.  `k_contig` != 0 means
 * the canonical array is contiguous along k (address f*ld + k), else along f
 * (address k*ld + f).  A left operand (free = rows) stored row-major, or a
 * right operand (free = columns) stored column-major, is k-contiguous. */
static inline size_t canon_index(int64_t f, int64_t k, int64_t ld, int k_contig)
{
    return k_contig ? (size_t)(f * ld + k) : (size_t)(k * ld + f);
}

/* Where block (kb, g) of a packed parent starts, in elements.  The parent is a
 * grid of blocks; gs / ks are the element distances from group to group and
 * from K block to K block (the "block order" and "store stride" parameters of
 * section III-C).  0, 0 selects the default order: the groups of a K block back
 * to back, K blocks back to back. */
static inline size_t block_start(int64_t kb, int64_t g, int64_t PFp, int64_t KB, int64_t gs, int64_t ks)
{
    if (gs == 0 && ks == 0) { gs = 32 * KB; ks = PFp * KB; }
    else if (gs == 0) gs = 32 * KB;
    else if (ks == 0) ks = 32 * KB;
    return (size_t)(kb * ks + g * gs);
}

/* Pack the view [f0, f0+F) x [k0, k0+K) of a packed parent with extents
 * (PF, PK).  `canon` points at canonical element (f=0,k=0) OF THE VIEW.
 * Every block the view touches is written whole: positions whose (f,k) falls
 * outside the view's logical extent receive zero bytes.  f0 must be a multiple
 * of 32 and k0 of KB.  Elements are moved as raw es-byte patterns.  gs, ks:
 * block strides of the parent (see block_start). */
void orc_pack_strided(const void *canon, int64_t ld, int k_contig, int es,
                      void *packed, int64_t PF, int64_t PK,
                      int64_t f0, int64_t k0, int64_t F, int64_t K, int64_t gs, int64_t ks)
{
    const int64_t KV = 16 / es, KF = 2 * KV, KB = 4 * KF;
    const int64_t PFp = (PF + 31) / 32 * 32;
    (void)PK;
    const int64_t Fp = (F + 31) / 32 * 32, Kp = (K + KB - 1) / KB * KB;
    const unsigned char *src = (const unsigned char *)canon;
    unsigned char *dst = (unsigned char *)packed;
    for (int64_t kb = 0; kb < Kp / KB; ++kb)
        for (int64_t g = 0; g < Fp / 32; ++g) {
            /* position of block (kb, g) of the view inside the parent buffer */
            size_t pos = block_start(k0 / KB + kb, f0 / 32 + g, PFp, KB, gs, ks);
            for (int64_t c = 0; c < 4; ++c)
                for (int64_t h = 0; h < 2; ++h)
                    for (int64_t fl = 0; fl < 32; ++fl)
                        for (int64_t v = 0; v < KV; ++v, ++pos) {
                            const int64_t f = 32 * g + fl;
                            const int64_t k = KB * kb + KF * c + 8 * (v / 4) + 4 * h + (v % 4);
                            if (f < F && k < K)
                                memcpy(dst + pos * es, src + canon_index(f, k, ld, k_contig) * es, es);
                            else
                                memset(dst + pos * es, 0, es);
                        }
        }
}

void orc_pack(const void *canon, int64_t ld, int k_contig, int es,
              void *packed, int64_t PF, int64_t PK,
              int64_t f0, int64_t k0, int64_t F, int64_t K)
{
    orc_pack_strided(canon, ld, k_contig, es, packed, PF, PK, f0, k0, F, K, 0, 0);
}

/* Inverse of orc_pack: copies the view's logical elements back to canonical
 * order and ignores padding. */
void orc_unpack_strided(void *canon, int64_t ld, int k_contig, int es,
                        const void *packed, int64_t PF, int64_t PK,
                        int64_t f0, int64_t k0, int64_t F, int64_t K, int64_t gs, int64_t ks)
{
    const int64_t KV = 16 / es, KF = 2 * KV, KB = 4 * KF;
    const int64_t PFp = (PF + 31) / 32 * 32;
    (void)PK;
    const int64_t Fp = (F + 31) / 32 * 32, Kp = (K + KB - 1) / KB * KB;
    unsigned char *dst = (unsigned char *)canon;
    const unsigned char *src = (const unsigned char *)packed;
    for (int64_t kb = 0; kb < Kp / KB; ++kb)
        for (int64_t g = 0; g < Fp / 32; ++g) {
            size_t pos = block_start(k0 / KB + kb, f0 / 32 + g, PFp, KB, gs, ks);
            for (int64_t c = 0; c < 4; ++c)
                for (int64_t h = 0; h < 2; ++h)
                    for (int64_t fl = 0; fl < 32; ++fl)
                        for (int64_t v = 0; v < KV; ++v, ++pos) {
                            const int64_t f = 32 * g + fl;
                            const int64_t k = KB * kb + KF * c + 8 * (v / 4) + 4 * h + (v % 4);
                            if (f < F && k < K)
                                memcpy(dst + canon_index(f, k, ld, k_contig) * es, src + pos * es, es);
                        }
        }
}

void orc_unpack(void *canon, int64_t ld, int k_contig, int es,
                const void *packed, int64_t PF, int64_t PK,
                int64_t f0, int64_t k0, int64_t F, int64_t K)
{
    orc_unpack_strided(canon, ld, k_contig, es, packed, PF, PK, f0, k0, F, K, 0, 0);
}
