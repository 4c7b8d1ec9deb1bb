/* Driver for an AddressSanitizer + UndefinedBehaviorSanitizer build of the CPU oracle
 * (oracle/lpg_oracle.c is compiled into this program).  It walks the oracle's entry points
 * over ragged shapes, views, block strides and degenerate sizes with exactly sized heap
 * buffers, so that any access outside them, any misaligned or overflowing arithmetic, is
 * reported by the sanitizers; a few invariants are checked on the way.  Exit code 0 = clean. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void orc_gemm(int64_t m, int64_t n, int64_t k, double alpha, const double *A, int64_t lda, const double *B, int64_t ldb,
              double beta, const double *Cin, int64_t ldcin, double *Cout, int64_t ldc);
void orc_round_f32(double *x, int64_t n);
void orc_round_bf16(double *x, int64_t n);
uint16_t orc_bf16_bits(uint32_t u);
void orc_silu_mul(const double *g, const double *u, double *out, int64_t n);
void orc_softmax_rows(const double *x, double *out, int64_t rows, int64_t cols, double scale, int causal);
void orc_pack_strided(const void *canon, int64_t ld, int k_contig, int es, void *packed, int64_t PF, int64_t PK,
                      int64_t f0, int64_t k0, int64_t F, int64_t K, int64_t gs, int64_t ks);
void orc_unpack_strided(void *canon, int64_t ld, int k_contig, int es, const void *packed, int64_t PF, int64_t PK,
                        int64_t f0, int64_t k0, int64_t F, int64_t K, int64_t gs, int64_t ks);

static int fails = 0;
#define CHECK(c) do { if (!(c)) { fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); ++fails; } } while (0)

static double *dvec(size_t n, unsigned seed)
{
    double *p = (double *)malloc((n ? n : 1) * sizeof(double));
    for (size_t i = 0; i < n; ++i) { seed = seed * 1664525u + 1013904223u; p[i] = (double)(int)(seed >> 24) / 64.0 - 2.0; }
    return p;
}

static void gemm_cases(void)
{
    const int64_t dims[] = {0, 1, 2, 5, 17, 33};
    for (int a = 0; a < 6; ++a) for (int b = 0; b < 6; ++b) for (int c = 0; c < 6; ++c) {
        const int64_t m = dims[a], n = dims[b], k = dims[c];
        double *A = dvec((size_t)(m * k), 1), *B = dvec((size_t)(k * n), 2), *C = dvec((size_t)(m * n), 3);
        double *out = dvec((size_t)(m * n), 4);
        orc_gemm(m, n, k, 1.5, A, k, B, n, 0.0, NULL, 0, out, n);           /* beta == 0: C_in never touched */
        orc_gemm(m, n, k, -1.0, A, k, B, n, 0.5, C, n, out, n);
        if (m && n) {                                                          /* one element against a direct sum */
            double s = 0.0;
            for (int64_t l = 0; l < k; ++l) s += A[(m - 1) * k + l] * B[l * n + (n - 1)];
            CHECK(fabs(out[m * n - 1] - (-s + 0.5 * C[m * n - 1])) <= 1e-9 * (1.0 + fabs(s)));
        }
        free(A); free(B); free(C); free(out);
    }
}

static void pack_cases(void)
{
    for (int es = 2; es <= 4; es += 2) {
        const int64_t KB = es == 4 ? 32 : 64, blk = 32 * KB;
        const int64_t PF = 70, PK = 2 * KB + 9;                                /* 3 groups x 3 K blocks */
        const int64_t ng = 3, nk = 3;
        const int64_t orders[3][2] = {{0, 0}, {nk * blk, blk}, {2 * blk, 7 * blk}};
        for (int o = 0; o < 3; ++o) {
            const int64_t gs = orders[o][0], ks = orders[o][1];
            const int64_t g_eff = gs ? gs : blk, k_eff = ks ? ks : (gs ? blk : ng * blk);
            const size_t elems = (size_t)((ng - 1) * g_eff + (nk - 1) * k_eff + blk);
            unsigned char *packed = (unsigned char *)malloc(elems * es);
            memset(packed, 0xAB, elems * es);
            /* whole parent, then a view on the grid with a ragged extent at the parent's edge */
            const int64_t views[2][4] = {{0, 0, PF, PK}, {32, KB, PF - 32, PK - KB}};
            for (int v = 0; v < 2; ++v) {
                const int64_t f0 = views[v][0], k0 = views[v][1], F = views[v][2], K = views[v][3];
                for (int kc = 0; kc < 2; ++kc) {
                    const int64_t ld = (kc ? K : F) + 3;
                    const size_t cn = (size_t)((kc ? F : K) * ld);
                    unsigned char *canon = (unsigned char *)malloc(cn * es), *back = (unsigned char *)malloc(cn * es);
                    for (size_t i = 0; i < cn * es; ++i) canon[i] = (unsigned char)(i * 7 + 1);
                    memset(back, 0, cn * es);
                    orc_pack_strided(canon, ld, kc, es, packed, PF, PK, f0, k0, F, K, gs, ks);
                    orc_unpack_strided(back, ld, kc, es, packed, PF, PK, f0, k0, F, K, gs, ks);
                    for (int64_t f = 0; f < F; ++f) for (int64_t k = 0; k < K; ++k) {
                        const size_t at = (size_t)(kc ? f * ld + k : k * ld + f) * es;
                        CHECK(memcmp(canon + at, back + at, es) == 0);
                    }
                    free(canon); free(back);
                }
            }
            free(packed);
        }
    }
}

static void elementwise_cases(void)
{
    const int64_t shapes[][2] = {{1, 1}, {3, 7}, {7, 3}, {5, 5}, {0, 4}, {4, 0}};
    for (int s = 0; s < 6; ++s) for (int causal = 0; causal < 2; ++causal) {
        const int64_t r = shapes[s][0], c = shapes[s][1];
        double *x = dvec((size_t)(r * c), 9), *out = dvec((size_t)(r * c), 10);
        orc_softmax_rows(x, out, r, c, 0.7, causal);
        for (int64_t i = 0; i < r; ++i) {
            double sum = 0.0;
            for (int64_t j = 0; j < c; ++j) sum += out[i * c + j];
            const int64_t last = causal ? i + c - r : c - 1;
            if (c) CHECK(last < 0 ? sum == 0.0 : fabs(sum - 1.0) < 1e-12);
        }
        free(x); free(out);
    }
    double *g = dvec(100, 5), *u = dvec(100, 6), *o = dvec(100, 7);
    orc_silu_mul(g, u, o, 100);
    orc_silu_mul(g, u, o, 0);
    orc_round_f32(o, 100);
    orc_round_bf16(o, 100);
    free(g); free(u); free(o);
    CHECK(orc_bf16_bits(0x3F800000u) == 0x3F80u);
    CHECK(orc_bf16_bits(0x3F808000u) == 0x3F80u);                               /* tie to even */
    CHECK(orc_bf16_bits(0x3F818000u) == 0x3F82u);
    CHECK((orc_bf16_bits(0x7F800001u) & 0x7FFFu) > 0x7F80u);                   /* NaN stays NaN */
    CHECK(orc_bf16_bits(0xFFFFFFFFu) != 0);
}

int main(void)
{
    gemm_cases();
    pack_cases();
    elementwise_cases();
    if (fails) { fprintf(stderr, "%d checks failed\n", fails); return 1; }
    puts("oracle sanitizer driver: clean");
    return 0;
}
