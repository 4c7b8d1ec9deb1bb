// Driver for an AddressSanitizer + UndefinedBehaviorSanitizer build of the library's host side
// (csrc/lpg_api.cpp is compiled into this program with the sanitizers; the kernels' launchers
// come from the in-tree liblpg.so and are never reached).  Every call below either fails
// validation or is a dry pass: no kernel is launched and no device memory is touched, so the
// pointers are fakes.  What is exercised: descriptor validation, view and stride arithmetic,
// the host index function over whole descriptors (checked to be a bijection into the sized
// buffer), the chain's link check and the control chain's dry pass.  Exit code 0 = clean.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <set>
#include <vector>

#include "lpg.h"

static int fails = 0;
#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "check failed: %s (line %d): %s\n", #c, __LINE__, lpg_last_error()); ++fails; } } while (0)

static lpg_desc D(int kind, int dtype, int64_t rows, int64_t cols)
{
    lpg_desc d;
    std::memset(&d, 0, sizeof(d));
    d.kind = kind; d.dtype = dtype; d.rows = rows; d.cols = cols; d.batch = 1; d.batch_div = 1;
    return d;
}

static void index_function_is_a_bijection(lpg_desc d)
{
    const size_t bytes = lpg_packed_bytes(&d);
    CHECK(bytes > 0);
    const int es = d.dtype == LPG_F32 ? 4 : 2;
    std::set<int64_t> seen;
    const int nb = d.batch > 0 ? d.batch : 1;
    for (int b = 0; b < nb; ++b)
        for (int64_t r = 0; r < d.rows; ++r)
            for (int64_t c = 0; c < d.cols; ++c) {
                int64_t off = -1;
                CHECK(lpg_layout_offset(&d, b, r, c, &off) == LPG_OK);
                CHECK(off >= 0 && (size_t)(off + 1) * es <= bytes);
                if (d.batch_div <= 1) CHECK(seen.insert(off).second);
            }
    int64_t off;
    CHECK(lpg_layout_offset(&d, 0, d.rows, 0, &off) == LPG_EINVAL);
    CHECK(lpg_layout_offset(&d, nb, 0, 0, &off) == LPG_EINVAL);
    CHECK(lpg_layout_offset(&d, 0, 0, 0, nullptr) == LPG_EINVAL);
}

static lpg_stage gemm_stage(const void *A, lpg_desc a, const void *B, lpg_desc b, void *C, lpg_desc c, float beta = 0.0f,
                            const void *cin = nullptr)
{
    lpg_stage s;
    std::memset(&s, 0, sizeof(s));
    s.type = LPG_STAGE_GEMM; s.alpha = 1.0f; s.beta = beta;
    s.in0 = A; s.in0_d = a; s.in1 = B; s.in1_d = b; s.in2 = cin; s.out = C; s.out_d = c;
    return s;
}

int main()
{
    char *const fake = (char *)0x100000;
    // ---- index function: plain, ragged, views on and off the grid, batches, both orders, strides
    for (int dtype = 0; dtype < 2; ++dtype) {
        const int64_t KB = dtype == LPG_F32 ? 32 : 64, blk = 32 * KB;
        index_function_is_a_bijection(D(LPG_PACKED_A, dtype, 33, 2 * KB + 5));
        index_function_is_a_bijection(D(LPG_PACKED_B, dtype, 2 * KB + 5, 33));
        lpg_desc v = D(LPG_PACKED_A, dtype, 20, 30);
        v.parent_rows = 100; v.parent_cols = 3 * KB; v.row0 = 37; v.col0 = 11;
        index_function_is_a_bijection(v);
        lpg_desc h = D(LPG_PACKED_A, dtype, 64, KB);
        h.parent_rows = 64; h.parent_cols = 4 * KB; h.batch = 4; h.batch_col_step = KB;
        index_function_is_a_bijection(h);
        lpg_desc s = D(LPG_PACKED_A, dtype, 70, 2 * KB + 9);
        s.group_stride = 3 * blk; s.kblock_stride = blk;
        index_function_is_a_bijection(s);
        s.group_stride = 2 * blk; s.kblock_stride = 7 * blk;
        index_function_is_a_bijection(s);
        s.group_stride = blk + 8;
        CHECK(lpg_packed_bytes(&s) == 0);
        s.group_stride = 2 * blk; s.kblock_stride = 3 * blk;      // blocks would overlap
        CHECK(lpg_packed_bytes(&s) == 0);
        lpg_desc rm = D(LPG_ROW_MAJOR, dtype, 9, 7);
        rm.ld = 10; rm.batch = 3; rm.batch_stride = 100;
        index_function_is_a_bijection(rm);
    }
    // ---- descriptor errors (nothing is launched: every call fails on the host)
    lpg_desc pa = D(LPG_PACKED_A, LPG_F32, 64, 64), pb = D(LPG_PACKED_B, LPG_F32, 64, 64), rm = D(LPG_ROW_MAJOR, LPG_F32, 64, 64);
    CHECK(lpg_pack(fake, &pa, fake, &pa, nullptr) == LPG_ELAYOUT);
    CHECK(lpg_pack(fake, &rm, fake + 4, &pa, nullptr) == LPG_EALIGN);
    CHECK(lpg_pack(nullptr, &rm, fake, &pa, nullptr) == LPG_EINVAL);
    CHECK(lpg_unpack(fake, &rm, fake, &rm, nullptr) == LPG_ELAYOUT);
    CHECK(lpg_gemm_packed(1.0f, fake, &pb, fake, &pb, 0.0f, nullptr, fake + 4096, &pa, 0, nullptr, nullptr) == LPG_ELAYOUT);
    CHECK(lpg_gemm_packed(1.0f, fake, &pa, fake, &pb, 1.0f, nullptr, fake + 4096, &pa, 0, nullptr, nullptr) == LPG_EINVAL);
    CHECK(lpg_gemm_packed(1.0f, fake, &pa, fake + 8192, &pb, 0.0f, nullptr, fake, &pa, 0, nullptr, nullptr) == LPG_EINVAL);
    CHECK(lpg_gemm_packed(1.0f, fake, &pa, fake, &pb, 0.0f, nullptr, fake + 4096, &pa, 7, nullptr, nullptr) == LPG_EINVAL);
    lpg_desc neg = pa; neg.rows = -1;
    CHECK(lpg_gemm_packed(1.0f, fake, &neg, fake, &pb, 0.0f, nullptr, fake + 4096, &pa, 0, nullptr, nullptr) == LPG_EINVAL);
    CHECK(lpg_elementwise_packed(9, fake, fake, 1.0f, fake, &pa, nullptr) == LPG_EINVAL);
    CHECK(lpg_softmax_packed(fake, fake, &pb, 1.0f, 0, nullptr) == LPG_EUNSUPPORTED);
    CHECK(lpg_softmax_packed(fake, fake, &pa, 0.0f, 0, nullptr) == LPG_EINVAL);
    CHECK(lpg_rmsnorm_packed(fake, nullptr, fake, &pa, 1e-5f, nullptr) == LPG_EINVAL);
    CHECK(lpg_rope_packed(fake, fake, &pa, (const float *)fake, (const float *)fake, 48, nullptr) == LPG_EINVAL);
    CHECK(lpg_rope_tables((float *)fake, (float *)fake, 8, 7, 10000.0, 0, nullptr) == LPG_EINVAL);
    CHECK(lpg_attention_packed(fake, &pa, fake, &pa, fake, &pb, fake + 4096, &pa, 1.0f, 64, nullptr) == LPG_EINVAL);
    CHECK(std::strlen(lpg_last_error()) > 0);
    CHECK(lpg_tune_set(99, 1) == LPG_EINVAL && lpg_tune_set(LPG_TUNE_TILE, 3) == LPG_OK);
    int val = 0;
    CHECK(lpg_tune_get(LPG_TUNE_TILE, &val) == LPG_OK && val == 3 && lpg_tune_set(LPG_TUNE_TILE, LPG_TUNE_AUTO) == LPG_OK);
    // ---- chains: the link check and the control chain's dry pass
    {
        const int64_t m = 70, d = 96, hdim = 130;
        lpg_desc xd = D(LPG_PACKED_A, LPG_F32, m, d), hd = D(LPG_PACKED_A, LPG_F32, m, hdim), w1 = D(LPG_PACKED_B, LPG_F32, d, hdim),
                 w2 = D(LPG_PACKED_B, LPG_F32, hdim, d), xr = D(LPG_ROW_MAJOR, LPG_F32, m, d);
        char *X = fake, *PX = fake + (1 << 20), *W1 = fake + (2 << 20), *W2 = fake + (3 << 20), *H = fake + (4 << 20),
             *H2 = fake + (5 << 20), *Y = fake + (6 << 20), *OUT = fake + (7 << 20);
        std::vector<lpg_stage> st(6);
        std::memset(st.data(), 0, st.size() * sizeof(lpg_stage));
        st[0].type = LPG_STAGE_PACK; st[0].in0 = X; st[0].in0_d = xr; st[0].out = PX; st[0].out_d = xd;
        st[1] = gemm_stage(PX, xd, W1, w1, H, hd);
        st[2].type = LPG_STAGE_ELEMENTWISE; st[2].op = LPG_EW_SCALE; st[2].scalar = 0.5f; st[2].in0 = H; st[2].out = H2; st[2].out_d = hd;
        st[3].type = LPG_STAGE_SOFTMAX; st[3].op = 1; st[3].scalar = 1.0f; st[3].in0 = H2; st[3].out = H2; st[3].out_d = hd;
        st[4] = gemm_stage(H2, hd, W2, w2, Y, xd, 1.0f, PX);
        st[5].type = LPG_STAGE_UNPACK; st[5].in0 = Y; st[5].in0_d = xd; st[5].out = OUT; st[5].out_d = xr;
        CHECK(lpg_chain_workspace_bytes(st.data(), (int)st.size(), LPG_CHAIN_PROPAGATED) == 0);
        const size_t need = lpg_chain_workspace_bytes(st.data(), (int)st.size(), LPG_CHAIN_CANONICAL);
        CHECK(need != (size_t)-1 && need >= (size_t)(2 * m * hdim * 4));
        // too small a workspace, a misaligned one, a bad mode: all refused before any launch
        CHECK(lpg_chain(st.data(), (int)st.size(), LPG_CHAIN_CANONICAL, fake + (8 << 20), need - 1, nullptr) == LPG_EWORKSPACE);
        CHECK(lpg_chain(st.data(), (int)st.size(), LPG_CHAIN_CANONICAL, fake + (8 << 20) + 16, need, nullptr) == LPG_EALIGN);
        CHECK(lpg_chain(st.data(), (int)st.size(), 5, nullptr, 0, nullptr) == LPG_EINVAL);
        // a consumer that names another geometry than the producer wrote
        lpg_desc wrong = hd; wrong.parent_rows = 128; wrong.parent_cols = hdim;
        std::vector<lpg_stage> bad = st;
        bad[4] = gemm_stage(H2, wrong, W2, w2, Y, xd, 1.0f, PX);
        CHECK(lpg_chain(bad.data(), (int)bad.size(), LPG_CHAIN_PROPAGATED, nullptr, 0, nullptr) == LPG_ELAYOUT);
        bad = st;
        bad[2].type = 42;
        CHECK(lpg_chain_workspace_bytes(bad.data(), (int)bad.size(), LPG_CHAIN_CANONICAL) == (size_t)-1);
        CHECK(lpg_chain(nullptr, 3, LPG_CHAIN_PROPAGATED, nullptr, 0, nullptr) == LPG_EINVAL);
    }
    if (fails) { std::fprintf(stderr, "%d checks failed\n", fails); return 1; }
    std::puts("host sanitizer driver: clean");
    return 0;
}
