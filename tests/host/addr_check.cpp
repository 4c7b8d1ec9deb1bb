// Host check of the per-tile index arithmetic the GEMM kernels use (csrc/lpg_addr.h):
//  * div_by equals the machine's unsigned division for every divisor up to 4096 and a
//    spread of larger ones, on dividends around every multiple boundary and over the range;
//  * the split (wave-uniform + per-lane) form of a staged fragment's source offset equals
//    the plain per-lane definition for every lane, row offset, ragged extent, group and
//    fragment, and the definition never leaves the operand.
// Prints "ok <cases>" and returns 0, or the first mismatch and 1.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <initializer_list>

#include "lpg_addr.h"

using namespace lpg;

static uint64_t cases = 0;

static int check_div(uint32_t d)
{
    const DivBy k = div_setup(d);
    auto one = [&](uint32_t n) {
        ++cases;
        if (div_by(n, k) != n / d) {
            std::printf("div_by(%u, %u) = %u, want %u\n", n, d, div_by(n, k), n / d);
            return 1;
        }
        return 0;
    };
    for (uint32_t n = 0; n < 20000; ++n)
        if (one(n)) return 1;
    for (uint64_t q = 0; q < 400; ++q)
        for (int e = -1; e <= 1; ++e) {
            const uint64_t lo = q * d + e, hi = (0xffffffffull / d - q) * (uint64_t)d + e;
            if (lo <= 0xffffffffull && one((uint32_t)lo)) return 1;
            if (hi <= 0xffffffffull && one((uint32_t)hi)) return 1;
        }
    uint32_t x = 2463534242u ^ d;
    for (int i = 0; i < 4000; ++i) {
        x ^= x << 13; x ^= x >> 17; x ^= x << 5;
        if (one(x)) return 1;
    }
    return 0;
}

static int check_packed(int foff, int rows, int TG, int fs)
{
    FragOperand o{};
    o.canon = 0;
    o.foff = foff;
    o.rows = rows;
    o.gs = 4096 * 3;           // a store stride: groups three blocks apart
    o.kbs = (int64_t)1 << 24;  // far larger than any group offset, so the parts can be told apart
    const int gmax = (foff + rows - 1) >> 5;
    const int groups = (rows + 31) / 32;  // groups of the view (the kernel's FLg / FRg)
    for (int g0 = 0; g0 < groups; g0 += TG) {
        int ng = groups - g0 < TG ? groups - g0 : TG;
        for (int grp = 0; grp < TG; ++grp)
            for (int c = 0; c < fs; ++c)
                for (int lane = 0; lane < 64; ++lane) {
                    ++cases;
                    const int64_t want = frag_offset_reference(o, g0, ng, grp, c, lane);
                    const int64_t got = frag_uniform_packed(o, g0, ng, grp, c, frag_lane_hi(o, lane)) + frag_lane_packed(o, lane);
                    if (want != got) {
                        std::printf("packed foff %d rows %d g0 %d grp %d c %d lane %d: %lld, want %lld\n", foff, rows, g0, grp,
                                    c, lane, (long long)got, (long long)want);
                        return 1;
                    }
                    // inside the operand: block index within [0, gmax], K block and fragment as asked
                    const int64_t kpart = (int64_t)(c / 4) * o.kbs;
                    const int64_t rest = want - kpart;
                    const int64_t grp_abs = rest / o.gs + g0 - (rest < 0 && rest % o.gs ? 1 : 0);
                    const int64_t in_group = rest - (grp_abs - g0) * o.gs;
                    if (grp_abs < 0 || grp_abs > gmax || in_group < 0 || in_group + 16 > 4096) {
                        std::printf("packed foff %d rows %d g0 %d grp %d c %d lane %d leaves the operand (block %lld of 0..%d, byte %lld)\n",
                                    foff, rows, g0, grp, c, lane, (long long)grp_abs, gmax, (long long)in_group);
                        return 1;
                    }
                }
    }
    return 0;
}

static int check_canon(int rows, int TG, int fs)
{
    FragOperand o{};
    o.canon = 1;
    o.rows = rows;
    o.ld = 4 * 1000003;  // bytes between rows
    o.kf_bytes = 32;
    const int groups = (rows + 31) / 32;
    for (int g0 = 0; g0 < groups; g0 += TG)
        for (int grp = 0; grp < TG; ++grp)
            for (int c = 0; c < fs; ++c)
                for (int lane = 0; lane < 64; ++lane) {
                    ++cases;
                    const int64_t want = frag_offset_reference(o, g0, 0, grp, c, lane);
                    const int64_t row = want / o.ld;
                    if (row < 0 || row > rows - 1 || want - row * o.ld != c * 32 + (lane >> 5) * 16) {
                        std::printf("canonical rows %d g0 %d grp %d c %d lane %d leaves the operand\n", rows, g0, grp, c, lane);
                        return 1;
                    }
                    if (!frag_group_inside(o, g0, grp)) continue;
                    const int64_t got = frag_uniform_canon(o, g0, grp, c) + frag_lane_canon(o, lane);
                    if (want != got) {
                        std::printf("canonical rows %d g0 %d grp %d c %d lane %d: %lld, want %lld\n", rows, g0, grp, c, lane,
                                    (long long)got, (long long)want);
                        return 1;
                    }
                }
    return 0;
}

// tile_at equals its definition, and the walk visits every (batch, row, column) exactly once
static int check_walk(int tiles_l, int tiles_r, int gm, int batch)
{
    const TileWalk w = tile_walk_setup(tiles_l, tiles_r, gm);
    const uint32_t total = (uint32_t)(tiles_l * tiles_r * batch);
    static unsigned char seen[64 * 64 * 8];
    for (uint32_t i = 0; i < total; ++i) seen[i] = 0;
    for (uint32_t pid = 0; pid < total; ++pid) {
        ++cases;
        int b, tl, tr, b2, tl2, tr2;
        tile_at_reference(w, pid, b, tl, tr);
        tile_at(w, pid, b2, tl2, tr2);
        if (b != b2 || tl != tl2 || tr != tr2) {
            std::printf("walk %dx%d gm %d pid %u: (%d,%d,%d), want (%d,%d,%d)\n", tiles_l, tiles_r, gm, pid, b2, tl2, tr2, b, tl, tr);
            return 1;
        }
        if (b < 0 || b >= batch || tl < 0 || tl >= tiles_l || tr < 0 || tr >= tiles_r) {
            std::printf("walk %dx%d gm %d pid %u leaves the grid: (%d,%d,%d)\n", tiles_l, tiles_r, gm, pid, b, tl, tr);
            return 1;
        }
        unsigned char &s = seen[(b * tiles_l + tl) * tiles_r + tr];
        if (s) {
            std::printf("walk %dx%d gm %d: tile (%d,%d,%d) visited twice\n", tiles_l, tiles_r, gm, b, tl, tr);
            return 1;
        }
        s = 1;
    }
    return 0;
}

int main()
{
    for (int tiles_l = 1; tiles_l <= 40; ++tiles_l)
        for (int tiles_r : {1, 2, 3, 7, 16, 33})
            for (int gm : {1, 2, 3, 4, 5, 8, 16})
                for (int batch : {1, 3})
                    if (check_walk(tiles_l, tiles_r, gm, batch)) return 1;
    for (uint32_t d = 1; d <= 4096; ++d)
        if (check_div(d)) return 1;
    const uint32_t big[] = {4097, 65535, 65536, 65537, 1u << 20, (1u << 20) + 1, 0x7fffffffu, 0x80000000u, 0x80000001u, 0xfffffffeu, 0xffffffffu};
    for (uint32_t d : big)
        if (check_div(d)) return 1;
    const int extents[] = {1, 2, 31, 32, 33, 63, 64, 65, 95, 127, 128, 129, 200, 255, 256, 257, 300};
    for (int TG : {2, 4, 8})
        for (int fs : {2, 4, 8})
            for (int rows : extents) {
                for (int foff = 0; foff < 32; ++foff)
                    if (check_packed(foff, rows, TG, fs)) return 1;
                if (check_canon(rows, TG, fs)) return 1;
            }
    std::printf("ok %llu\n", (unsigned long long)cases);
    return 0;
}
