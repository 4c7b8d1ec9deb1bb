// Index arithmetic of the GEMM kernels that runs once per tile, written so that it can be
// checked on the host: exact division by launch constants without a divide instruction, and
// the source address of a staged fragment split into a part that is the same for all lanes
// of a wave (scalar registers, a few scalar instructions per fragment) and a part that is
// the same for all fragments of an operand (computed once per tile).  The plain per-lane
// definitions stand beside the split forms; tests/host/addr_check.cpp compares them over
// every lane, offset and ragged extent.  With short contractions (attention scores, K = 64)
// a tile is only a few thousand MFMA cycles long, and the per-lane form of this arithmetic
// (two 64-bit multiplies per fragment and lane, eight divisions per tile) cost about a third
// of that.
#pragma once

#include <cstdint>

#if defined(__HIPCC__)
#define LPG_HD __host__ __device__ __forceinline__
#else
#define LPG_HD inline
#endif

namespace lpg {

// ---- exact unsigned division by a divisor fixed at launch (round-up reciprocal, Granlund
// and Montgomery 1994): n / d = (t + ((n - t) >> s1)) >> s2 with t = high word of n * m, for
// every 32-bit n and every d >= 1.
struct DivBy {
    uint32_t m, s1, s2;
};

inline DivBy div_setup(uint32_t d)
{
    uint32_t l = 0;
    while (l < 32 && ((uint64_t)1 << l) < d) ++l;  // l = ceil(log2 d)
    DivBy r;
    r.m = (uint32_t)(((((uint64_t)1 << l) - d) << 32) / d + 1);
    r.s1 = l < 1 ? l : 1;
    r.s2 = l < 1 ? 0 : l - 1;
    return r;
}

LPG_HD uint32_t div_by(uint32_t n, DivBy d)
{
    const uint32_t t = (uint32_t)(((uint64_t)n * d.m) >> 32);
    return (t + ((n - t) >> d.s1)) >> d.s2;
}

// ---- the tile walk: position pid of a launch's tile sequence -> (batch, tile row, tile column).
// A batch's tiles_l x tiles_r tiles are walked in bands of gm tile rows, down the band's rows
// first, so that consecutive positions share operand panels; the last band may be lower.
struct TileWalk {
    int tiles_l, tiles_r, gm;
    DivBy by_tiles, by_band;  // division by tiles_l * tiles_r and by gm * tiles_r
};

inline TileWalk tile_walk_setup(int tiles_l, int tiles_r, int gm)
{
    TileWalk w;
    w.tiles_l = tiles_l;
    w.tiles_r = tiles_r;
    w.gm = gm;
    w.by_tiles = div_setup((uint32_t)(tiles_l * tiles_r));
    w.by_band = div_setup((uint32_t)(gm * tiles_r));
    return w;
}

// Definition, with the machine's division.
LPG_HD void tile_at_reference(const TileWalk &w, uint32_t pid, int &b, int &tl, int &tr)
{
    const uint32_t ntile = (uint32_t)(w.tiles_l * w.tiles_r);
    b = (int)(pid / ntile);
    const int tp = (int)(pid % ntile);
    const int width = w.gm * w.tiles_r;
    const int first_l = (tp / width) * w.gm;
    const int gsz = w.tiles_l - first_l < w.gm ? w.tiles_l - first_l : w.gm;
    tl = first_l + (tp % width) % gsz;
    tr = (tp % width) / gsz;
}

// The same through the launch's reciprocals; full bands of a power-of-two height need no
// division at all.
LPG_HD void tile_at(const TileWalk &w, uint32_t pid, int &b, int &tl, int &tr)
{
    const uint32_t ntile = (uint32_t)(w.tiles_l * w.tiles_r);
    const uint32_t bb = div_by(pid, w.by_tiles);
    b = (int)bb;
    const int tp = (int)(pid - bb * ntile);
    const int width = w.gm * w.tiles_r;
    const int band = (int)div_by((uint32_t)tp, w.by_band);
    const int first_l = band * w.gm;
    const int in_band = tp - band * width;
    const int gsz = w.tiles_l - first_l < w.gm ? w.tiles_l - first_l : w.gm;
    if (gsz == w.gm && (w.gm & (w.gm - 1)) == 0) {
        tl = first_l + (in_band & (w.gm - 1));
        tr = in_band >> (31 - __builtin_clz((unsigned)w.gm));
    } else {  // the last, lower band, or a band height that is no power of two
        tl = first_l + in_band % gsz;
        tr = in_band / gsz;
    }
}

// ---- where a lane fetches its 16 bytes of a staged fragment from.
// One operand of a launch, as the fragment fetch sees it.
struct FragOperand {
    int canon;        // 0: packed; 1: canonical, contiguous along the contraction index
    int foff;         // packed: rows between the view's origin and the 32-grid (0..31)
    int rows;         // logical extent of the free dimension
    int64_t gs, kbs;  // packed: bytes between 32-groups / between K blocks
    int64_t ld;       // canonical: bytes between consecutive free indices
    int kf_bytes;     // canonical: bytes of one fragment's contraction extent in a row
};

constexpr int kAddrFragBytes = 1024;   // one fragment
constexpr int kAddrFragsPerBlock = 4;  // fragments of a K block

// Definition.  Offset from the tile's operand base (packed: first block of the tile's first
// group at the step's first K block; canonical: element (0, k of the step) of the operand)
// of the 16 bytes that lane `lane` contributes to fragment c of the step for group `grp` of
// the tile (g0 = the tile's first group, ng = how many of its groups exist).  A group the
// tile does not have is replaced by its last existing one, a row past the view's end by the
// view's last block (packed) or last row (canonical): such data is never used, and the
// address stays inside the operand.
LPG_HD int64_t frag_offset_reference(const FragOperand &o, int g0, int ng, int grp, int c, int lane)
{
    if (o.canon) {
        int row = (g0 + grp) * 32 + (lane & 31);
        if (row > o.rows - 1) row = o.rows - 1;
        return (int64_t)row * o.ld + c * o.kf_bytes + (lane >> 5) * 16;
    }
    const int row = (lane & 31) + o.foff;
    int g = grp < ng - 1 ? grp : ng - 1;
    if (g < 0) g = 0;
    const int gmax = (o.foff + o.rows - 1) >> 5;  // last block of the view, counted from its first
    int gsrc = g0 + g + (row >> 5);
    if (gsrc > gmax) gsrc = gmax;
    gsrc -= g0;
    return (int64_t)gsrc * o.gs + (int64_t)(c / kAddrFragsPerBlock) * o.kbs + (c % kAddrFragsPerBlock) * kAddrFragBytes +
           ((lane >> 5) * 32 + (row & 31)) * 16;
}

// Split form, packed operand: offset = frag_uniform_packed(.., hi) + frag_lane_packed(lane),
// hi = frag_lane_hi(lane) in {0, 1} (1: the lane's row lies in the next block of the parent).
LPG_HD int frag_lane_hi(const FragOperand &o, int lane) { return ((lane & 31) + o.foff) >> 5; }

LPG_HD int frag_lane_packed(const FragOperand &o, int lane)
{
    return ((lane >> 5) * 32 + (((lane & 31) + o.foff) & 31)) * 16;
}

LPG_HD int64_t frag_uniform_packed(const FragOperand &o, int g0, int ng, int grp, int c, int hi)
{
    int g = grp < ng - 1 ? grp : ng - 1;
    if (g < 0) g = 0;
    const int gmax = (o.foff + o.rows - 1) >> 5;
    int gsrc = g0 + g + hi;
    if (gsrc > gmax) gsrc = gmax;
    gsrc -= g0;
    return (int64_t)gsrc * o.gs + (int64_t)(c / kAddrFragsPerBlock) * o.kbs + (c % kAddrFragsPerBlock) * kAddrFragBytes;
}

// Split form, canonical operand, valid when the whole group lies inside the operand
// (frag_group_inside): offset = frag_uniform_canon(..) + frag_lane_canon(lane).
LPG_HD bool frag_group_inside(const FragOperand &o, int g0, int grp) { return (g0 + grp) * 32 + 31 <= o.rows - 1; }

LPG_HD int64_t frag_lane_canon(const FragOperand &o, int lane) { return (int64_t)(lane & 31) * o.ld + (lane >> 5) * 16; }

LPG_HD int64_t frag_uniform_canon(const FragOperand &o, int g0, int grp, int c)
{
    return (int64_t)((g0 + grp) * 32) * o.ld + c * o.kf_bytes;
}

}  // namespace lpg
