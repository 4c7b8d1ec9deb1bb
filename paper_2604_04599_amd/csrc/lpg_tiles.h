// Tile configurations of the MFMA GEMM kernel and what the host needs to know of them (LDS
// ring sizes, workgroups per compute unit): shared by the kernel's translation units and by
// the cost model that picks a configuration.
#pragma once

#include "lpg_internal.h"

namespace lpg {

// Tile configurations (TLG, TRG, WL, WR) in 32-groups; index = position in this list.
struct TileCfg {
    int tlg, trg, wl, wr;
};
static const TileCfg kCfgs[] = {
    {2, 2, 2, 2},  // 0:  64 x  64, 4 waves of 1x1
    {4, 2, 2, 2},  // 1: 128 x  64, 4 waves of 2x1
    {2, 4, 2, 2},  // 2:  64 x 128, 4 waves of 1x2
    {4, 4, 2, 2},  // 3: 128 x 128, 4 waves of 2x2
    {8, 4, 2, 2},  // 4: 256 x 128, 4 waves of 4x2
    {4, 8, 2, 2},  // 5: 128 x 256, 4 waves of 2x4
    {8, 8, 2, 4},  // 6: 256 x 256, 8 waves of 4x2
    {8, 2, 4, 1},  // 7: 256 x  64, 4 waves of 2x2
};
constexpr int kNumCfgs = sizeof(kCfgs) / sizeof(kCfgs[0]);

// Staging ring per input type and tile: fp32 moves whole K blocks through two stages (its
// MFMAs are slow enough to cover memory latency); bf16 moves half blocks through a ring of
// four stages (three where four would keep a second workgroup off the compute unit) and
// reads the next step's first fragment ahead.
constexpr int ring_fs(bool bf16) { return bf16 ? 2 : 4; }
constexpr int ring_ns(bool bf16, int tlg, int trg, int nw)
{
    if (!bf16) return 2;
    const int stage = (tlg + trg) * 2 * kFragBytes;
    if (nw == 8) return 5 * stage <= 160 * 1024 ? 5 : 4;  // one workgroup per compute unit: use all the LDS
    return 4 * stage <= 80 * 1024 ? 4 : 3;
}

// fp32 with small tiles and no more tiles than compute units: a step's MFMAs (2048 cycles
// for a 128 x 64 tile) are shorter than the memory latency under load, and no second
// workgroup shares the compute unit to cover for it, so the ring is made deeper instead: as
// deep as the whole LDS allows, the lone workgroup has it to itself.
constexpr int ring_ns_lone(int tlg, int trg)
{
    const int stage = (tlg + trg) * 4 * kFragBytes;
    return 4 * stage <= 160 * 1024 ? 4 : (3 * stage <= 160 * 1024 ? 3 : 2);
}

static int lds_bytes(const TileCfg &c, bool bf16)
{
    return ring_ns(bf16, c.tlg, c.trg, c.wl * c.wr) * (c.tlg + c.trg) * ring_fs(bf16) * kFragBytes;
}

static int workgroups_per_cu(const TileCfg &c, bool bf16)
{
    int occ = device_info().lds_bytes / lds_bytes(c, bf16);
    const int waves = c.wl * c.wr;
    // accumulators + operand registers per lane decide how many waves fit a SIMD
    const int regs = (c.tlg / c.wl) * (c.trg / c.wr) * 16 + 64;
    const int waves_per_simd = regs > 256 ? 1 : (regs > 128 ? 2 : 4);
    const int by_regs = waves_per_simd * 4 / waves;
    if (occ > by_regs) occ = by_regs;
    if (occ > 4) occ = 4;
    return occ < 1 ? 1 : occ;
}

}  // namespace lpg
