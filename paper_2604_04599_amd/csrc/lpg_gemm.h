// The MFMA GEMM kernel (main loop + layout-writing epilogue) and its launchers.  Included by
// one translation unit per dtype pair (lpg_gemm_*.hip), which instantiates every tile
// configuration for that pair.
#pragma once

#include "lpg_device.h"
#include "lpg_tiles.h"

namespace lpg {

// ---------------------------------------------------------------------------------
// GEMM.  out[fl][fr] = epilogue(alpha * sum_k L[fl][k] * R[fr][k] + beta * Cin[fl][fr]),
// L = P(L; FL, K), R = P(R; FR, K), out = P(out; free = FL, contraction = FR).
//
// The MFMA computes a 32x32 tile D[i][j] = sum_k Aop[i][k] * Bop[k][j]; lane l of the
// A operand carries row i = l%32, lane l of the B operand carries column j = l%32, and
// lane l, register r of D holds D[8*(r/4) + 4*(l/32) + r%4][l%32].  With R's fragment
// in the A slot and L's fragment in the B slot, lanes run along out's free index and
// each group of four registers is four consecutive contraction indices of out: the
// accumulators already are fragments of P(out; FL, FR) and are stored as they stand.
//
// Workgroup tile: TLG x TRG 32-groups; WL x WR waves, each owning (TLG/WL) x (TRG/WR)
// 32x32 tiles.  A step stages FS fragments per group (FS = 4: a whole K block, FS = 2:
// half of one) into one of NS LDS stages used as a ring; NS-1 steps are in flight ahead of
// the one being multiplied.  The packed block already is the register image, so the copy
// is verbatim: each wave moves whole 1 KiB fragments with the direct global->LDS load (no
// VGPR round trip), and every ds_read_b128 at lane*16 is conflict free.
//
// Workgroups are persistent: workgroup j walks the virtual tile ids j, j + G, j + 2G, ...
// (G = grid size) and the staging ring runs across tile boundaries, so the next tile's
// first steps are in flight while the current tile's epilogue stores drain.  Every
// workgroup runs a fixed, finite number of steps; there is no queue and no atomics.

// registers -> fragments of P(out; FL, FR) for one 32x32 accumulator tile
template <typename OUT>
__device__ __forceinline__ void store_tile(const GemmArgs &p, const f32x16 &acc, int grL, int grR, int lane,
                                           char *Ob, const char *Cb, const char *Eb, bool use_c, bool use_e)
{
    const int h = lane >> 5;
    const int fl = grL * 32 + (lane & 31);
    const bool have = grR < p.FRg;
    float v[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) v[e] = have ? acc[e] : 0.0f;
    if (p.alpha != 1.0f) {
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e] *= p.alpha;
    }
    if (p.o_canon) {
        // Ending kernel: straight to row/column-major.  Lanes run along out's free index, so
        // for each register the 32 lanes of a half wave write one contiguous run.  The same
        // element-by-element walk serves a packed out whose origin is off the grid.
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int fr = grR * 32 + 8 * (e >> 2) + 4 * h + (e & 3);
            if (fl >= p.FL || fr >= p.FR) continue;
            int64_t off;
            if (p.o_canon == 2) {
                // packed out with its origin off the grid: the element's own position in the
                // parent's blocks, o_foff / o_koff further along than in an aligned view
                const int fp = fl + p.o_foff, kp = fr + p.o_koff;
                const int kin = kp % OUT::KB, r = kin % OUT::KF;
                off = (int64_t)(kp / OUT::KB) * p.o_kbs + (int64_t)(fp >> 5) * p.o_gs + (kin / OUT::KF) * kFragBytes +
                      (((r >> 2) & 1) * 32 + (fp & 31)) * 16 + (4 * (r >> 3) + (r & 3)) * OUT::ES;
            } else {
                off = (int64_t)fl * p.o_sf + (int64_t)fr * p.o_sk;
            }
            float x = v[e];
            if (use_c) {
                if constexpr (OUT::ES == 4) x = __builtin_fmaf(p.beta, *(const float *)(Cb + off), x);
                else x = __builtin_fmaf(p.beta, bf16_to_f32(*(const uint16_t *)(Cb + off)), x);
            }
            float gte = 0.0f;
            if (use_e) {
                if constexpr (OUT::ES == 4) gte = *(const float *)(Eb + off);
                else gte = bf16_to_f32(*(const uint16_t *)(Eb + off));
            }
            x = epi_apply(p.epi, x, gte);
            if constexpr (OUT::ES == 4) *(float *)(Ob + off) = x;
            else *(uint16_t *)(Ob + off) = (uint16_t)bf16_rne(x);
        }
        return;
    }
    int64_t obase;  // byte offset of this tile's first fragment inside out
    if constexpr (OUT::ES == 4)
        obase = (int64_t)grR * p.o_kbs + (int64_t)grL * p.o_gs + lane * 16;
    else
        obase = (int64_t)(grR >> 1) * p.o_kbs + (int64_t)grL * p.o_gs + (grR & 1) * 2 * kFragBytes + lane * 16;
    constexpr int NF = (OUT::ES == 4) ? 4 : 2;  // fragments this tile spans
    constexpr int PER = 16 / NF;
    if (use_c || use_e) {
#pragma unroll
        for (int fgi = 0; fgi < NF; ++fgi) {
            float cv[PER], ev[PER];
            if (use_c) {
                const uint4 t4 = *(const uint4 *)(Cb + obase + fgi * kFragBytes);
                const uint32_t w[4] = {t4.x, t4.y, t4.z, t4.w};
#pragma unroll
                for (int j = 0; j < PER; ++j) {
                    if constexpr (OUT::ES == 4) cv[j] = __uint_as_float(w[j]);
                    else cv[j] = bf16_to_f32((w[j >> 1] >> (16 * (j & 1))) & 0xffff);
                }
            }
            if (use_e) {
                const uint4 t4 = *(const uint4 *)(Eb + obase + fgi * kFragBytes);
                const uint32_t w[4] = {t4.x, t4.y, t4.z, t4.w};
#pragma unroll
                for (int j = 0; j < PER; ++j) {
                    if constexpr (OUT::ES == 4) ev[j] = __uint_as_float(w[j]);
                    else ev[j] = bf16_to_f32((w[j >> 1] >> (16 * (j & 1))) & 0xffff);
                }
            }
#pragma unroll
            for (int j = 0; j < PER; ++j) {
                float x = v[fgi * PER + j];
                if (use_c) x = __builtin_fmaf(p.beta, cv[j], x);
                v[fgi * PER + j] = epi_apply(p.epi, x, use_e ? ev[j] : 0.0f);
            }
        }
    } else if (p.epi == LPG_EPI_SILU) {
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e] = silu_f(v[e]);
    }
    // zero the padding of ragged edge tiles
    if (grL * 32 + 32 > p.FL || grR * 32 + 32 > p.FR) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int fr = grR * 32 + 8 * (e >> 2) + 4 * h + (e & 3);
            if (fl >= p.FL || fr >= p.FR) v[e] = 0.0f;
        }
        if (p.o_keep_l | p.o_keep_r) {
            // the view's ragged extent ends inside its parent: what lies past it in this tile
            // belongs to the parent's other elements and is left as it is
            const bool l_mine = fl < p.FL || !p.o_keep_l;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int fr = grR * 32 + 8 * (e >> 2) + 4 * h + (e & 3);
                if (!l_mine || (fr >= p.FR && p.o_keep_r)) continue;
                char *dst = Ob + obase + (e / PER) * kFragBytes + (e % PER) * OUT::ES;
                if constexpr (OUT::ES == 4) *(float *)dst = v[e];
                else *(uint16_t *)dst = (uint16_t)bf16_rne(v[e]);
            }
            return;
        }
    }
    if constexpr (OUT::ES == 4) {
#pragma unroll
        for (int fgi = 0; fgi < 4; ++fgi)
            *(uint4 *)(Ob + obase + fgi * kFragBytes) =
                make_uint4(__float_as_uint(v[4 * fgi]), __float_as_uint(v[4 * fgi + 1]),
                           __float_as_uint(v[4 * fgi + 2]), __float_as_uint(v[4 * fgi + 3]));
    } else {
#pragma unroll
        for (int fgi = 0; fgi < 2; ++fgi) {
            uint32_t w[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) w[j] = bf16_pack2(v[8 * fgi + 2 * j], v[8 * fgi + 2 * j + 1]);
            *(uint4 *)(Ob + obase + fgi * kFragBytes) = make_uint4(w[0], w[1], w[2], w[3]);
        }
    }
}

// The common case of store_tile, kept small: packed output, no C_in, no fused operation, a
// tile wholly inside the logical extents.  The epilogue is instantiated once per accumulator
// tile of the wave; with only the general form, a launch of many short tiles (attention
// scores) spends its time fetching that code.
// 16 bytes of a packed fragment as floats (4 fp32 or 8 bf16 elements)
template <typename OUT>
__device__ __forceinline__ void frag_vals(const char *ptr, float (&x)[16 / OUT::ES])
{
    const uint4 t = *(const uint4 *)ptr;
    const uint32_t w[4] = {t.x, t.y, t.z, t.w};
    if constexpr (OUT::ES == 4) {
#pragma unroll
        for (int j = 0; j < 4; ++j) x[j] = __uint_as_float(w[j]);
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) x[j] = bf16_to_f32((w[j >> 1] >> (16 * (j & 1))) & 0xffff);
    }
}

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
// NT: streaming stores (the output is far larger than the caches and is not read again soon)
template <typename OUT, bool USE_C, int EPI, bool NT = false>
__device__ __forceinline__ void store_tile_plain(const GemmArgs &p, const f32x16 &acc, int grL, int grR, int lane, char *Ob,
                                                 const char *Cb, const char *Eb)
{
    constexpr int NF = (OUT::ES == 4) ? 4 : 2, PER = 16 / NF;
    int64_t off;
    if constexpr (OUT::ES == 4) off = (int64_t)grR * p.o_kbs + (int64_t)grL * p.o_gs + lane * 16;
    else off = (int64_t)(grR >> 1) * p.o_kbs + (int64_t)grL * p.o_gs + (grR & 1) * 2 * kFragBytes + lane * 16;
#pragma unroll
    for (int fgi = 0; fgi < NF; ++fgi) {
        float v[PER];
#pragma unroll
        for (int j = 0; j < PER; ++j) v[j] = acc[fgi * PER + j] * p.alpha;
        if constexpr (USE_C) {
            float c[PER];
            frag_vals<OUT>(Cb + off + fgi * kFragBytes, c);
#pragma unroll
            for (int j = 0; j < PER; ++j) v[j] = __builtin_fmaf(p.beta, c[j], v[j]);
        }
        if constexpr (EPI == LPG_EPI_SILU) {
#pragma unroll
            for (int j = 0; j < PER; ++j) v[j] = silu_f(v[j]);
        } else if constexpr (EPI == LPG_EPI_GATE_SILU) {
            float g[PER];
            frag_vals<OUT>(Eb + off + fgi * kFragBytes, g);
#pragma unroll
            for (int j = 0; j < PER; ++j) v[j] = silu_f(g[j]) * v[j];
        }
        u32x4_t w;
        if constexpr (OUT::ES == 4) {
            w = u32x4_t{__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])};
        } else {
            w = u32x4_t{bf16_pack2(v[0], v[1]), bf16_pack2(v[2], v[3]), bf16_pack2(v[4], v[5]), bf16_pack2(v[6], v[7])};
        }
        if constexpr (NT) __builtin_nontemporal_store(w, (u32x4_t *)(Ob + off + fgi * kFragBytes));
        else *(u32x4_t *)(Ob + off + fgi * kFragBytes) = w;
    }
}

// The same for a row- or column-major output (Ending kernel), interior tiles, no C_in, no
// fused operation: lanes run along out's free index, so for each register the 32 lanes of a
// half wave write one contiguous run.
template <typename OUT>
__device__ __forceinline__ void store_tile_canon_plain(const GemmArgs &p, const f32x16 &acc, int grL, int grR, int lane, char *Ob)
{
    const int h = lane >> 5;
    char *o = Ob + (int64_t)(grL * 32 + (lane & 31)) * p.o_sf + (int64_t)(grR * 32 + 4 * h) * p.o_sk;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        char *dst = o + (int64_t)(8 * (e >> 2) + (e & 3)) * p.o_sk;
        const float x = acc[e] * p.alpha;
        if constexpr (OUT::ES == 4) *(float *)dst = x;
        else *(uint16_t *)dst = (uint16_t)bf16_rne(x);
    }
}

// virtual block id -> (batch, tile).  Hardware deals consecutive workgroups round-robin
// to the 8 XCDs; ids congruent mod 8 get one contiguous range of tile ids, walked in
// bands of GM tile-rows, so the tiles an XCD works on share L and R panels in its L2.
template <int TLG, int TRG>
__device__ __forceinline__ TileInfo decode_tile(const GemmArgs &p, uint32_t vb, uint32_t total, uint32_t ntile)
{
    const uint32_t per = total / 8, rem = total % 8, x = vb % 8, idx = vb / 8;
    const uint32_t pid = (x < rem) ? x * (per + 1) + idx : rem * (per + 1) + (x - rem) * per + idx;
    TileInfo t;
    int tl, tr;
    tile_at(p.walk, pid, t.b, tl, tr);
    t.gl0 = tl * TLG;
    t.gr0 = tr * TRG;
    t.nlg = min(TLG, p.FLg - t.gl0);
    t.nrg = max(0, min(TRG, p.FRg - t.gr0));
    // packed: first block of the tile; canonical: the operand's (slot's) first element
    t.Lp = p.L + (int64_t)div_by((uint32_t)t.b, p.by_ldiv) * p.l_slot + (p.l_canon ? 0 : (int64_t)t.gl0 * p.l_gs);
    t.Rp = p.R + (int64_t)div_by((uint32_t)t.b, p.by_rdiv) * p.r_slot + (p.r_canon ? 0 : (int64_t)t.gr0 * p.r_gs);
    return t;
}

// The epilogue of one workgroup tile: every accumulator tile of the wave goes out through the
// compact form that fits (tiles wholly inside the logical extents) or the general one.  All forms
// round alike (v = alpha * acc, then one fused multiply-add with beta * C_in), so an element's
// value does not depend on the tile configuration that happened to compute it.
template <typename OUT, int TLG, int TRG, int WTL, int WTR>
__device__ __forceinline__ void write_tiles(const GemmArgs &p, f32x16 (&acc)[WTL][WTR], const TileInfo &cur, int wl, int wr,
                                            int lane, bool use_c, bool use_e)
{
    const int64_t oslot = (int64_t)cur.b * p.o_slot;
    // compact forms for tiles wholly inside the logical extents; 0: general form
    const bool interior = (cur.gl0 + TLG) * 32 <= p.FL && (cur.gr0 + TRG) * 32 <= p.FR;
    int form = 0;
    if (interior && !p.o_canon) {
        if (p.epi == LPG_EPI_NONE) form = use_c ? 2 : 1;
        else if (!use_c) form = (p.epi == LPG_EPI_SILU) ? 3 : (use_e ? 4 : 0);
    } else if (p.o_canon == 1 && interior && !use_c && p.epi == LPG_EPI_NONE) {
        form = 5;
    }
#define LPG_EPILOGUE_FORM(CALL)                                                                    \
static_for<WTL * WTR>([&](auto I) {                                                            \
    constexpr int a = decltype(I)::value / WTR, q = decltype(I)::value % WTR;                  \
    const int grL = cur.gl0 + wl * WTL + a, grR = cur.gr0 + wr * WTR + q;                      \
    CALL;                                                                                      \
})
    char *Oo = p.Out + oslot;
    if (form == 1 && p.o_stream) {
        LPG_EPILOGUE_FORM((store_tile_plain<OUT, false, LPG_EPI_NONE, true>(p, acc[a][q], grL, grR, lane, Oo, nullptr, nullptr)));
    } else if (form == 1) {
        LPG_EPILOGUE_FORM((store_tile_plain<OUT, false, LPG_EPI_NONE>(p, acc[a][q], grL, grR, lane, Oo, nullptr, nullptr)));
    } else if (form == 2) {
        LPG_EPILOGUE_FORM((store_tile_plain<OUT, true, LPG_EPI_NONE>(p, acc[a][q], grL, grR, lane, Oo, p.Cin + oslot, nullptr)));
    } else if (form == 3) {
        LPG_EPILOGUE_FORM((store_tile_plain<OUT, false, LPG_EPI_SILU>(p, acc[a][q], grL, grR, lane, Oo, nullptr, nullptr)));
    } else if (form == 4) {
        LPG_EPILOGUE_FORM((store_tile_plain<OUT, false, LPG_EPI_GATE_SILU>(p, acc[a][q], grL, grR, lane, Oo, nullptr, p.Epi + oslot)));
    } else if (form == 5) {
        LPG_EPILOGUE_FORM((store_tile_canon_plain<OUT>(p, acc[a][q], grL, grR, lane, Oo)));
#undef LPG_EPILOGUE_FORM
    } else {
        static_for<WTL * WTR>([&](auto I) {
            constexpr int a = decltype(I)::value / WTR, q = decltype(I)::value % WTR;
            const int grL = cur.gl0 + wl * WTL + a;
            const int grR = cur.gr0 + wr * WTR + q;
            if (grL < p.FLg && grR < p.FRg_out)
                store_tile<OUT>(p, acc[a][q], grL, grR, lane, p.Out + oslot, p.Cin + oslot, p.Epi + oslot, use_c,
                                use_e);
        });
    }
}

// XPF (needs NS >= 3): the first fragment of the NEXT step is read into registers while the
// last fragment of the current step is multiplied, so no LDS latency is exposed after the
// barrier; the barrier of a step then also publishes the step after it.
template <typename IN, typename OUT, int TLG, int TRG, int WL, int WR, int FS, int NS, bool XPF>
__global__ __launch_bounds__(WL *WR * 64, ((TLG / WL) * (TRG / WR) >= 8 ? 2 : 1)) void gemm_kernel(GemmArgs p)
{
    static_assert(!XPF || NS >= 3, "cross-step prefetch needs a landed stage beyond the current one");
    constexpr int DEPTH = NS - 1;  // steps the copy side runs ahead of the multiply side
    constexpr bool kSplitLoops = TLG * TRG >= 16;  // split step loops (below) in the kernels of tiles of 128 x 128 elements and more
    constexpr int NW = WL * WR;
    constexpr int WTL = TLG / WL, WTR = TRG / WR;
    constexpr int NFRAG = (TLG + TRG) * FS;  // fragments per stage
    constexpr int FPW = NFRAG / NW;          // fragments each wave copies per stage
    constexpr int FPW_L = TLG * FS / NW;     // ... of which the first FPW_L come from L
    constexpr int STAGE = NFRAG * kFragBytes;
    constexpr int BPS = FS > kFragsPerBlock ? FS / kFragsPerBlock : 1;  // K blocks per step
    static_assert(NFRAG % NW == 0 && (TLG * FS) % NW == 0, "stage must divide over the waves");
    static_assert(TLG % WL == 0 && TRG % WR == 0, "tile must divide over the waves");
    static_assert(FS == 2 || FS == 4 || FS == 8, "a step is half a K block, one, or two");
    static_assert(NS >= 2 && NS <= 5 && (NS - 2) * FPW <= 63, "ring depth limited by the vmcnt field");
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const uint32_t sbase = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)smem;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wl = wave % WL, wr = wave / WL;

    const uint32_t ntile = (uint32_t)(p.walk.tiles_l * p.walk.tiles_r);
    const uint32_t total = ntile * (uint32_t)p.batch;
    const uint32_t G = gridDim.x;
    const int spt = FS > kFragsPerBlock ? p.nkb / BPS : p.nkb * (kFragsPerBlock / FS);  // steps per tile (launcher: BPS divides nkb)
    if (blockIdx.x >= total) return;
    const uint32_t my_tiles = (total - blockIdx.x + G - 1) / G;

    auto decode = [&](uint32_t vb) __attribute__((always_inline)) -> TileInfo { return decode_tile<TLG, TRG>(p, vb, total, ntile); };

    // ---- copy side.  Wave w copies fragments w, w + NW, ... of a stage; src[i] is this
    // lane's address of its i-th fragment at the step the copy cursor stands on.  Every wave
    // always issues exactly FPW transfers per step, so outstanding-transfer counts agree
    // across waves: a group the tile does not have is replaced by the tile's last existing
    // group (its data is never used), which keeps every address inside the operand.
    const char *src[FPW];
    // The two operands as the fragment fetch sees them (lpg_addr.h).  A source address is a
    // wave-uniform part (which group, K block and fragment: scalar arithmetic) plus a part
    // that depends on the lane alone and is the same for all fragments of an operand.
    const FragOperand opL = {p.l_canon, p.l_foff, p.FL, p.l_gs, p.l_kbs, p.l_ld, IN::KF * IN::ES};
    const FragOperand opR = {p.r_canon, p.r_foff, p.FR, p.r_gs, p.r_kbs, p.r_ld, IN::KF * IN::ES};
    auto aim = [&](const TileInfo &t) __attribute__((always_inline)) {
        // per-lane parts, once per tile and operand
        const int64_t laneL = p.l_canon ? frag_lane_canon(opL, lane) : (int64_t)frag_lane_packed(opL, lane);
        const int64_t laneR = p.r_canon ? frag_lane_canon(opR, lane) : (int64_t)frag_lane_packed(opR, lane);
        const bool hiL = frag_lane_hi(opL, lane) != 0, hiR = frag_lane_hi(opR, lane) != 0;
        static_for<FPW>([&](auto I) {
            constexpr int i = decltype(I)::value;
            constexpr bool is_l = i < FPW_L;
            const int fid = i * NW + wave;
            const int c = fid % FS;
            const int grp = is_l ? fid / FS : fid / FS - TLG;  // group of the tile, in its operand
            const int g0 = is_l ? t.gl0 : t.gr0, ng = is_l ? t.nlg : t.nrg;
            const char *base = is_l ? t.Lp : t.Rp;
            const int64_t lane_part = is_l ? laneL : laneR;
            const bool canon = is_l ? p.l_canon != 0 : p.r_canon != 0;
            const int foff = is_l ? p.l_foff : p.r_foff;
            if (canon) {
                // Initial kernel: the fragment comes straight from the canonical matrix.  Lane
                // (fl, h) of fragment c needs k = KF*c + 4*h .. +3 of free index fl: 16 contiguous
                // bytes of a k-contiguous fp32 row, which the transfer drops at lane*16 of the
                // stage, i.e. in fragment order.  A group that ends past the operand's last row
                // takes the per-lane form, which replaces the missing rows by the last one.
                if (frag_group_inside(is_l ? opL : opR, g0, grp)) src[i] = base + frag_uniform_canon(is_l ? opL : opR, g0, grp, c) + lane_part;
                else src[i] = base + frag_offset_reference(is_l ? opL : opR, g0, ng, grp, c, lane);
            } else {
                // A view whose free-dimension origin is foff rows off the 32-grid: view row v of a
                // group is parent row v + foff, i.e. lane slot (v + foff) % 32 of this block or of
                // the next one.  The transfer takes a source address per lane, so the shift costs
                // one select per fragment: each lane fetches its 16 bytes from where they are and
                // drops them at lane * 16.
                const int64_t u0 = frag_uniform_packed(is_l ? opL : opR, g0, ng, grp, c, 0);
                if (foff == 0) {
                    src[i] = base + u0 + lane_part;
                } else {
                    const int64_t u1 = frag_uniform_packed(is_l ? opL : opR, g0, ng, grp, c, 1);
                    src[i] = base + ((is_l ? hiL : hiR) ? u1 : u0) + lane_part;
                }
            }
        });
    };
    uint32_t c_tiles_left = my_tiles;  // tiles the copy cursor still has to start or finish
    uint32_t c_vb = blockIdx.x;
    int c_s = 0;                       // step of its tile the copy cursor stands on
    int c_st = 0;                      // ring stage it fills next
    int pending = 0;                   // steps copied (or in flight) and not yet multiplied
    bool c_live = spt > 0;
    // fragment i of the step the copy cursor stands on -> ring stage c_st
    auto copy_issue = [&](int i) __attribute__((always_inline)) {
        // The ring stage is the same for all lanes; taking it through readfirstlane keeps the address computation of
        // the transfers off the scalar unit's critical path (measured: 4096^3 fp32 957 -> 932 us).
        lds_dma16(src[i], __builtin_amdgcn_readfirstlane(sbase + c_st * STAGE + (i * NW + wave) * kFragBytes));
    };
    // Address increments of a step inside a tile, fixed for the launch.  Whole K blocks per step:
    // one increment; half blocks: from the first half of a block to its second half (d*_in), and
    // from there to the first half of the next block (d*_out).  Canonical rows are contiguous along k.
    const int64_t dl_in = p.l_canon ? FS * IN::KF * IN::ES : (FS >= kFragsPerBlock ? BPS * p.l_kbs : (int64_t)FS * kFragBytes);
    const int64_t dr_in = p.r_canon ? FS * IN::KF * IN::ES : (FS >= kFragsPerBlock ? BPS * p.r_kbs : (int64_t)FS * kFragBytes);
    const int64_t dl_out = (p.l_canon || FS >= kFragsPerBlock) ? dl_in : p.l_kbs - (kFragsPerBlock - FS) * kFragBytes;
    const int64_t dr_out = (p.r_canon || FS >= kFragsPerBlock) ? dr_in : p.r_kbs - (kFragsPerBlock - FS) * kFragBytes;
    // Move the copy cursor one step on: inside its tile (FPW additions), or on to its next tile
    // (tile decode, fresh addresses).
    auto advance_in_tile = [&]() __attribute__((always_inline)) {
        c_st = (c_st + 1 == NS) ? 0 : c_st + 1;
        ++pending;
        ++c_s;
        const bool leaving = (c_s & 1) == 0;  // (half-block steps) the step just copied was a block's second half
        const int64_t dl = leaving ? dl_out : dl_in, dr = leaving ? dr_out : dr_in;
#pragma unroll
        for (int i = 0; i < FPW; ++i) src[i] += (i < FPW_L) ? dl : dr;
    };
    auto advance_to_next_tile = [&]() __attribute__((always_inline)) {
        c_st = (c_st + 1 == NS) ? 0 : c_st + 1;
        ++pending;
        c_s = 0;
        c_vb += G;
        if (--c_tiles_left == 0) c_live = false;
        else aim(decode(c_vb));
    };
    auto copy_advance = [&]() __attribute__((always_inline)) {
        if (c_s + 1 == spt) advance_to_next_tile();
        else advance_in_tile();
    };
    auto copy_step = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < FPW; ++i) copy_issue(i);
        copy_advance();
    };
    aim(decode(c_vb));
#pragma unroll
    for (int j = 0; j < DEPTH; ++j)
        if (c_live) copy_step();

    const bool use_c = (p.beta != 0.0f) && p.Cin;
    const bool use_e = (p.epi == LPG_EPI_GATE_SILU) && p.Epi;

    // ---- multiply side
    int st = 0;
    const char *sLw = smem + (wl * WTL) * (FS * kFragBytes) + lane * 16;
    const char *sRw = smem + (TLG + wr * WTR) * (FS * kFragBytes) + lane * 16;
    uint4 lf[2][WTL], rf[2][WTR];
    if constexpr (XPF) {
        // prime: fragment 0 of the very first step
        if (pending == NS - 1) wait_vmcnt<(NS - 2) * FPW>();
        else wait_vmcnt<0>();
        __syncthreads();
#pragma unroll
        for (int a = 0; a < WTL; ++a) lf[0][a] = *(const uint4 *)(sLw + a * (FS * kFragBytes));
#pragma unroll
        for (int q = 0; q < WTR; ++q) rf[0][q] = *(const uint4 *)(sRw + q * (FS * kFragBytes));
    }
    uint32_t vb = blockIdx.x;
    for (uint32_t ti = 0; ti < my_tiles; ++ti, vb += G) {
        f32x16 acc[WTL][WTR];
#pragma unroll
        for (int a = 0; a < WTL; ++a)
#pragma unroll
            for (int q = 0; q < WTR; ++q)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[a][q][e] = 0.0f;

        // One step of the tile.  ADV says where the copy cursor goes after it: 0 = wherever it must
        // (the general case), 1 = on inside its tile, 2 = to its next tile.
        auto step = [&](const int ADV) __attribute__((always_inline)) {
            // Wait until this wave's transfers of the step that must be readable have landed
            // (XPF: the step after the current one; otherwise the current one); later steps
            // stay in flight (transfers complete in issue order).
            constexpr int KEEP = XPF ? NS - 3 : NS - 2;
            if (pending == NS - 1) wait_vmcnt<KEEP * FPW>();
            else wait_vmcnt<0>();
            __syncthreads();  // everyone's transfers landed; the stage multiplied last step is free

            const char *sL = sLw + st * STAGE;
            const char *sR = sRw + st * STAGE;
            const int stn = (st + 1 == NS) ? 0 : st + 1;
            if constexpr (!XPF) {
#pragma unroll
                for (int a = 0; a < WTL; ++a) lf[0][a] = *(const uint4 *)(sL + a * (FS * kFragBytes));
#pragma unroll
                for (int q = 0; q < WTR; ++q) rf[0][q] = *(const uint4 *)(sR + q * (FS * kFragBytes));
            }
            // The step is cut into FS*WTL phases (one row of the wave's tiles each).  A phase
            // reads its share of the NEXT fragment from LDS, multiplies one row of the current
            // fragment, and issues its share of this step's global->LDS transfers, so that
            // neither LDS reads nor transfer issue ever pile up in front of the MFMAs.  After
            // the last real step the transfers go on as harmless refills of the one ring
            // stage nobody reads again (their sources stay valid), which keeps this loop free
            // of branches.
            // A fragment is J MFMAs deep (fp32: four k-pairs, bf16: one); the k-pairs are the
            // outer loop so that consecutive MFMAs go to different accumulators and a tile's
            // accumulator comes round again only after all the wave's other tiles.
            constexpr int J = mma_depth<IN>();
            constexpr int SLOTS = FS * J * WTL;
            // With two stages the transfers issued during this step are awaited at the start of
            // the next one, so the last of them has only the rest of this step to land: they go
            // out during the first half of the step's phases (the stage they fill was released by
            // the barrier above).  Measured against an even spread over the whole step: bf16 gate /
            // up projections 3-5 % faster, down projection 5-7 %, Q / O projections 3-4 %, fp32
            // unchanged (its steps are long enough either way); all of them in the first quarter
            // is slower again.  Deeper rings have slack and keep the even spread.
            constexpr int ISLOTS = NS == 2 ? SLOTS / 2 : SLOTS;
            static_assert(ISLOTS >= 1, "issue window inside the step");
#pragma unroll
            for (int c = 0; c < FS; ++c) {
                const int cb = c & 1, nb = (c + 1) & 1;
                const bool more = c + 1 < FS;
                const char *nL = more ? sL + (c + 1) * kFragBytes : sLw + stn * STAGE;
                const char *nR = more ? sR + (c + 1) * kFragBytes : sRw + stn * STAGE;
#pragma unroll
                for (int j = 0; j < J; ++j) {
#pragma unroll
                    for (int a = 0; a < WTL; ++a) {
                        if (j == 0 && (more || XPF)) {
                            lf[nb][a] = *(const uint4 *)(nL + a * (FS * kFragBytes));
                            if (a < WTR) rf[nb][a] = *(const uint4 *)(nR + a * (FS * kFragBytes));
                            if (a == WTL - 1) {
#pragma unroll
                                for (int q = WTL; q < WTR; ++q) rf[nb][q] = *(const uint4 *)(nR + q * (FS * kFragBytes));
                            }
                        }
#pragma unroll
                        for (int q = 0; q < WTR; ++q) mma_part<IN>(acc[a][q], rf[cb][q], lf[cb][a], j);
                        const int slot = (c * J + j) * WTL + a;
                        if (slot < ISLOTS) {
#pragma unroll
                            for (int i = (slot * FPW) / ISLOTS; i < ((slot + 1) * FPW) / ISLOTS; ++i) copy_issue(i);
                        }
                        // fp32: one fence per k-pair round (a round already touches every accumulator
                        // once); bf16: one per row of tiles
                        if (J == 1 || a == WTL - 1) __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
            st = stn;
            --pending;
            if (c_live) {
                if (ADV == 0) copy_advance();
                else if (ADV == 1) advance_in_tile();
                else advance_to_next_tile();
            }
        };
        if (kSplitLoops && spt > DEPTH) {
            // The copy cursor runs DEPTH steps ahead, so with more than DEPTH steps per tile it leaves
            // this tile exactly once, after step spt - DEPTH - 1.  That step stands alone between two
            // loops whose own cursor movement is a handful of additions: the tile decode and the
            // fresh addresses are then not part of any loop body.
            // The kernels of smaller tiles keep the one general loop: they serve small launches,
            // which spend their time fetching code, and three loop bodies instead of one cost
            // 256^3 .. 1024^3 products about a microsecond.
            int s = 0;
            for (; s < spt - DEPTH - 1; ++s) step(1);
            step(2);
            for (++s; s < spt; ++s) step(1);
        } else {
            for (int s = 0; s < spt; ++s) step(0);
        }

        // ---- epilogue
        write_tiles<OUT, TLG, TRG, WTL, WTR>(p, acc, decode(vb), wl, wr, lane, use_c, use_e);
    }
    wait_vmcnt<0>();  // no transfer into this workgroup's LDS may outlive the wave
}

template <typename IN, typename OUT, int TLG, int TRG, int WL, int WR, int NS, int FSX = 0>
static hipError_t launch_gemm_ring(const GemmArgs &a, int64_t grid, hipStream_t st)
{
    constexpr int NT = WL * WR * 64;
    constexpr bool BF = IN::ES == 2;
    constexpr int FS = FSX ? FSX : ring_fs(BF);
    constexpr size_t lds = (size_t)NS * (TLG + TRG) * FS * kFragBytes;
    static_assert(lds <= 160 * 1024, "ring does not fit the LDS");
    auto kern = gemm_kernel<IN, OUT, TLG, TRG, WL, WR, FS, NS, (BF && NS >= 3)>;
    if (lds > (size_t)device_info().lds_bytes) return hipErrorInvalidConfiguration;
    if (lds > 64 * 1024) {
        static PerDeviceFlag raised;  // per instantiation
        if (first_use_on_device(raised)) {
            hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            mark_used_on_device(raised);
        }
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(NT), lds, st, a);
    return hipGetLastError();
}

template <typename IN, typename OUT, int TLG, int TRG, int WL, int WR>
static hipError_t launch_gemm_cfg(GemmArgs a, hipStream_t st)
{
    constexpr bool BF = IN::ES == 2;
    constexpr int NS = ring_ns(BF, TLG, TRG, WL * WR), NS_LONE = BF ? NS : ring_ns_lone(TLG, TRG);
    a.walk.tiles_l = (a.FLg + TLG - 1) / TLG;
    a.walk.tiles_r = (a.FRg_out + TRG - 1) / TRG;
    const int64_t total = (int64_t)a.walk.tiles_l * a.walk.tiles_r * a.batch;
    if (total <= 0) return hipSuccess;
    if (total > 0x7fffffff) return hipErrorInvalidValue;  // the kernel counts tiles in 32 bits
    const TileCfg c = {TLG, TRG, WL, WR};
    const int ncu = device_info().ncu;
    int64_t grid = (int64_t)ncu * workgroups_per_cu(c, BF);
    if (grid > total) grid = total;
    // Band height of the tile walk.  An XCD works on a contiguous range of tile ids, gm tile rows x
    // (range / gm) tile columns at a time, and fetches gm row panels and range / gm column panels
    // into its L2: take the height that makes the sum of their bytes smallest.
    {
        const int64_t range = (grid < total ? grid : total) / 8 > 0 ? (grid < total ? grid : total) / 8 : 1;
        int best = 8;
        int64_t best_cost = -1;
        for (int gm : {8, 4, 2, 16}) {
            const int64_t rows = gm < a.walk.tiles_l ? gm : a.walk.tiles_l;
            const int64_t cols = (range + rows - 1) / rows < a.walk.tiles_r ? (range + rows - 1) / rows : a.walk.tiles_r;
            const int64_t cost = rows * TLG + cols * TRG;
            if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = gm; }
        }
        const int force = tune_get(LPG_TUNE_BAND);
        a.walk = tile_walk_setup(a.walk.tiles_l, a.walk.tiles_r, force > 0 ? force : best);
        a.by_ldiv = div_setup((uint32_t)(a.l_div > 0 ? a.l_div : 1));
        a.by_rdiv = div_setup((uint32_t)(a.r_div > 0 ? a.r_div : 1));
    }
    {
        // An output larger than the memory-side cache that nothing reads back soon (attention scores)
        // is written with streaming stores: 3-5 % on 32 heads of 2048^2 fp32 scores, nothing lost
        // elsewhere.
        const int force = tune_get(LPG_TUNE_STREAM_STORES);
        const int64_t out_bytes = (int64_t)a.FL * a.FR * a.batch * OUT::ES;
        a.o_stream = force < 0 ? out_bytes >= ((int64_t)256 << 20) : force > 0;
    }
    if constexpr (NS_LONE != NS) {
        if (total <= ncu) {
            // Small lone tiles: a step of one K block is 2048-4096 MFMA cycles and every step ends
            // at a workgroup barrier that costs about 290 of them (no second wave on the SIMD to
            // fill the gap), so an even number of K blocks is walked two per step.
            constexpr int STAGE2 = (TLG + TRG) * 8 * kFragBytes;
            constexpr int NS2 = 4 * STAGE2 <= 160 * 1024 ? 4 : (3 * STAGE2 <= 160 * 1024 ? 3 : 2);
            if constexpr (!BF && TLG * TRG <= 16) {
                if (tune_get(LPG_TUNE_TWO_BLOCK_STEPS) != 0 && a.nkb % 2 == 0 && a.nkb >= 4)
                    return launch_gemm_ring<IN, OUT, TLG, TRG, WL, WR, NS2, 8>(a, grid, st);
            }
            return launch_gemm_ring<IN, OUT, TLG, TRG, WL, WR, NS_LONE>(a, grid, st);
        }
    }
    if constexpr (BF && TLG * TRG <= 8) {
        // bf16, small lone tiles: a half-block step is 64-256 MFMA cycles, far less than the
        // barrier that ends it; two whole K blocks per step (four times fewer barriers), in as
        // many stages as the LDS holds (the next-step prefetch needs three).
        constexpr int STAGE2 = (TLG + TRG) * 8 * kFragBytes;
        constexpr int NS2 = 5 * STAGE2 <= 160 * 1024 ? 5 : (4 * STAGE2 <= 160 * 1024 ? 4 : 3);
        static_assert(NS2 * STAGE2 <= 160 * 1024, "two-block stages of the small tiles fit three times");
        if (tune_get(LPG_TUNE_TWO_BLOCK_STEPS) != 0 && total <= ncu && a.nkb % 2 == 0 && a.nkb >= 4)
            return launch_gemm_ring<IN, OUT, TLG, TRG, WL, WR, NS2, 8>(a, grid, st);
    }
    if constexpr (BF && TLG * TRG >= 8 && TLG * TRG <= 16 && WL * WR == 4) {
        // bf16 tiles of 128 x 64 to 128 x 128 (several workgroups per compute unit): whole K
        // blocks per step in two stages, without the next-step prefetch, instead of half blocks
        // in four stages with it: half the barriers in the same LDS; measured 2-8 % faster on
        // 2048^3, 4096 x 2048 x 2048, 16384 x 1024 x 1024 and ragged shapes.  The tuning hook
        // LPG_TUNE_BF16_WHOLE_BLOCK_STEPS = 0 restores the half-block ring.
        if (tune_get(LPG_TUNE_BF16_WHOLE_BLOCK_STEPS) != 0) return launch_gemm_ring<IN, OUT, TLG, TRG, WL, WR, 2, 4>(a, grid, st);
    }
    if constexpr (BF && TLG == 8 && TRG == 8) {
        // bf16, 256 x 256 (eight waves, the whole compute unit): whole K blocks in two stages of
        // 64 KiB as well, half as many barriers as the ring of five half-block stages: 2-3 % on the
        // gate / up projections (4096 x 2048 x 8192).  LPG_TUNE_BF16_WHOLE_BLOCK_STEPS = 0: the ring.
        if (tune_get(LPG_TUNE_BF16_WHOLE_BLOCK_STEPS) != 0) return launch_gemm_ring<IN, OUT, TLG, TRG, WL, WR, 2, 4>(a, grid, st);
    }
    return launch_gemm_ring<IN, OUT, TLG, TRG, WL, WR, NS>(a, grid, st);
}


// ---------------------------------------------------------------------------------
// The general GEMM kernel: the Initial kernel of section III-A.1 for ANY operand.  The main kernel
// copies fragments verbatim (packed operands on the block grid, k-contiguous fp32 canonical ones);
// everything else - canonical matrices contiguous along the free index (a row-major weight B[k x n]),
// bf16 canonical matrices, fp32 canonical matrices feeding a bf16 product (rounded to nearest even on
// the way, exactly as lpg_pack would), contractions of any length (the tail reads as zero), views of
// packed parents with any origin and any extent - goes through registers here: every thread fetches
// the elements of its lane vectors of the next K block (vector loads where the source is contiguous
// along k and aligned) while the current block is multiplied, then converts them, writes the vectors
// to the LDS, and the multiply side and the epilogue are the main kernel's.  One K block per step, two LDS stages, 128 x 128 tiles, 4 waves of 2 x 2.
// The per-accumulator order of the sums is the main kernel's, so results are bit-identical to
// lpg_pack followed by the packed product.

// How an operand's lane vectors are fetched (GatherOperand::mode, chosen on the host).  All loads of a
// K block are issued first and land in raw registers while the current block is multiplied; they are
// converted and packed into lane vectors only when they go to the LDS.
enum { kGatherElem = 0,     // canonical, element by element (lanes run along the free index)
       kGatherVec32 = 1,    // canonical fp32, contiguous along k, 16-byte aligned rows, K a multiple of 4
       kGatherVec16 = 2,    // canonical bf16, contiguous along k, 8-byte aligned rows, K a multiple of 4
       kGatherPacked = 3 }; // view of a packed parent, element by element through the closed-form position

// One lane vector as fetched: KV dwords.  Element modes: one element per dword (fp32 bits, or a bf16
// pattern in the low half).  kGatherVec32: the dwords of the 16-byte loads.  kGatherVec16: dwords
// 2u, 2u+1 hold run u's four bf16 values.
template <typename IN>
struct RawVector {
    uint32_t w[IN::KV];
};

// Lane (fl, h) of fragment c of K block kb of 32-group g holds k = KB*kb + KF*c + 8*u + 4*h + j
// (u < KV/4 runs of j < 4 consecutive k) of free index 32*g + fl.
template <typename IN>
__device__ __forceinline__ void gather_fetch(RawVector<IN> &raw, const GatherOperand &o, const char *base, int g, int kb, int c,
                                             int lane)
{
    const int f = g * 32 + (lane & 31), h = lane >> 5;
    const int k0 = kb * IN::KB + c * IN::KF + 4 * h;
    constexpr int RUNS = IN::KV / 4;
    const bool row_in = f < o.F;
#pragma unroll
    for (int v = 0; v < IN::KV; ++v) raw.w[v] = 0;
    if (o.mode == kGatherVec32) {
#pragma unroll
        for (int u = 0; u < RUNS; ++u) {
            const int k = k0 + 8 * u;
            if (row_in && k < o.K) {   // K is a multiple of 4: the run is inside or outside as a whole
                const uint4 q = *(const uint4 *)(base + (int64_t)f * o.sf + (int64_t)k * 4);
                raw.w[4 * u] = q.x; raw.w[4 * u + 1] = q.y; raw.w[4 * u + 2] = q.z; raw.w[4 * u + 3] = q.w;
            }
        }
    } else if (o.mode == kGatherVec16) {
        if constexpr (IN::ES == 2) {
#pragma unroll
            for (int u = 0; u < RUNS; ++u) {
                const int k = k0 + 8 * u;
                if (row_in && k < o.K) {
                    const uint2 q = *(const uint2 *)(base + (int64_t)f * o.sf + (int64_t)k * 2);
                    raw.w[2 * u] = q.x; raw.w[2 * u + 1] = q.y;
                }
            }
        }
    } else if (o.mode == kGatherPacked) {
#pragma unroll
        for (int v = 0; v < IN::KV; ++v) {
            const int k = k0 + 8 * (v >> 2) + (v & 3);
            if (row_in && k < o.K) {
                const int fp = f + o.foff, kp = k + o.koff;
                const int kin = kp % IN::KB, r = kin % IN::KF;
                const int64_t off = (int64_t)(kp / IN::KB) * o.kbs + (int64_t)(fp >> 5) * o.gs + (kin / IN::KF) * kFragBytes +
                                    (((r >> 2) & 1) * 32 + (fp & 31)) * 16 + (4 * (r >> 3) + (r & 3)) * IN::ES;
                raw.w[v] = *(const typename IN::raw *)(base + off);
            }
        }
    } else {
#pragma unroll
        for (int v = 0; v < IN::KV; ++v) {
            const int k = k0 + 8 * (v >> 2) + (v & 3);
            if (row_in && k < o.K) {
                const char *ptr = base + (int64_t)f * o.sf + (int64_t)k * o.sk;
                raw.w[v] = o.es == 4 ? *(const uint32_t *)ptr : (uint32_t) * (const uint16_t *)ptr;
            }
        }
    }
}

// raw registers -> the 16-byte lane vector of the type the GEMM multiplies (fp32 sources of a bf16
// product are rounded to nearest even here, exactly as lpg_pack rounds)
template <typename IN>
__device__ __forceinline__ uint4 gather_finish(const RawVector<IN> &raw, const GatherOperand &o)
{
    if constexpr (IN::ES == 4) {
        return make_uint4(raw.w[0], raw.w[1], raw.w[2], raw.w[3]);   // fp32 sources only (checked on the host)
    } else {
        uint32_t e[8];
        if (o.mode == kGatherVec16) {
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                e[4 * u] = raw.w[2 * u] & 0xffff; e[4 * u + 1] = raw.w[2 * u] >> 16;
                e[4 * u + 2] = raw.w[2 * u + 1] & 0xffff; e[4 * u + 3] = raw.w[2 * u + 1] >> 16;
            }
        } else if (o.mode != kGatherPacked && o.es == 4) {
#pragma unroll
            for (int v = 0; v < 8; ++v) e[v] = bf16_rne(__uint_as_float(raw.w[v]));
        } else {
#pragma unroll
            for (int v = 0; v < 8; ++v) e[v] = raw.w[v] & 0xffff;
        }
        return make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
    }
}

template <typename IN, typename OUT>
__global__ __launch_bounds__(256) void gemm_gather_kernel(GatherArgs ga)
{
    constexpr int TLG = 4, TRG = 4, WL = 2, NW = 4, WTL = 2, WTR = 2;   // 2 x 2 waves of 2 x 2 tiles
    constexpr int FS = kFragsPerBlock;                 // one K block per step
    constexpr int NFRAG = (TLG + TRG) * FS;
    constexpr int STAGE = NFRAG * kFragBytes;
    static_assert(FS == NW, "wave w builds fragment w of every 32-group");
    const GemmArgs &p = ga.g;
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wl = wave % WL, wr = wave / WL;
    const uint32_t ntile = (uint32_t)(p.walk.tiles_l * p.walk.tiles_r);
    const uint32_t total = ntile * (uint32_t)p.batch;
    const bool use_c = (p.beta != 0.0f) && p.Cin;
    const bool use_e = (p.epi == LPG_EPI_GATE_SILU) && p.Epi;

    for (uint32_t vb = blockIdx.x; vb < total; vb += gridDim.x) {
        const TileInfo t = decode_tile<TLG, TRG>(p, vb, total, ntile);
        const char *lbase = ga.l.base + (int64_t)(t.b / ga.l.div) * ga.l.slot;
        const char *rbase = ga.r.base + (int64_t)(t.b / ga.r.div) * ga.r.slot;
        // wave w builds fragment c = w of every 32-group of the stage: groups 0 .. TLG-1 of L, then R's
        RawVector<IN> rawl[TLG], rawr[TRG];
        auto fetch = [&](int kb) {
#pragma unroll
            for (int i = 0; i < TLG; ++i) gather_fetch<IN>(rawl[i], ga.l, lbase, t.gl0 + i, kb, wave, lane);
#pragma unroll
            for (int i = 0; i < TRG; ++i) gather_fetch<IN>(rawr[i], ga.r, rbase, t.gr0 + i, kb, wave, lane);
        };
        auto deposit = [&](int stage) {
            char *dst = smem + stage * STAGE + wave * kFragBytes + lane * 16;
#pragma unroll
            for (int i = 0; i < TLG; ++i) *(uint4 *)(dst + i * (FS * kFragBytes)) = gather_finish<IN>(rawl[i], ga.l);
#pragma unroll
            for (int i = 0; i < TRG; ++i) *(uint4 *)(dst + (TLG + i) * (FS * kFragBytes)) = gather_finish<IN>(rawr[i], ga.r);
        };
        f32x16 acc[WTL][WTR];
#pragma unroll
        for (int a = 0; a < WTL; ++a)
#pragma unroll
            for (int q = 0; q < WTR; ++q)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[a][q][e] = 0.0f;

        if (p.nkb > 0) {
            fetch(0);
            __syncthreads();   // the previous tile's last stage has been read by everyone
            deposit(0);
            __syncthreads();
        }
        for (int s = 0; s < p.nkb; ++s) {
            const bool more = s + 1 < p.nkb;
            if (more) fetch(s + 1);     // in flight while this step is multiplied
            const char *sL = smem + (s & 1) * STAGE + (wl * WTL) * (FS * kFragBytes) + lane * 16;
            const char *sR = smem + (s & 1) * STAGE + (TLG + wr * WTR) * (FS * kFragBytes) + lane * 16;
            constexpr int J = mma_depth<IN>();
#pragma unroll
            for (int c = 0; c < FS; ++c) {
                uint4 lf[WTL], rf[WTR];
#pragma unroll
                for (int a = 0; a < WTL; ++a) lf[a] = *(const uint4 *)(sL + a * (FS * kFragBytes) + c * kFragBytes);
#pragma unroll
                for (int q = 0; q < WTR; ++q) rf[q] = *(const uint4 *)(sR + q * (FS * kFragBytes) + c * kFragBytes);
#pragma unroll
                for (int j = 0; j < J; ++j)
#pragma unroll
                    for (int a = 0; a < WTL; ++a)
#pragma unroll
                        for (int q = 0; q < WTR; ++q) mma_part<IN>(acc[a][q], rf[q], lf[a], j);
            }
            if (more) deposit((s + 1) & 1);   // that stage was last read in step s - 1
            __syncthreads();
        }
        write_tiles<OUT, TLG, TRG, WTL, WTR>(p, acc, t, wl, wr, lane, use_c, use_e);
    }
}

template <typename IN, typename OUT>
static hipError_t launch_gemm_gather_dtype(GatherArgs ga, hipStream_t st)
{
    GemmArgs &a = ga.g;
    constexpr int TLG = 4, TRG = 4;
    a.walk.tiles_l = (a.FLg + TLG - 1) / TLG;
    a.walk.tiles_r = (a.FRg_out + TRG - 1) / TRG;
    const int64_t total = (int64_t)a.walk.tiles_l * a.walk.tiles_r * a.batch;
    if (total <= 0) return hipSuccess;
    if (total > 0x7fffffff) return hipErrorInvalidValue;
    a.walk = tile_walk_setup(a.walk.tiles_l, a.walk.tiles_r, 8);
    a.by_ldiv = div_setup((uint32_t)(a.l_div > 0 ? a.l_div : 1));
    a.by_rdiv = div_setup((uint32_t)(a.r_div > 0 ? a.r_div : 1));
    a.o_stream = 0;
    constexpr size_t lds = 2 * (size_t)(TLG + TRG) * kFragsPerBlock * kFragBytes;   // 64 KiB
    int64_t grid = (int64_t)device_info().ncu * 2;
    if (grid > total) grid = total;
    hipLaunchKernelGGL((gemm_gather_kernel<IN, OUT>), dim3((unsigned)grid), dim3(256), lds, st, ga);
    return hipGetLastError();
}

template <typename IN, typename OUT>
static hipError_t launch_gemm_dtype(const GemmArgs &a, int cfg, hipStream_t st)
{
    switch (cfg) {
        case 0: return launch_gemm_cfg<IN, OUT, 2, 2, 2, 2>(a, st);
        case 1: return launch_gemm_cfg<IN, OUT, 4, 2, 2, 2>(a, st);
        case 2: return launch_gemm_cfg<IN, OUT, 2, 4, 2, 2>(a, st);
        case 3: return launch_gemm_cfg<IN, OUT, 4, 4, 2, 2>(a, st);
        case 4: return launch_gemm_cfg<IN, OUT, 8, 4, 2, 2>(a, st);
        case 5: return launch_gemm_cfg<IN, OUT, 4, 8, 2, 2>(a, st);
        case 6: return launch_gemm_cfg<IN, OUT, 8, 8, 2, 4>(a, st);
        case 7: return launch_gemm_cfg<IN, OUT, 8, 2, 4, 1>(a, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace lpg
