"""GPU parity of whole chains (lpg_chain) against the oracle's workloads, and of the
propagated mode against the canonical-layout control.

Acceptance per stage s of a chain (fp32: 1e-5, bf16 inputs: 2e-2, relative Frobenius):
  stage-local  - the oracle GEMM fed with the device's own previous intermediate;
  end-to-end   - the fp64 chain, allowing s times the per-GEMM tolerance.
"""
import numpy as np
import pytest
import torch

from oracle import ref, workloads
from paper_2604_04599_amd import api, chains, inputs
from paper_2604_04599_amd.api import LPG_CHAIN_CANONICAL, LPG_CHAIN_PROPAGATED
from tests.gpu_util import assert_elements_bf16, assert_elements_f32, fetch_slot, spread_rows

pytestmark = pytest.mark.gpu

F32_TOL = 1e-5
BF16_TOL = 2e-2


def build(name, **over):
    inp, shape = inputs.make(name, **over)
    return inp, shape, chains.build(name, inp, shape)


def run_both_modes(ch, out_name):
    ch.run(LPG_CHAIN_PROPAGATED)
    prop = ch.output(out_name).copy()
    ch.outputs[out_name].fill_(float("nan"))
    ch.run(LPG_CHAIN_CANONICAL)
    canon = ch.output(out_name).copy()
    return prop, canon


def test_two_gemm_full_size():
    inp, shape, ch = build("two_gemm")
    prop, canon = run_both_modes(ch, "C2")
    assert np.array_equal(prop.view(np.uint32), canon.view(np.uint32))      # same kernels, pure permutations
    want = workloads.two_gemm(inp)
    c1 = ch.fetch("C1")
    assert ref.rel_frobenius(c1, want["C1"]) <= F32_TOL
    assert ref.rel_frobenius(prop, ref.gemm(c1, inp["B2"])) <= F32_TOL       # stage-local
    assert ref.rel_frobenius(prop, want["C2"]) <= 2 * F32_TOL                # end-to-end


def test_two_gemm_integer_chain_is_bit_exact():
    rng = np.random.default_rng(3)
    n = 96
    inp = {k: rng.integers(-2, 3, (n, n)).astype(np.float32) for k in ("A", "B1", "B2")}
    inp["B2"] = (inp["B2"] * (rng.random((n, n)) < 0.2)).astype(np.float32)
    ch = chains.build("two_gemm", inp, {"n": n})
    ch.run()
    want = ref.gemm(inp["A"], ref.gemm(inp["B1"], inp["B2"]))                # (AB)C == A(BC) exactly
    assert np.abs(want).max() < 2 ** 24
    assert np.array_equal(ch.output("C2").astype(np.float64), want)


@pytest.mark.parametrize("over", [dict(m=160, d=96, h=224), dict()])
def test_mlp(over):
    inp, shape, ch = build("mlp", **over)
    prop, canon = run_both_modes(ch, "Y")
    assert np.array_equal(prop.view(np.uint32), canon.view(np.uint32))
    rows = None if over else np.arange(0, shape["m"], 37)
    want = workloads.mlp(inp, rows=rows)
    sel = slice(None) if rows is None else rows
    h = ch.fetch("H")
    assert ref.rel_frobenius(h[sel], want["H"]) <= F32_TOL
    x = inp["X"][sel]
    local = ref.gemm(h[sel], inp["W2"], 1.0, 1.0, x)
    assert ref.rel_frobenius(prop[sel], local) <= F32_TOL
    assert ref.rel_frobenius(prop[sel], want["Y"]) <= 2 * F32_TOL
    assert_elements_f32(h[sel], want["H"], "H")
    assert_elements_f32(prop[sel], local, "Y")


@pytest.mark.parametrize("over", [dict(heads=3, t=160, dh=64), dict()])
def test_attention(over):
    inp, shape, ch = build("attention", **over)
    prop, canon = run_both_modes(ch, "O")
    assert np.array_equal(prop.view(np.uint32), canon.view(np.uint32))
    if over:
        want = workloads.attention(inp, keep_s=True)
        s = ch.fetch("S")
        for h in range(shape["heads"]):
            assert ref.rel_frobenius(s[h], want["S"][h]) <= F32_TOL
            assert ref.rel_frobenius(prop[h], ref.gemm(s[h], inp["V"][h])) <= F32_TOL
            assert ref.rel_frobenius(prop[h], want["O"][h]) <= 2 * F32_TOL
    else:
        # full size: per GEMM, on rows that fall into every 32-row group of the tiles.  S against the
        # oracle on the inputs; O against the oracle fed with the device's own S (stage-local) and
        # against the fp64 chain (end to end).
        rows = spread_rows(shape["t"], 5)
        heads = [0, 13, 31]
        want = workloads.attention(inp, rows=rows, heads=heads, keep_s=True)
        for h in heads:
            s = fetch_slot(ch, "S", h)
            assert ref.rel_frobenius(s[rows], want["S"][h]) <= F32_TOL, h
            assert_elements_f32(s[rows], want["S"][h], ("S", h))
            local = ref.gemm(s[rows], inp["V"][h])
            assert ref.rel_frobenius(prop[h][rows], local) <= F32_TOL, h
            assert_elements_f32(prop[h][rows], local, ("O", h))
            assert ref.rel_frobenius(prop[h][rows], want["O"][h]) <= 2 * F32_TOL, h
            # columns of S as well (every tile column): all queries against a sample of keys
            cols = spread_rows(shape["t"], 77, 16)
            s_cols = ref.gemm(inp["Q"][h], np.ascontiguousarray(inp["K"][h][cols].T), alpha=shape["dh"] ** -0.5)
            assert_elements_f32(s[:, cols], s_cols, ("S columns", h))


@pytest.mark.parametrize("over", [dict(n=192, depth=5), dict(n=160, depth=8), dict()])
def test_deep_chain(over):
    inp, shape, ch = build("deep_chain", **over)
    prop, canon = run_both_modes(ch, "C")
    assert np.array_equal(prop.view(np.uint32), canon.view(np.uint32))
    depth = shape["depth"]
    rows = None if over else spread_rows(shape["n"], 3)
    cols = None if over else spread_rows(shape["n"], 70, 16)
    sel = slice(None) if rows is None else rows
    want = workloads.deep_chain(inp, rows=rows)
    prev = np.asarray(inp["C0"], dtype=np.float64)
    for i in range(1, depth + 1):
        ci = ch.fetch(f"C{i}")
        local = ref.gemm(prev[sel], inp["B"][i - 1])
        assert ref.rel_frobenius(ci[sel], local) <= F32_TOL, i
        assert_elements_f32(ci[sel], local, f"C{i}")
        assert ref.rel_frobenius(ci[sel], want["C"][i]) <= i * F32_TOL, i
        if cols is not None:
            # sampled columns over all rows: with the row sample, every tile of the output is met
            assert_elements_f32(ci[:, cols], ref.gemm(prev, np.ascontiguousarray(inp["B"][i - 1][:, cols])), f"C{i} columns")
        prev = ci
    assert np.array_equal(prop, ch.fetch(f"C{depth}"))


def _check_decoder(inp, shape, ch, prop, rows, s_heads=None):
    nq, nkv = shape["n_q"], shape["n_kv"]
    dh = shape["hidden"] // nq
    rep = nq // nkv
    sel = slice(None) if rows is None else rows
    want = workloads.decoder_layer(inp, nq, nkv, rows=rows)
    got = {n: ch.fetch(n) for n in ("Q", "K", "V", "O", "attn", "gate", "up", "act")}
    # end-to-end against the fp64 chain
    for n in ("Q", "K", "V", "O", "attn", "gate", "up", "act"):
        g = got[n] if n in ("K", "V") else got[n][sel]
        assert ref.rel_frobenius(g, want[n]) <= BF16_TOL, n
    assert ref.rel_frobenius(prop[sel], want["Y"]) <= BF16_TOL
    # stage-local, per GEMM: the oracle on the device's own (bf16-exact) intermediates, by norm and
    # element by element
    x = np.asarray(inp["X"], dtype=np.float64)
    local = {"Q": ref.gemm(x[sel], inp["Wq"]), "K": ref.gemm(x, inp["Wk"]), "V": ref.gemm(x, inp["Wv"]),
             "attn": ref.gemm(got["O"][sel], inp["Wo"]), "gate": ref.gemm(got["attn"][sel], inp["Wg"]),
             "up": ref.gemm(got["attn"][sel], inp["Wu"]), "act": ref.silu_mul(got["gate"][sel], got["up"][sel])}
    for n, w in local.items():
        g = got[n] if n in ("K", "V") else got[n][sel]
        assert ref.rel_frobenius(g, w) <= BF16_TOL, n
        assert_elements_bf16(g, w, n)
    y_local = ref.gemm(got["act"][sel], inp["Wd"])
    assert ref.rel_frobenius(prop[sel], y_local) <= 1e-5   # fp32 out
    assert_elements_f32(prop[sel], y_local, "Y")
    # the two attention GEMMs per head: S against the oracle on the device's own Q and K, O against
    # the oracle on the device's own S and V
    ridx = np.arange(shape["t"]) if rows is None else rows
    for h in (range(nq) if s_heads is None else s_heads):
        g = h // rep
        s = fetch_slot(ch, "S", h)
        s_ref = ref.gemm(np.ascontiguousarray(got["Q"][ridx, h * dh:(h + 1) * dh]),
                         np.ascontiguousarray(got["K"][:, g * dh:(g + 1) * dh].T), alpha=dh ** -0.5)
        assert ref.rel_frobenius(s[ridx], s_ref) <= BF16_TOL, h
        assert_elements_bf16(s[ridx], s_ref, ("S", h))
        o_ref = ref.gemm(s[ridx], np.ascontiguousarray(got["V"][:, g * dh:(g + 1) * dh]))
        assert ref.rel_frobenius(got["O"][ridx, h * dh:(h + 1) * dh], o_ref) <= BF16_TOL, h
        assert_elements_bf16(got["O"][ridx, h * dh:(h + 1) * dh], o_ref, ("O", h))


def test_decoder_layer_small():
    inp, shape, ch = build("decoder_layer", t=192, hidden=256, n_q=4, n_kv=2, ffn=320)
    prop, canon = run_both_modes(ch, "Y")
    assert np.array_equal(prop.view(np.uint32), canon.view(np.uint32))
    _check_decoder(inp, shape, ch, prop, None)


def test_decoder_layer_full_size_sampled_rows():
    inp, shape, ch = build("decoder_layer")
    prop, canon = run_both_modes(ch, "Y")
    assert np.array_equal(prop.view(np.uint32), canon.view(np.uint32))
    rows = spread_rows(shape["t"], 11)           # 32 rows; K and V are checked whole
    _check_decoder(inp, shape, ch, prop, rows, s_heads=[0, 13, 31])


def test_chain_rejects_mismatched_geometry_on_device_buffers():
    inp, shape, ch = build("two_gemm", n=64)
    bad = list(ch.stages)
    wrong = api.desc(api.LPG_PACKED_A, api.LPG_F32, 64, 64, parent=(128, 64))
    bad[2] = api.stage_gemm(1.0, ch.bufs["C1"][0], wrong, ch.bufs["B2"][0], ch.bufs["B2"][1], 0.0, None,
                            ch.bufs["C2"][0], ch.bufs["C2"][1])
    with pytest.raises(api.LpgError) as e:
        api.lpg_chain(bad)
    assert e.value.code == api.LPG_ELAYOUT
    torch.cuda.synchronize()


@pytest.mark.parametrize("name,over,out", [
    ("two_gemm", dict(n=160), "C2"), ("mlp", dict(m=160, d=96, h=224), "Y"),
    ("attention", dict(heads=3, t=160, dh=64), "O"), ("deep_chain", dict(n=192, depth=5), "C"),
    ("deep_chain", dict(n=160, depth=4), "C"),
    ("decoder_layer", dict(t=192, hidden=256, n_q=4, n_kv=2, ffn=320), "Y"), ("mlp", dict(), "Y")])
def test_fused_initial_and_ending_kernels_give_the_same_bits(name, over, out):
    """The chain whose first GEMM reads the canonical input itself and whose last GEMM writes
    the canonical output itself (no pack / unpack pass) equals the standard chain bit for bit."""
    inp, shape = inputs.make(name, **over)
    std = chains.build(name, inp, shape)
    fus = chains.build(name, inp, shape, fused=True)
    assert len(fus.stages) < len(std.stages)
    std.run()
    fus.run()
    a, b = std.output(out).copy(), fus.output(out).copy()
    if name == "decoder_layer":
        # its fused form also applies SiLU(gate)*up in the up projection's epilogue, which skips
        # one bf16 rounding (of U): close to, not identical with, the standard chain
        assert ref.rel_frobenius(b, a) <= 5e-3
        want = workloads.decoder_layer(inp, shape["n_q"], shape["n_kv"])["Y"]
        assert ref.rel_frobenius(b, want) <= BF16_TOL
    else:
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    # the control mode of a fused chain still agrees with its propagated mode
    fus.outputs[out].fill_(float("nan"))
    fus.run(LPG_CHAIN_CANONICAL)
    assert np.array_equal(fus.output(out).view(np.uint32), b.view(np.uint32))


@pytest.mark.parametrize("dtype", [api.LPG_F32, api.LPG_BF16])
@pytest.mark.parametrize("m,widths", [(70, (33, 100, 65, 17)), (256, (512, 512, 512, 512)), (1000, (1000, 3000, 1000, 300))])
def test_three_gemm_chains_of_unequal_widths(m, widths, dtype):
    """The DNN-style chains of the size sweep (section V): propagated = canonical bit for bit,
    both against the fp64 chain; the fused-boundary form gives the same bits."""
    rng = np.random.default_rng(m + sum(widths))
    x = rng.standard_normal((m, widths[0]), dtype=np.float32)
    ws = [rng.standard_normal((a, b), dtype=np.float32) / np.float32(np.sqrt(a)) for a, b in zip(widths, widths[1:])]
    if dtype == api.LPG_BF16:
        x = inputs._bf16_representable(x)
        ws = [inputs._bf16_representable(w) for w in ws]
    ch = chains.build_linear_chain(x, ws, dtype)
    prop, canon = run_both_modes(ch, "Y")
    assert np.array_equal(prop.view(np.uint32), canon.view(np.uint32))
    tol = F32_TOL if dtype == api.LPG_F32 else BF16_TOL
    assert ref.rel_frobenius(prop, ref.chain(x, ws)) <= 3 * tol
    c2 = ch.fetch("C2")
    assert ref.rel_frobenius(prop, ref.gemm(c2, ws[2])) <= F32_TOL           # last stage, fp32 out, stage-local
    fch = chains.build_linear_chain(x, ws, dtype, fused=True)
    fch.run()
    assert np.array_equal(fch.output("Y").view(np.uint32), prop.view(np.uint32))


@pytest.mark.parametrize("dtype", [api.LPG_F32, api.LPG_BF16])
@pytest.mark.parametrize("m,k,n", [(33, 35, 35), (1, 1, 1), (70, 100, 100)])
def test_elementwise_stage_of_odd_sizes_in_both_modes(m, k, n, dtype):
    """GEMM -> SCALE -> ADD -> GEMM with extents that make the control's tight row-major copies end
    off a 16-byte boundary: both modes run and agree bit for bit, and match the oracle."""
    rng = np.random.default_rng(m + k)
    A = inputs._bf16_representable(rng.standard_normal((m, k), dtype=np.float32))
    B = inputs._bf16_representable(rng.standard_normal((k, n), dtype=np.float32) / np.float32(np.sqrt(k)))
    ch = chains.Chain("odd", {}, 0)
    a_d, c_d = api.desc(api.LPG_PACKED_A, dtype, m, k), api.desc(api.LPG_PACKED_A, dtype, m, n)
    y_d = api.desc(api.LPG_PACKED_A, api.LPG_F32, m, n)
    xa = ch.inputs["A"] = chains.device_array(A)
    _, b_d = ch.pack_weight("B", B, api.LPG_PACKED_B, dtype)
    pa, c1, c2, c3, py = (ch.new_packed(nm, d) for nm, d in (("A", a_d), ("C1", c_d), ("C2", c_d), ("C3", c_d), ("Y", y_d)))
    out = ch.outputs["Y"] = torch.empty((m, n), dtype=torch.float32, device="cuda")
    rm_a, rm_y = api.desc(api.LPG_ROW_MAJOR, api.LPG_F32, m, k), api.desc(api.LPG_ROW_MAJOR, api.LPG_F32, m, n)
    ch.add(api.stage_pack(xa, rm_a, pa, a_d))
    ch.add(api.stage_gemm(1.0, pa, a_d, ch.bufs["B"][0], b_d, 0.0, None, c1, c_d))
    ch.add(api.stage_elementwise(api.LPG_EW_SCALE, c1, None, 0.5, c2, c_d))
    ch.add(api.stage_elementwise(api.LPG_EW_ADD, c1, c2, 2.0, c3, c_d))
    ch.add(api.stage_gemm(1.0, c3, c_d, ch.bufs["B"][0], b_d, 0.0, None, py, y_d))
    ch.add(api.stage_unpack(py, y_d, out, rm_y))
    prop, canon = run_both_modes(ch, "Y")
    assert np.array_equal(prop.view(np.uint32), canon.view(np.uint32))
    want = ref.gemm(2.0 * ref.gemm(A, B), B)
    assert ref.rel_frobenius(prop, want) <= (3 * F32_TOL if dtype == api.LPG_F32 else BF16_TOL)


@pytest.mark.parametrize("name,over,out", [("two_gemm", dict(), "C2"), ("mlp", dict(m=160, d=96, h=224), "Y"),
                                           ("attention", dict(heads=3, t=160, dh=64), "O")])
def test_graph_replay_matches_eager(name, over, out):
    """A chain captured into a HIP graph: every replay, with eager work and synchronisation
    between replays, gives the eager result bit for bit, also after the inputs change."""
    inp, shape, ch = build(name, **over)
    ch.run()
    eager = ch.output(out).copy()
    replay = ch.capture()
    for it in range(4):
        ch.outputs[out].fill_(float("nan"))
        torch.cuda.synchronize()
        replay()
        assert np.array_equal(ch.output(out).view(np.uint32), eager.view(np.uint32)), it
        (torch.ones(1024, device="cuda") * it).sum().item()          # unrelated eager work in between
    # new input values in the same buffers: the graph reads them, and matches a fresh eager run
    first = next(iter(ch.inputs.values()))
    first.mul_(0.5)
    replay()
    got = ch.output(out).copy()
    ch.run()
    assert np.array_equal(ch.output(out).view(np.uint32), got.view(np.uint32))
    canon_replay = ch.capture(LPG_CHAIN_CANONICAL)
    ch.outputs[out].fill_(float("nan"))
    canon_replay()
    assert np.array_equal(ch.output(out).view(np.uint32), got.view(np.uint32))
