"""Pin for the oracle's fp32 -> bf16 rounding: exhaustive over all upper halves
against the definition of round-to-nearest, ties-to-even, evaluated with exact
fp64 arithmetic (every fp32 and the midpoint between bf16 neighbours is exact in fp64)."""
import numpy as np

from oracle import ref


def _definition(bits):
    bits = bits.astype(np.uint64)
    lo = bits & 0xFFFF0000
    low16 = bits & 0xFFFF
    hi = lo + 0x10000                       # next bf16 away from zero (sign-magnitude)
    # exact distances in units of the dropped field: low16 vs 0x10000 - low16
    up = (low16 > 0x8000) | ((low16 == 0x8000) & (((lo >> 16) & 1) == 1))
    return np.where(up, hi, lo) >> 16


def test_exhaustive_upper_halves():
    uppers = np.arange(1 << 16, dtype=np.uint64) << 16
    lowers = np.array([0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF], dtype=np.uint64)
    bits = (uppers[:, None] | lowers[None, :]).ravel()
    exp_all_ones = (bits & 0x7F800000) == 0x7F800000
    finite = ~exp_all_ones
    got = ref.bf16_bits(bits.astype(np.uint32)).astype(np.uint64)
    want = _definition(bits)
    assert np.array_equal(got[finite], want[finite] & 0xFFFF)
    # the integer rule above is itself checked against real-number distances
    x = bits[finite].astype(np.uint32).view(np.float32).astype(np.float64)
    chosen = (got[finite].astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    lo = (bits[finite] & 0xFFFF0000).astype(np.uint32).view(np.float32).astype(np.float64)
    hi_bits = ((bits[finite] & 0xFFFF0000) + 0x10000).astype(np.uint32)
    hi_is_inf = (hi_bits & 0x7FFFFFFF) == 0x7F800000
    hi = hi_bits.view(np.float32).astype(np.float64)
    # unbounded-exponent value of the upper neighbour where the pattern says infinity
    hi = np.where(hi_is_inf, lo * (1 + 2.0 ** -7 / (1 + 127 * 2.0 ** -7)), hi)
    ch = np.where(np.isinf(chosen), hi, chosen)
    assert np.all(np.abs(ch - x) <= np.minimum(np.abs(lo - x), np.abs(hi - x)))
    # infinities stay, NaNs stay NaN
    inf = exp_all_ones & ((bits & 0x007FFFFF) == 0)
    assert np.array_equal(got[inf], bits[inf] >> 16)
    nan = exp_all_ones & ~inf
    g = got[nan]
    assert np.all((g & 0x7F80) == 0x7F80) and np.all((g & 0x007F) != 0)


def test_round_arrays():
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -1.0 - 2.0 ** -8, 3.14159, 1e-3])
    r = ref.round_bf16(x)
    assert r[0] == 1.0
    assert r[1] == 1.0                         # tie -> even mantissa (1.0)
    assert r[2] == 1.0 + 2.0 ** -6             # tie -> even mantissa (1 + 2/128)
    assert r[3] == -1.0
    assert abs(r[4] - 3.14159) <= 2.0 ** -7    # half ulp at exponent 1 (ulp = 2^-6)
    assert np.array_equal(ref.round_bf16(r), r)
    f = ref.round_f32(np.array([0.1, 1.0 + 2.0 ** -30]))
    assert f[0] == float(np.float32(0.1)) and f[1] == 1.0


def test_bf16_workload_inputs_are_rounded_to_nearest_even():
    """The bf16 workloads draw fp32 values and round them once (nearest, ties to even) before
    either side sees them: the generator's rounding equals the oracle's, ties included."""
    from paper_2604_04599_amd import inputs
    rng = np.random.default_rng(3)
    x = rng.standard_normal(50000).astype(np.float32)
    ties = (np.arange(0x3F80, 0x3F90, dtype=np.uint32) << 16 | 0x8000).view(np.float32)      # exact halves
    x = np.concatenate([x, ties, -ties])
    y = inputs._bf16_representable(x)
    assert np.array_equal(y.astype(np.float64), ref.round_bf16(x.astype(np.float64)))
    assert np.all(y.view(np.uint32) & 0xFFFF == 0)
    inp, _ = inputs.make("decoder_layer", t=64, hidden=64, n_q=1, n_kv=1, ffn=64)
    for v in inp.values():
        assert np.all(v.view(np.uint32) & 0xFFFF == 0)
