"""lpg_chain_static, the entry point for callers that cannot allocate: the canonical-layout
control chain with its row-major copies in the library's static device scratch instead of a
caller's workspace.  Checked through the C ABI against lpg_chain (same kernels: bit-identical)
and against the oracle, on calls in a row of which the later ones are smaller, so that whatever
an earlier call left in the shared scratch is still there."""
import numpy as np
import pytest
import torch

from oracle import ref, workloads
from paper_2604_04599_amd import api, chains, inputs
from paper_2604_04599_amd.api import LPG_CHAIN_CANONICAL, LPG_CHAIN_PROPAGATED

pytestmark = pytest.mark.gpu


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _both(name, over, out, **options):
    """The workload through lpg_chain (caller's workspace) and through lpg_chain_static."""
    inp, shape = inputs.make(name, **over)
    ch = chains.build(name, inp, shape, **options)
    need = api.lpg_chain_workspace_bytes(ch.stage_array(), LPG_CHAIN_CANONICAL)
    assert 0 < need <= api.LPG_STATIC_SCRATCH_BYTES
    ch.run(LPG_CHAIN_CANONICAL)
    want = ch.output(out).copy()
    ch.outputs[out].fill_(float("nan"))
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    api.lpg_chain_static(ch.stage_array(), LPG_CHAIN_CANONICAL, _stream())
    torch.cuda.synchronize()
    free1 = torch.cuda.mem_get_info()[0]
    got = ch.output(out).copy()
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), (name, over)
    return inp, shape, got, free0 - free1


def test_two_calls_in_a_row_the_second_smaller():
    # first call: intermediates of 8 MiB in the scratch; second: a ragged, much smaller chain that
    # reuses the start of the same scratch; third: the first shape again
    inp, shape, y, _ = _both("mlp", dict(m=512, d=256, h=1024), "Y")
    assert ref.rel_frobenius(y, workloads.mlp(inp)["Y"]) <= 2e-5
    inp, shape, y, grew = _both("mlp", dict(m=160, d=96, h=224), "Y")
    assert ref.rel_frobenius(y, workloads.mlp(inp)["Y"]) <= 2e-5
    assert grew == 0                                    # the call took no device memory
    inp, shape, y, grew = _both("mlp", dict(m=512, d=256, h=1024), "Y")
    assert ref.rel_frobenius(y, workloads.mlp(inp)["Y"]) <= 2e-5
    assert grew == 0


def test_batched_heads_with_a_softmax_stage_then_a_smaller_bf16_layer():
    inp, shape, o, _ = _both("attention", dict(heads=3, t=160, dh=64), "O", softmax=True, causal=True)
    want = workloads.attention(inp, softmax=True, causal=True)
    for h in range(shape["heads"]):
        assert ref.rel_frobenius(o[h], want["O"][h]) <= 2e-5
    inp, shape, y, grew = _both("decoder_layer", dict(t=128, hidden=128, n_q=2, n_kv=1, ffn=192), "Y")
    assert ref.rel_frobenius(y, workloads.decoder_layer(inp, 2, 1)["Y"]) <= 2e-2
    assert grew == 0


def test_propagated_mode_needs_no_scratch():
    inp, shape = inputs.make("two_gemm", n=160)
    ch = chains.build("two_gemm", inp, shape)
    api.lpg_chain_static(ch.stage_array(), LPG_CHAIN_PROPAGATED, _stream())
    got = ch.output("C2").copy()
    ch.outputs["C2"].fill_(float("nan"))
    ch.run(LPG_CHAIN_PROPAGATED)
    assert np.array_equal(got.view(np.uint32), ch.output("C2").view(np.uint32))
    assert ref.rel_frobenius(got, workloads.two_gemm(inp)["C2"]) <= 2e-5


def test_a_chain_past_the_scratch_size_is_refused_before_any_launch():
    inp, shape = inputs.make("mlp", m=4096, d=1024, h=8192)          # H alone is 128 MiB row-major
    ch = chains.build("mlp", inp, shape)
    assert api.lpg_chain_workspace_bytes(ch.stage_array(), LPG_CHAIN_CANONICAL) > api.LPG_STATIC_SCRATCH_BYTES
    ch.outputs["Y"].fill_(123.0)
    with pytest.raises(api.LpgError) as e:
        api.lpg_chain_static(ch.stage_array(), LPG_CHAIN_CANONICAL, _stream())
    assert e.value.code == api.LPG_EWORKSPACE
    assert "static scratch" in str(e.value)
    assert np.all(ch.output("Y") == 123.0)                            # nothing ran
