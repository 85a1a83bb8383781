"""The allocation-free variant of the stand-alone importance reduction against the allocating entry point."""
import numpy as np
import pytest
import torch

from paper_2602_06822_amd import synth

from gpu_util import dev, host

pytestmark = pytest.mark.gpu


def test_importance_reduce_static_matches_allocating_entry_point():
    """Two calls in a row through the C ABI, the second with a smaller input (fewer tokens, fewer channels, the
    other dtype): the static-scratch variant must reproduce pop_importance_reduce bit for bit, whatever the
    earlier call left in the shared array; sizes beyond its limit are rejected."""
    assert torch.cuda.is_available(), "this test needs the MI355X"
    from paper_2602_06822_amd import binding as pop
    g = synth.rng("no_alloc")
    for T, m, dtype in ((1500, 11008, synth.F32), (77, 1000, synth.BF16), (1, 3, synth.F32)):
        H = g.standard_normal((T, m), dtype=np.float32)
        H[:, ::53] *= np.float32(100.0)
        nrm = np.abs(g.standard_normal(m, dtype=np.float32)) + np.float32(0.1)
        Hd = dev(H if dtype == synth.F32 else synth.f32_to_bf16_bits(H))
        nd = dev(nrm)
        ref = torch.full((m,), -1.0, dtype=torch.float32, device="cuda")
        out = torch.full((m,), -2.0, dtype=torch.float32, device="cuda")
        pop.pop_importance_reduce(Hd, dtype, T, m, nd, ref)
        pop.pop_importance_reduce_static(Hd, dtype, T, m, nd, out)
        assert np.array_equal(host(out), host(ref)), (T, m, dtype)
        assert np.all(host(out) > 0)
    with pytest.raises(pop.PopError) as e:
        big = torch.zeros((1, 40000), dtype=torch.float32, device="cuda")
        pop.pop_importance_reduce_static(big, synth.F32, 1, 40000, big, big)
    assert e.value.status == pop.POP_EUNSUPPORTED
