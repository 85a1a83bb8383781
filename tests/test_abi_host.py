"""Host-only checks of the C-ABI library: it loads, exports every symbol the header declares, and its
host-side integer logic agrees with the oracle.  No GPU work is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "pop.h")
LIB = os.path.join(ROOT, "paper_2602_06822_amd", "libpop_hip.so")


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pop_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2602_06822_amd import build
        build.build_hip()
    return ctypes.CDLL(LIB)


def test_header_declares_the_three_entry_points():
    names = _declared_functions()
    for need in ("pop_prefill_partition", "pop_decode_mask", "pop_pruned_ffn"):
        assert need in names


def test_library_exports_every_declared_symbol(lib):
    names = _declared_functions()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), f"{n} declared in pop.h but not exported"


def test_binding_covers_every_declared_symbol(lib):
    from paper_2602_06822_amd import binding
    assert sorted(binding.EXPORTED) == _declared_functions()
    for n in binding.EXPORTED:
        assert callable(getattr(binding, n))


def test_host_logic_matches_oracle(lib, oracle):
    from paper_2602_06822_amd import binding as pop
    assert pop.pop_version() >= 100
    for m in (1, 2, 7, 333, 1376, 11008, 13824, 14336):
        for fr, fc in ((0.0, 0.0), (0.3, 0.4), (0.6, 0.1), (0.75, 0.1), (0.45, 0.1), (0.0, 1.0), (1.0, 0.0),
                       (0.55, 0.2), (0.625, 0.05)):
            got = pop.pop_region_counts(m, fr, fc)
            assert got == oracle.region_counts(m, fr, fc)
            for r in (0.0, 0.2, 0.35, 0.5, 0.9, 1.0):
                assert pop.pop_k_for_ratio(m, r, got[0], got[1]) == oracle.k_for_ratio(m, r, got[0], got[1])
    with pytest.raises(pop.PopError):
        pop.pop_region_counts(10, 0.8, 0.3)
    with pytest.raises(pop.PopError):
        pop.pop_region_counts(0, 0.3, 0.3)
    with pytest.raises(pop.PopError):
        pop.pop_k_for_ratio(10, 1.5, 3, 3)
    assert pop.pop_strerror(0) == "ok" and "order" in pop.pop_strerror(pop.POP_ESTATE)


def test_strategy_counts(lib, oracle):
    """Region sizes of the ablation's decode strategies: the method's band from the oracle's count rules, the static
    prefill mask as "everything active is retained", full re-scoring as "everything is a candidate"; all three keep
    the same number of active channels per token."""
    from paper_2602_06822_amd import binding as pop
    for m in (7, 1376, 11008, 14336):
        for r in (0.2, 0.35, 0.5):
            a = int(np.floor((1.0 - r) * m + 0.5))
            for gamma in (0.05, 0.1, 0.2):
                n_ret, n_cand, k = pop.pop_strategy_counts(pop.POP_STRATEGY_POP, m, r, gamma)
                assert (n_ret, n_cand) == oracle.region_counts(m, 1.0 - r - gamma / 2, gamma)[:2]
                assert k == oracle.k_for_ratio(m, r, n_ret, n_cand)
                if n_cand >= 2:
                    assert n_ret + k == a
            assert pop.pop_strategy_counts(pop.POP_STRATEGY_STATIC_MASK, m, r, 0.1) == (a, 0, 0)
            assert pop.pop_strategy_counts(pop.POP_STRATEGY_RESCORE_ALL, m, r, 0.1) == (0, m, a)
    for bad in ((7, 100, 0.3, 0.1), (pop.POP_STRATEGY_POP, 100, 0.01, 0.1), (pop.POP_STRATEGY_POP, 100, 0.99, 0.1),
                (pop.POP_STRATEGY_POP, 0, 0.3, 0.1)):
        with pytest.raises(pop.PopError):
            pop.pop_strategy_counts(*bad)


def test_null_handle_is_an_error_not_a_crash(lib):
    from paper_2602_06822_amd import binding as pop
    raw = pop.raw()
    assert raw.pop_layer_destroy(None) == pop.POP_EINVAL
    assert raw.pop_prefill_partition(None, None, 1, 0, 0, None, None, None, None, None) == pop.POP_EINVAL
    assert raw.pop_decode_mask(None, None, 1, None, None, None, None, None, None) == pop.POP_EINVAL
    assert raw.pop_pruned_ffn(None, None, 1, None, 0, None, 0, None) == pop.POP_EINVAL
    assert raw.pop_layer_get_norms(None, None, None) == pop.POP_EINVAL
