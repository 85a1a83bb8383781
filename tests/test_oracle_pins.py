"""Pins for the CPU oracle: every check here ties the oracle to something other than itself --
a library routine, a closed form, a brute-force definition, an invariant the paper states, or a
value the paper prints.  CPU only.
"""
import itertools
import math
import os

import numpy as np
import pytest
import torch

from paper_2602_06822_amd import synth

F32, BF16 = synth.F32, synth.BF16


def _tiny_layer(d, m, dtype, name="pin"):
    return synth.make_layer(synth.small_config(f"{name}_{d}_{m}_{dtype}", d, m, dtype))


def _t64(a, dtype):
    return torch.from_numpy(synth.storage_to_f64(a, dtype))


# ---------------------------------------------------------------- storage widening

def test_bf16_widening_matches_torch(oracle):
    g = synth.rng("bf16widen")
    a = g.standard_normal(4096, dtype=np.float32) * np.float32(3.0)
    bits = synth.f32_to_bf16_bits(a)
    ref = torch.from_numpy(a).to(torch.bfloat16)
    assert np.array_equal(bits.view(np.int16), ref.view(torch.int16).numpy())
    # the oracle reads bf16 exactly: norms of a 1-row matrix are |value|
    n = oracle.down_norms(bits.reshape(1, -1), BF16)
    assert np.array_equal(n, np.abs(ref.to(torch.float64).numpy()))


# ---------------------------------------------------------------- P1: dense SwiGLU

@pytest.mark.parametrize("dtype", [F32, BF16])
def test_zero_pruning_is_dense_swiglu_library(oracle, dtype):
    """0 % pruning (all-ones mask) must equal silu(x Wg^T) * (x Wu^T) Wd^T from torch float64."""
    L = _tiny_layer(48, 100, dtype)
    x = synth.make_activations(L, 5, "p1")
    X, Wg, Wu, Wd = (_t64(a, dtype) for a in (x, L.w_gate, L.w_up, L.w_down))
    ref = (torch.nn.functional.silu(X @ Wg.T) * (X @ Wu.T)) @ Wd.T
    y = oracle.pruned_ffn(x, L.w_gate, L.w_up, L.w_down, dtype, np.ones(100, np.uint8))
    np.testing.assert_allclose(y, ref.numpy(), rtol=1e-12, atol=1e-15)
    H = oracle.hidden(x, L.w_gate, L.w_up, dtype)
    Href = torch.nn.functional.silu(X @ Wg.T) * (X @ Wu.T)
    np.testing.assert_allclose(H, Href.numpy(), rtol=1e-12, atol=1e-18)


def test_dense_swiglu_triple_loop(oracle):
    """Same special case against loops written out here (catches a transposed operand)."""
    d, m, T = 6, 7, 3
    L = _tiny_layer(d, m, F32, "loop")
    x = synth.make_activations(L, T, "loop")
    y = oracle.pruned_ffn(x, L.w_gate, L.w_up, L.w_down, F32, np.ones(m, np.uint8))
    for t in range(T):
        for o in range(d):
            acc = 0.0
            for j in range(m):
                g = sum(float(x[t, k]) * float(L.w_gate[j, k]) for k in range(d))
                u = sum(float(x[t, k]) * float(L.w_up[j, k]) for k in range(d))
                acc += g / (1.0 + math.exp(-g)) * u * float(L.w_down[o, j])
            assert y[t, o] == pytest.approx(acc, rel=1e-12, abs=1e-18)


def test_silu_closed_form(oracle):
    """silu(ln 3) = 0.75 ln 3, silu(0) = 0, silu(-ln 3) = -0.25 ln 3 (exactly representable inputs aside)."""
    z = np.float32(math.log(3.0))
    x = np.array([[1.0, 0.0]], dtype=np.float32)
    w_gate = np.array([[z, 5.0], [0.0, 5.0], [-z, 5.0]], dtype=np.float32)
    w_up = np.array([[2.0, 7.0], [2.0, 7.0], [2.0, 7.0]], dtype=np.float32)
    H = oracle.hidden(x, w_gate, w_up, F32)
    zz = float(z)
    expect = [2.0 * zz / (1.0 + math.exp(-zz)), 0.0, -2.0 * zz / (1.0 + math.exp(zz))]
    np.testing.assert_allclose(H[0], expect, rtol=1e-14)
    assert H[0, 0] == pytest.approx(2 * 0.75 * math.log(3.0), rel=1e-6)
    assert H[0, 2] == pytest.approx(-2 * 0.25 * math.log(3.0), rel=1e-6)


def test_masked_ffn_equals_dense_on_submatrix(oracle):
    """A mask is the dense FFN of the sub-layer made of the kept channels (library routine)."""
    d, m, T = 32, 60, 4
    L = _tiny_layer(d, m, BF16, "sub")
    x = synth.make_activations(L, T, "sub")
    mask = (synth.rng("submask").random(m) < 0.4).astype(np.uint8)
    keep = np.nonzero(mask)[0]
    X, Wg, Wu, Wd = (_t64(a, BF16) for a in (x, L.w_gate, L.w_up, L.w_down))
    ref = (torch.nn.functional.silu(X @ Wg[keep].T) * (X @ Wu[keep].T)) @ Wd[:, keep].T
    y = oracle.pruned_ffn(x, L.w_gate, L.w_up, L.w_down, BF16, mask)
    np.testing.assert_allclose(y, ref.numpy(), rtol=1e-11, atol=1e-15)
    # per-token masks: each row is its own sub-layer
    masks = (synth.rng("submask2").random((T, m)) < 0.5).astype(np.uint8)
    y2 = oracle.pruned_ffn(x, L.w_gate, L.w_up, L.w_down, BF16, masks)
    for t in range(T):
        kp = np.nonzero(masks[t])[0]
        r = (torch.nn.functional.silu(X[t:t + 1] @ Wg[kp].T) * (X[t:t + 1] @ Wu[kp].T)) @ Wd[:, kp].T
        np.testing.assert_allclose(y2[t], r.numpy()[0], rtol=1e-11, atol=1e-15)


# ---------------------------------------------------------------- importance: P5, P6, directed

def test_importance_literal_equals_factorised(oracle):
    """Eq. 1 -> Eq. 2 (l2) summed element by element equals ||W_down[:,j]|| * ||H[:,j]|| (Eq. 3)."""
    d, m, T = 40, 72, 9
    L = _tiny_layer(d, m, BF16, "fact")
    x = synth.make_activations(L, T, "fact")
    H = oracle.hidden(x, L.w_gate, L.w_up, BF16)
    I = oracle.importance(L.w_down, BF16, H)
    Wd = synth.storage_to_f64(L.w_down, BF16)
    # independent: numpy norms
    ref = np.linalg.norm(Wd, axis=0) * np.linalg.norm(H, axis=0)
    np.testing.assert_allclose(I, ref, rtol=1e-12)
    # element-wise definition through numpy broadcasting: I_{t,o,j} = |W[o,j]| * |H[t,j]| summed in squares
    elem = (np.abs(Wd)[None, :, :] * np.abs(H)[:, None, :]) ** 2
    np.testing.assert_allclose(I, np.sqrt(elem.sum(axis=(0, 1))), rtol=1e-12)
    np.testing.assert_allclose(oracle.down_norms(L.w_down, BF16), np.linalg.norm(Wd, axis=0), rtol=1e-13)


def test_importance_single_token(oracle):
    """T = 1: I_j = n_j * |h_j|."""
    d, m = 24, 50
    L = _tiny_layer(d, m, F32, "t1")
    x = synth.make_activations(L, 1, "t1")
    H = oracle.hidden(x, L.w_gate, L.w_up, F32)
    I = oracle.importance(L.w_down, F32, H)
    n = np.linalg.norm(synth.storage_to_f64(L.w_down, F32), axis=0)
    np.testing.assert_allclose(I, n * np.abs(H[0]), rtol=1e-12)


def test_importance_token_order_and_sign_invariance(oracle):
    """The score depends on H only through column norms: permuting tokens or flipping signs keeps it."""
    d, m, T = 16, 30, 7
    L = _tiny_layer(d, m, F32, "inv")
    H = synth.rng("invH").standard_normal((T, m))
    I0 = oracle.importance(L.w_down, F32, H)
    perm = synth.rng("invperm").permutation(T)
    np.testing.assert_allclose(oracle.importance(L.w_down, F32, H[perm]), I0, rtol=1e-13)
    np.testing.assert_allclose(oracle.importance(L.w_down, F32, -H), I0, rtol=1e-15)
    # doubling the activations of one channel doubles exactly that channel's score
    H2 = H.copy()
    H2[:, 3] *= 2.0
    I2 = oracle.importance(L.w_down, F32, H2)
    assert I2[3] == pytest.approx(2 * I0[3], rel=1e-14)
    assert np.array_equal(np.delete(I2, 3), np.delete(I0, 3))


# ---------------------------------------------------------------- importance, input-side reading of Eq. 1-2

@pytest.mark.parametrize("dtype", [F32, BF16])
def test_input_side_importance_against_norms_and_loops(oracle, dtype):
    """I_j = || [W_gate[j,:], W_up[j,:]] * s ||_2, s_k = ||X[:,k]||_2: numpy's norm routine on the weighted rows,
    and the element scores of Eq. 1 summed one by one in Python on a few channels."""
    d, m, T = 24, 30, 7
    L = _tiny_layer(d, m, dtype, "inside")
    x = synth.make_activations(L, T, "inside")
    I = oracle.importance_input_side(x, L.w_gate, L.w_up, dtype)
    X, Wg, Wu = (synth.storage_to_f64(a, dtype) for a in (x, L.w_gate, L.w_up))
    s = np.linalg.norm(X, axis=0)
    ref = np.linalg.norm(np.concatenate([Wg * s, Wu * s], axis=1), axis=1)
    np.testing.assert_allclose(I, ref, rtol=1e-12)
    for j in (0, 11, m - 1):
        acc = 0.0
        for k in range(d):
            for t in range(T):
                acc += (abs(Wg[j, k]) * abs(X[t, k])) ** 2 + (abs(Wu[j, k]) * abs(X[t, k])) ** 2
        assert math.isclose(I[j], math.sqrt(acc), rel_tol=1e-12)
    # listed channels only
    part = oracle.importance_input_side(x, L.w_gate, L.w_up, dtype, chan=np.array([3, 9], np.int32))
    assert part[3] == I[3] and part[9] == I[9] and not part[[0, 1, 2, 4]].any()


def test_input_side_importance_over_rows_is_the_root_of_the_rows_squared_scores(oracle):
    """The input-side importance over several rows (a prompt, or the sequences of one batched step) equals the root
    of the sum of the squared single-row importances: what the batch-wide mask of that reading is built from."""
    d, m, T = 20, 26, 6
    L = _tiny_layer(d, m, BF16, "inside_rows")
    x = synth.make_activations(L, T, "inside_rows")
    whole = oracle.importance_input_side(x, L.w_gate, L.w_up, BF16)
    rows = np.stack([oracle.importance_input_side(x[t:t + 1], L.w_gate, L.w_up, BF16) for t in range(T)])
    np.testing.assert_allclose(whole, np.sqrt((rows ** 2).sum(axis=0)), rtol=1e-12)
    # and the output-side counterpart (Eq. 3 over the step's sequences): n_j * ||h_{:,j}|| from the per-row n_j |h_bj|
    H = oracle.hidden(x, L.w_gate, L.w_up, BF16)
    per_row = np.stack([oracle.importance(L.w_down, BF16, H[t:t + 1]) for t in range(T)])
    np.testing.assert_allclose(oracle.importance(L.w_down, BF16, H), np.sqrt((per_row ** 2).sum(axis=0)), rtol=1e-12)


def test_input_side_importance_closed_forms(oracle):
    """One-hot input: I_j = |c| * hypot(W_gate[j,k0], W_up[j,k0]).  All-ones input over T tokens with W_up = 0:
    I_j = sqrt(T) * ||W_gate[j,:]||.  Scaling x by a scales every score by |a|; scaling one channel's rows by b
    scales that score alone; token order and signs do not matter."""
    d, m, T = 16, 20, 5
    L = _tiny_layer(d, m, F32, "inside_cf")
    Wg, Wu = L.w_gate.astype(np.float64), L.w_up.astype(np.float64)
    x = np.zeros((T, d), np.float32)
    x[2, 5] = -3.0
    I = oracle.importance_input_side(x, L.w_gate, L.w_up, F32)
    np.testing.assert_allclose(I, 3.0 * np.hypot(Wg[:, 5], Wu[:, 5]), rtol=1e-13)
    ones = np.ones((T, d), np.float32)
    I = oracle.importance_input_side(ones, L.w_gate, np.zeros_like(L.w_up), F32)
    np.testing.assert_allclose(I, math.sqrt(T) * np.linalg.norm(Wg, axis=1), rtol=1e-13)
    x = synth.make_activations(L, T, "inside_cf")
    I = oracle.importance_input_side(x, L.w_gate, L.w_up, F32)
    np.testing.assert_allclose(oracle.importance_input_side(-2.0 * x, L.w_gate, L.w_up, F32), 2.0 * I, rtol=1e-13)
    wg2, wu2 = L.w_gate.copy(), L.w_up.copy()
    wg2[7] *= 4.0
    wu2[7] *= 4.0
    I2 = oracle.importance_input_side(x, wg2, wu2, F32)
    assert math.isclose(I2[7], 4.0 * I[7], rel_tol=1e-13)
    assert np.array_equal(np.delete(I2, 7), np.delete(I, 7))
    perm = np.array([4, 0, 3, 1, 2])
    flip = np.array([1, -1, 1, -1, -1], np.float32)[:, None]
    np.testing.assert_allclose(oracle.importance_input_side(x[perm] * flip, L.w_gate, L.w_up, F32), I, rtol=1e-13)
    # one token: s = |x|
    I1 = oracle.importance_input_side(x[:1], L.w_gate, L.w_up, F32)
    xa = np.abs(x[0].astype(np.float64))
    np.testing.assert_allclose(I1, np.sqrt(((Wg * xa) ** 2 + (Wu * xa) ** 2).sum(axis=1)), rtol=1e-13)
    # it is a different quantity from the output-side importance
    H = oracle.hidden(x, L.w_gate, L.w_up, F32)
    assert not np.allclose(I, oracle.importance(L.w_down, F32, H), rtol=1e-2)


def test_directed_weight_scaling_moves_channel(oracle):
    """Scaling a channel's down-projection column by 1e3 puts it in R; zeroing it puts it in P."""
    d, m, T = 32, 64, 8
    L = _tiny_layer(d, m, F32, "dir")
    x = synth.make_activations(L, T, "dir")
    n_ret, n_cand, _ = oracle.region_counts(m, 0.3, 0.4)
    _, region, _, _ = oracle.prefill(x, L.w_gate, L.w_up, L.w_down, F32, n_ret, n_cand)
    j_low = int(np.nonzero(region == 2)[0][0])
    j_high = int(np.nonzero(region == 0)[0][0])
    wd = L.w_down.copy()
    wd[:, j_low] *= np.float32(1e3)
    wd[:, j_high] = 0
    _, region2, _, _ = oracle.prefill(x, L.w_gate, L.w_up, wd, F32, n_ret, n_cand)
    assert region2[j_low] == 0 and region2[j_high] == 2


def test_partition_equivariant_under_channel_permutation(oracle):
    d, m, T = 32, 48, 6
    L = _tiny_layer(d, m, F32, "perm")
    x = synth.make_activations(L, T, "perm")
    n_ret, n_cand, _ = oracle.region_counts(m, 0.25, 0.5)
    s, region, _, _ = oracle.prefill(x, L.w_gate, L.w_up, L.w_down, F32, n_ret, n_cand)
    assert len(np.unique(s)) == m  # tie-free
    p = synth.rng("chanperm").permutation(m)
    s2, region2, _, _ = oracle.prefill(x, L.w_gate[p], L.w_up[p], np.ascontiguousarray(L.w_down[:, p]), F32,
                                       n_ret, n_cand)
    np.testing.assert_allclose(s2, s[p], rtol=1e-13)
    assert np.array_equal(region2, region[p])


# ---------------------------------------------------------------- counts

def test_region_counts_rule(oracle):
    # worked sizes for the Llama-2-7B shape at 35 % sparsity, candidate band 0.1
    assert oracle.region_counts(11008, 0.60, 0.10) == (6605, 1101, 3302)
    assert oracle.k_for_ratio(11008, 0.35, 6605, 1101) == 550
    assert oracle.region_counts(1376, 0.3, 0.4) == (413, 550, 413)
    assert oracle.k_for_ratio(1376, 0.5, 413, 550) == 275
    assert oracle.region_counts(10, 0.0, 1.0) == (0, 10, 0)
    assert oracle.region_counts(10, 1.0, 0.0) == (10, 0, 0)
    for m in (1, 7, 100, 11008, 14336):
        for fr, fc in ((0.0, 0.0), (0.3, 0.4), (0.55, 0.1), (0.45, 0.1), (0.2, 0.8)):
            a, b, c = oracle.region_counts(m, fr, fc)
            assert a + b + c == m and min(a, b, c) >= 0
            assert a == math.floor(fr * m + 0.5)
    with pytest.raises(ValueError):
        oracle.region_counts(10, 0.7, 0.5)


# ---------------------------------------------------------------- P2: invariants

@pytest.mark.parametrize("ties", ["none", "some", "all", "zeros"])
def test_partition_and_select_invariants(oracle, ties):
    m = 257
    s = synth.make_scores(m, "inv", ties)
    for n_ret, n_cand in ((77, 103), (0, 257), (257, 0), (0, 0), (1, 1), (100, 157)):
        region, ret, cand = oracle.partition(s, n_ret, n_cand)
        assert (region == 0).sum() == n_ret and (region == 1).sum() == n_cand
        assert (region == 2).sum() == m - n_ret - n_cand
        assert np.array_equal(ret, np.nonzero(region == 0)[0])
        assert np.array_equal(cand, np.nonzero(region == 1)[0])
        cs = synth.make_scores(n_cand, "inv_c", ties) if n_cand else np.zeros(0, np.float32)
        for k in sorted({0, n_cand // 2, n_cand}):
            mask, sel, act = oracle.select(region, cs, cand, k)
            assert mask.sum() == n_ret + k
            assert np.all(mask[region == 0] == 1) and np.all(mask[region == 2] == 0)
            assert np.all(region[sel] == 1) and np.all(np.diff(sel) > 0)
            assert np.array_equal(act, np.concatenate([ret, sel]))
            assert np.array_equal(np.sort(act), np.nonzero(mask)[0])


# ---------------------------------------------------------------- P3: brute force

def _precedes(s, a, b):
    """a ranks before b: higher score first, equal scores by lower index."""
    return s[a] > s[b] or (s[a] == s[b] and a < b)


def _brute_regions(s, n_ret, n_cand):
    """Enumerate all (R, C) set pairs; keep those where every member of a higher region precedes
    every member of a lower one.  Returns the list of solutions (must be exactly one)."""
    m = len(s)
    idx = range(m)
    sols = []
    for R in itertools.combinations(idx, n_ret):
        rest = [j for j in idx if j not in R]
        if any(not _precedes(s, a, b) for a in R for b in rest):
            continue
        for Cset in itertools.combinations(rest, n_cand):
            Pset = [j for j in rest if j not in Cset]
            if all(_precedes(s, a, b) for a in Cset for b in Pset):
                sols.append((set(R), set(Cset)))
    return sols


@pytest.mark.parametrize("case", range(12))
def test_partition_brute_force_tiny(oracle, case):
    g = synth.rng("brute", case)
    m = int(g.integers(3, 9))
    if case % 3 == 0:
        s = g.integers(0, 3, size=m).astype(np.float32)  # heavy ties
    elif case % 3 == 1:
        s = np.abs(g.standard_normal(m)).astype(np.float32)
    else:
        s = np.array([0.0, -0.0, 1.5, 1.5, 0.0, 2.0, -0.0, 1.5, 3.0][:m], dtype=np.float32)
    n_ret = int(g.integers(0, m + 1))
    n_cand = int(g.integers(0, m - n_ret + 1))
    sols = _brute_regions(s, n_ret, n_cand)
    assert len(sols) == 1
    region, ret, cand = oracle.partition(s, n_ret, n_cand)
    assert set(ret.tolist()) == sols[0][0] and set(cand.tolist()) == sols[0][1]


@pytest.mark.parametrize("case", range(10))
def test_topk_brute_force_tiny(oracle, case):
    g = synth.rng("brutek", case)
    m = int(g.integers(4, 11))
    region = g.integers(0, 3, size=m).astype(np.uint8)
    cand = np.nonzero(region == 1)[0].astype(np.int32)
    n_cand = len(cand)
    cs = (g.integers(0, 3, size=n_cand).astype(np.float32) if case % 2 == 0
          else np.abs(g.standard_normal(n_cand)).astype(np.float32))
    by_chan = {int(j): cs[i] for i, j in enumerate(cand)}
    for k in range(n_cand + 1):
        sols = []
        for S in itertools.combinations(cand.tolist(), k):
            rest = [j for j in cand.tolist() if j not in S]
            if all(_precedes(by_chan, a, b) for a in S for b in rest):
                sols.append(set(S))
        assert len(sols) == 1
        mask, sel, act = oracle.select(region, cs, cand, k)
        assert set(sel.tolist()) == sols[0]
        assert set(np.nonzero(mask)[0].tolist()) == sols[0] | set(np.nonzero(region == 0)[0].tolist())


def test_rank_counting_definition(oracle):
    """rank_j = #{i : i precedes j}; regions are rank intervals (O(m^2) definition, medium m, ties)."""
    m = 300
    s = synth.make_scores(m, "rank", "some")
    rank = np.array([sum(_precedes(s, i, j) for i in range(m)) for j in range(m)])
    assert sorted(rank.tolist()) == list(range(m))
    n_ret, n_cand = 90, 120
    region, _, _ = oracle.partition(s, n_ret, n_cand)
    expect = np.where(rank < n_ret, 0, np.where(rank < n_ret + n_cand, 1, 2))
    assert np.array_equal(region, expect)


# ---------------------------------------------------------------- P4: threshold form (Sec. 3.3)

def test_threshold_form_on_tie_free_scores(oracle):
    """R = {I >= tau_high}, P = {I <= tau_low}, C strictly between, with order-statistic quantiles."""
    m = 1000
    s = synth.make_scores(m, "thr", "none").astype(np.float64)
    for n_ret, n_cand in ((300, 400), (550, 100), (1, 998), (999, 0)):
        n_prn = m - n_ret - n_cand
        asc = np.sort(s)
        tau_high = asc[m - n_ret]                    # n_ret-th largest
        R = s >= tau_high
        if n_prn > 0:
            tau_low = asc[n_prn - 1]                 # n_prn-th smallest
            P = s <= tau_low
        else:
            tau_low = -np.inf
            P = np.zeros(m, bool)
        Cnd = (s > tau_low) & (s < tau_high)
        region, _, _ = oracle.partition(s, n_ret, n_cand)
        assert np.array_equal(region == 0, R)
        assert np.array_equal(region == 2, P)
        assert np.array_equal(region == 1, Cnd)


# ---------------------------------------------------------------- P7 / P8: the ablation variants

def test_variant1_static_mask_is_global_topk_of_prefill_scores(oracle):
    """Selecting inside C with the prefill scores themselves gives the global top-(n_ret+k)."""
    m = 500
    s = synth.make_scores(m, "v1", "some")
    n_ret, n_cand = 200, 150
    region, ret, cand = oracle.partition(s, n_ret, n_cand)
    for k in (0, 40, 150):
        mask, _, _ = oracle.select(region, s[cand], cand, k)
        top_region, _, _ = oracle.partition(s, n_ret + k, 0)
        assert np.array_equal(mask, (top_region == 0).astype(np.uint8))


def test_variant2_all_candidates_is_plain_topk(oracle):
    """n_ret = n_prn = 0: the step mask is torch.topk of the step scores (distinct values)."""
    m = 640
    region, ret, cand = oracle.partition(synth.make_scores(m, "v2a", "none"), 0, m)
    assert len(ret) == 0 and np.array_equal(cand, np.arange(m))
    cs = synth.make_scores(m, "v2b", "none")
    for k in (1, 17, 320, 640):
        mask, sel, _ = oracle.select(region, cs, cand, k)
        top = torch.topk(torch.from_numpy(cs), k).indices.numpy()
        assert np.array_equal(np.sort(top), sel)
        assert mask.sum() == k


# ---------------------------------------------------------------- decode step consistency

@pytest.mark.parametrize("dtype", [F32, BF16])
def test_decode_step_against_pieces(oracle, dtype):
    """The decode step is: hidden over R+C (library check), |h| * n for C, top-k, masked dense FFN."""
    d, m, T = 64, 150, 12
    L = _tiny_layer(d, m, dtype, "dec")
    x = synth.make_activations(L, T, "prompt")
    xt = synth.make_activations(L, 3, "decode")
    n_ret, n_cand, n_prn = oracle.region_counts(m, 0.3, 0.4)
    k = oracle.k_for_ratio(m, 0.5, n_ret, n_cand)
    scores, region, ret, cand = oracle.prefill(x, L.w_gate, L.w_up, L.w_down, dtype, n_ret, n_cand)
    X, Wg, Wu, Wd = (_t64(a, dtype) for a in (xt, L.w_gate, L.w_up, L.w_down))
    Href = (torch.nn.functional.silu(X @ Wg.T) * (X @ Wu.T)).numpy()
    nrm = np.linalg.norm(Wd.numpy(), axis=0)
    for t in range(3):
        out = oracle.decode(xt[t], L.w_gate, L.w_up, L.w_down, dtype, region, cand, k)
        rc = region != 2
        np.testing.assert_allclose(out["h"][rc], Href[t][rc], rtol=1e-11, atol=1e-18)
        assert np.all(out["h"][~rc] == 0)
        np.testing.assert_allclose(out["cscore"], nrm[cand] * np.abs(Href[t][cand]), rtol=1e-11)
        # decode never selects outside the candidate region; active count matches
        assert np.all(region[out["sel_idx"]] == 1)
        assert out["mask"].sum() == n_ret + k == out["n_active"]
        order = np.lexsort((cand, -out["cscore"]))
        assert np.array_equal(np.sort(cand[order[:k]]), out["sel_idx"])
        keep = np.nonzero(out["mask"])[0]
        yref = (Href[t][keep] * Wd.numpy()[:, keep]).sum(axis=1)
        np.testing.assert_allclose(out["y"], yref, rtol=1e-10, atol=1e-16)
    # k = n_cand and nothing pruned: the decode output is the dense FFN
    region0, _, cand0 = oracle.partition(scores, n_ret, m - n_ret)
    out = oracle.decode(xt[0], L.w_gate, L.w_up, L.w_down, dtype, region0, cand0, m - n_ret)
    dense = (torch.from_numpy(Href[0]) @ Wd.T).numpy()
    np.testing.assert_allclose(out["y"], dense, rtol=1e-10, atol=1e-16)


def test_prefill_scores_use_all_tokens(oracle):
    """Prefill aggregates over every prompt token: s^2 over a split prompt adds up."""
    d, m, T = 32, 40, 10
    L = _tiny_layer(d, m, F32, "split")
    x = synth.make_activations(L, T, "split")
    s_all, *_ = oracle.prefill(x, L.w_gate, L.w_up, L.w_down, F32, 10, 10)
    s_a, *_ = oracle.prefill(x[:4], L.w_gate, L.w_up, L.w_down, F32, 10, 10)
    s_b, *_ = oracle.prefill(x[4:], L.w_gate, L.w_up, L.w_down, F32, 10, 10)
    np.testing.assert_allclose(s_all ** 2, s_a ** 2 + s_b ** 2, rtol=1e-12)


# ---------------------------------------------------------------- P9: printed overhead ratios

def test_printed_overheads_support_candidate_fraction_reading():
    """Scoring a channel without factorising costs one pass over its d down-projection weights,
    a dense channel costs three; so re-scoring all channels adds 1/3 and re-scoring a candidate band of
    fraction gamma adds gamma/3.  The printed table (gamma = 0.1) is closer to gamma/3 than to 2*gamma/3,
    i.e. gamma is the whole candidate fraction |C|/m."""
    path = os.path.join(os.path.dirname(__file__), "golden", "overhead_table.txt")
    rows = [ln.split() for ln in open(path) if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 2
    for _, dense, v2, v2pct, pop, poppct in rows:
        dense, v2, v2pct, pop, poppct = map(float, (dense, v2, v2pct, pop, poppct))
        assert 100 * v2 / dense == pytest.approx(v2pct, abs=0.1)
        assert 100 * pop / dense == pytest.approx(poppct, abs=0.01)
        assert v2pct == pytest.approx(100 / 3, abs=0.5)
        gamma = 0.1
        assert abs(poppct - 100 * gamma / 3) < abs(poppct - 200 * gamma / 3)
