"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs.

Bars: partitions, masks and index lists byte-identical when both sides are given identical float32
scores; scores within 1e-5 relative (prefill: purely relative; single-token decode quantities: purely relative
for float32 layers, with a floor of 1e-2 * max for bf16 layers, see DECODE_FLOOR);
FFN outputs within 1e-4 (float32 weights) / 2e-2 (bf16 weights) max-abs relative to max|y|.
"""
import numpy as np
import pytest
import torch

from paper_2602_06822_amd import synth

from gpu_util import GpuLayer, dev, host, max_abs_rel, score_rel_err

pytestmark = pytest.mark.gpu

F32, BF16 = synth.F32, synth.BF16
SCORE_TOL = 1e-5
# Floor of the relative measure for single-token (decode) quantities, as a fraction of the largest value.
# float32 layers accumulate dot products in float64, so h is accurate to a few ulp and the measure is purely
# relative.  bf16 layers accumulate in float32: a dot product that cancels carries an absolute error of about
# log2(d) * 2^-24 * sum|x_k w_k|, which is ~1e-7 of the largest h, so relative accuracy 1e-5 holds down to 1e-2 of it.
DECODE_FLOOR = {0: 1e-9, 1: 1e-2}
Y_TOL = {F32: 1e-4, BF16: 2e-2}


@pytest.fixture(scope="module")
def pop():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2602_06822_amd import binding
    return binding


# ---------------------------------------------------------------- selection on given scores (bit-exact)

SEL_CASES = [
    # m, n_ret, n_cand
    (1, 0, 1), (1, 1, 0), (1, 0, 0), (7, 3, 2), (64, 20, 30), (257, 77, 103), (1000, 0, 1000), (1000, 1000, 0),
    (1376, 413, 550), (4097, 1, 4095), (11008, 6605, 1101), (11008, 0, 0), (14336, 8602, 1433), (30000, 12000, 9000),
]


@pytest.mark.parametrize("ties", ["none", "some", "all", "zeros"])
def test_partition_from_scores_bit_exact(pop, oracle, ties):
    for m, n_ret, n_cand in SEL_CASES:
        s = synth.make_scores(m, f"gpu_part_{m}", ties)
        region = torch.full((m,), 9, dtype=torch.uint8, device="cuda")
        ret = torch.full((max(n_ret, 1),), -1, dtype=torch.int32, device="cuda")
        cand = torch.full((max(n_cand, 1),), -1, dtype=torch.int32, device="cuda")
        pop.pop_partition_from_scores(dev(s), m, n_ret, n_cand, region, ret, cand)
        r0, ret0, cand0 = oracle.partition(s, n_ret, n_cand)
        assert np.array_equal(host(region), r0), (m, n_ret, n_cand, ties)
        assert np.array_equal(host(ret)[:n_ret], ret0), (m, n_ret, n_cand, ties)
        assert np.array_equal(host(cand)[:n_cand], cand0), (m, n_ret, n_cand, ties)


@pytest.mark.parametrize("shape", synth.SCORE_SHAPES)
def test_partition_from_scores_shaped_keys(pop, oracle, shape):
    """Score vectors whose keys crowd into few digit values, differ in few bits or span many binades: the two
    thresholds fall into one digit bucket or into different ones, into short buckets or into ones too long for the
    selector's key lists, with the keys staged on chip (m <= 24576) or read from memory."""
    for m in (5000, 11008, 24576, 30000):
        s = synth.make_scores_shaped(m, f"gpu_part_shaped_{m}", shape)
        for n_ret, n_cand in ((int(0.6 * m), int(0.1 * m)), (1, 1), (m - 2, 1), (m // 2, 3), (m // 3, m - m // 3)):
            region = torch.full((m,), 9, dtype=torch.uint8, device="cuda")
            ret = torch.full((n_ret,), -1, dtype=torch.int32, device="cuda")
            cand = torch.full((n_cand,), -1, dtype=torch.int32, device="cuda")
            pop.pop_partition_from_scores(dev(s), m, n_ret, n_cand, region, ret, cand)
            r0, ret0, cand0 = oracle.partition(s, n_ret, n_cand)
            assert np.array_equal(host(region), r0), (m, n_ret, n_cand, shape)
            assert np.array_equal(host(ret), ret0), (m, n_ret, n_cand, shape)
            assert np.array_equal(host(cand), cand0), (m, n_ret, n_cand, shape)


@pytest.mark.parametrize("kind", ["none", "some", "all", "zeros"] + list(synth.SCORE_SHAPES))
def test_partition_top_from_scores_bit_exact(pop, oracle, kind):
    """The partition launch that also emits the n_top best channels (the prompt's own mask): regions as before, and
    the top set equal to the retained set of a partition with n_ret = n_top, on tied and on shaped score vectors, with
    the third rank inside, at the edges of and outside the candidate band."""
    for m in (301, 5000, 11008, 30000):
        s = synth.make_scores(m, f"gpu_top_{m}", kind) if kind in ("none", "some", "all", "zeros") \
            else synth.make_scores_shaped(m, f"gpu_top_{m}", kind)
        n_ret, n_cand = int(0.6 * m), int(0.1 * m)
        for nr, nc, n_top in ((n_ret, n_cand, n_ret + n_cand // 2), (n_ret, n_cand, n_ret), (n_ret, n_cand, n_ret + n_cand),
                              (n_ret, n_cand, 0), (n_ret, n_cand, m), (0, 0, 7), (0, m, 1), (m, 0, m - 1),
                              (m // 2, 3, m // 2 + 2)):
            region = torch.full((m,), 9, dtype=torch.uint8, device="cuda")
            ret = torch.full((max(nr, 1),), -1, dtype=torch.int32, device="cuda")
            cand = torch.full((max(nc, 1),), -1, dtype=torch.int32, device="cuda")
            tmask = torch.full((m,), 9, dtype=torch.uint8, device="cuda")
            tlist = torch.full((max(n_top, 1),), -1, dtype=torch.int32, device="cuda")
            pop.pop_partition_top_from_scores(dev(s), m, nr, nc, n_top, region, ret, cand, tmask, tlist)
            r0, ret0, cand0 = oracle.partition(s, nr, nc)
            rt, top0, _ = oracle.partition(s, n_top, 0)
            case = (m, nr, nc, n_top, kind)
            assert np.array_equal(host(region), r0), case
            assert np.array_equal(host(ret)[:nr], ret0) and np.array_equal(host(cand)[:nc], cand0), case
            assert np.array_equal(host(tmask), (rt == 0).astype(np.uint8)), case
            assert np.array_equal(host(tlist)[:n_top], top0), case


@pytest.mark.parametrize("ties", ["none", "some", "all", "zeros"])
def test_topk_from_scores_bit_exact(pop, oracle, ties):
    for m, n_ret, n_cand in SEL_CASES:
        region, ret, cand = oracle.partition(synth.make_scores(m, f"gpu_topk_r_{m}", "some"), n_ret, n_cand)
        cs = synth.make_scores(n_cand, f"gpu_topk_{m}", ties) if n_cand else np.zeros(0, np.float32)
        for k in sorted({0, 1 if n_cand else 0, n_cand // 2, max(n_cand - 1, 0), n_cand}):
            mask = torch.full((m,), 9, dtype=torch.uint8, device="cuda")
            sel = torch.full((max(k, 1),), -1, dtype=torch.int32, device="cuda")
            pop.pop_topk_from_scores(dev(cs) if n_cand else None, dev(cand) if n_cand else None, n_cand, k,
                                     dev(region), m, mask, sel)
            mask0, sel0, _ = oracle.select(region, cs, cand, k)
            assert np.array_equal(host(mask), mask0), (m, n_ret, n_cand, k, ties)
            assert np.array_equal(host(sel)[:k], sel0), (m, n_ret, n_cand, k, ties)


# ---------------------------------------------------------------- whole path on small layers

SMALL = [
    # name, d, m, dtype, T, fractions, r
    ("f32_ragged", 260, 333, F32, 70, (0.3, 0.4), 0.5),
    ("bf16_ragged", 264, 333, BF16, 150, (0.3, 0.4), 0.5),
    ("bf16_tiles", 512, 640, BF16, 300, (0.6, 0.1), 0.35),
    ("f32_tiles", 512, 200, F32, 130, (0.45, 0.1), 0.5),
    ("bf16_wide", 2056, 96, BF16, 9, (0.25, 0.5), 0.4),
]


def _check_prefill(oracle, G, L, x, n_ret, n_cand, score_tol=SCORE_TOL):
    scores, region, ret, cand = G.prefill(x, n_ret, n_cand)
    s_ref, region_ref, ret_ref, cand_ref = oracle.prefill(x, L.w_gate, L.w_up, L.w_down, L.cfg.dtype, n_ret, n_cand)
    err = score_rel_err(scores, s_ref, eps=1e-6)
    assert err <= score_tol, f"prefill score error {err:.3e}"
    # identical scores -> identical partition, both ways
    r1, ret1, cand1 = oracle.partition(scores, n_ret, n_cand)
    assert np.array_equal(region, r1) and np.array_equal(ret, ret1) and np.array_equal(cand, cand1)
    return scores, region, ret, cand, s_ref


def _check_decode(oracle, G, L, region, cand, x_t, ks, ydtype=None):
    dtype = L.cfg.dtype
    out = G.decode(x_t, ks, ydtype)
    B = x_t.shape[0]
    ks = [ks] * B if isinstance(ks, int) else ks
    n_ret = int((region == 0).sum())
    rc = region != 2
    out["y_ref"] = []
    for b in range(B):
        ref = oracle.decode(x_t[b], L.w_gate, L.w_up, L.w_down, dtype, region, cand, ks[b], want_y=False)
        herr = score_rel_err(out["h"][b][rc], ref["h"][rc], eps=DECODE_FLOOR[dtype])
        assert herr <= SCORE_TOL, f"h error {herr:.3e}"
        cerr = score_rel_err(out["cscore"][b], ref["cscore"], eps=DECODE_FLOOR[dtype])
        assert cerr <= SCORE_TOL, f"candidate score error {cerr:.3e}"
        # the GPU's own float32 scores through the oracle's selector: byte-identical decisions
        mask1, sel1, act1 = oracle.select(region, out["cscore"][b], cand, ks[b])
        assert np.array_equal(out["mask"][b], mask1)
        assert out["n_active"][b] == n_ret + ks[b]
        assert np.array_equal(out["active_idx"][b][:n_ret + ks[b]], act1)
        # FFN output under the same mask, oracle in double
        y_ref = oracle.down(ref["h"].reshape(1, -1), L.w_down, dtype, mask1)[0]
        yerr = max_abs_rel(out["y"][b], y_ref)
        assert yerr <= Y_TOL[dtype], f"y error {yerr:.3e}"
        out["y_ref"].append(y_ref)
    # the whole step in one call: the same results bit for bit, y included (a single-sequence step is the same
    # launch either way, with the same fixed summation order), and again when repeated
    for rep in range(2):
        one = G.decode(x_t, ks, ydtype, one_call=True)
        for key in ("mask", "active_idx", "n_active", "cscore", "y"):
            assert np.array_equal(one[key], out[key]), (rep, key)
        assert np.array_equal(one["h"][:, rc], out["h"][:, rc]), rep
    return out


@pytest.mark.parametrize("name,d,m,dtype,T,fr,r", SMALL)
def test_small_layer_end_to_end(pop, oracle, name, d, m, dtype, T, fr, r):
    L = synth.make_layer(synth.small_config(name, d, m, dtype, n_outlier=3, heavy_tail=dtype == BF16))
    x = synth.make_activations(L, T, "prompt")
    xt = synth.make_activations(L, 5, "decode")
    n_ret, n_cand, _ = pop.pop_region_counts(m, *fr)
    assert (n_ret, n_cand) == oracle.region_counts(m, *fr)[:2]
    k = pop.pop_k_for_ratio(m, r, n_ret, n_cand)
    assert k == oracle.k_for_ratio(m, r, n_ret, n_cand)
    with GpuLayer(pop, L, max_tokens=T, max_batch=4) as G:
        np.testing.assert_allclose(G.norms(), oracle.down_norms(L.w_down, dtype), rtol=2e-7)
        scores, region, ret, cand, s_ref = _check_prefill(oracle, G, L, x, n_ret, n_cand)
        # oracle scores rounded to float32 through the GPU selector
        s32 = s_ref.astype(np.float32)
        reg_t = torch.empty(m, dtype=torch.uint8, device="cuda")
        pop.pop_partition_from_scores(dev(s32), m, n_ret, n_cand, reg_t, None, None)
        assert np.array_equal(host(reg_t), oracle.partition(s32, n_ret, n_cand)[0])
        for t in range(3):
            _check_decode(oracle, G, L, region, cand, xt[t:t + 1], k)
        # edge selections: nothing / everything selected
        _check_decode(oracle, G, L, region, cand, xt[3:4], 0)
        _check_decode(oracle, G, L, region, cand, xt[4:5], n_cand)
        # batch with a different k per sequence
        _check_decode(oracle, G, L, region, cand, xt[:4], [k, 0, n_cand, max(k - 1, 0)])
        _check_decode(oracle, G, L, region, cand, xt[1:3], [k, k], ydtype=F32)


@pytest.mark.parametrize("dtype,wgs", [(BF16, 6), (F32, 6), (BF16, 4), (BF16, 40)])
def test_fused_step_many_rounds_per_workgroup(pop, oracle, monkeypatch, dtype, wgs):
    """Few workgroups => many rounds each: exercises the ping-pong stream, the candidate and selected rows that
    ride along with the retained rounds and, with 4 workgroups, many candidate slots per workgroup."""
    monkeypatch.setenv("POP_FUSED_WGS", str(wgs))
    d, m, T = 512, 768, 40
    L = synth.make_layer(synth.small_config(f"many_rounds_{wgs}", d, m, dtype, n_outlier=2, heavy_tail=dtype == BF16))
    x = synth.make_activations(L, T, "prompt")
    xt = synth.make_activations(L, 6, "decode")
    n_ret, n_cand, _ = pop.pop_region_counts(m, 0.25 if wgs == 4 else 0.6, 0.1)
    k = n_cand // 2
    with GpuLayer(pop, L, max_tokens=T, max_batch=1) as G:
        scores, region, ret, cand, _ = _check_prefill(oracle, G, L, x, n_ret, n_cand)
        outs = [_check_decode(oracle, G, L, region, cand, xt[t:t + 1], kk)
                for t, kk in enumerate([k, k, 0, n_cand, 1, k])]
        assert pop.pop_layer_step_kind(G.handle) == (1, wgs)  # the fused kernel ran, with the forced grid
        # the same step again gives the same bits (the in-kernel flags were rearmed correctly; the assignment
        # of channels to workgroups is fixed, so the summation order of y is too)
        first = outs[5]
        for _ in range(3):
            again = G.decode(xt[5:6], k)
            for key in ("mask", "active_idx", "y", "cscore"):
                assert np.array_equal(first[key], again[key]), key


@pytest.mark.parametrize("dtype,wgs", [(BF16, 4), (F32, 6)])
def test_fused_step_input_side_many_candidate_slots(pop, oracle, monkeypatch, dtype, wgs):
    """The input-side reading in the fused kernel with few workgroups: many candidate slots each, so rounds of
    candidates only (four per round, two of them in the retained channels' buffers) and a last round of one to
    three; candidate scores, selection, h of the active channels and y against the oracle."""
    monkeypatch.setenv("POP_FUSED_WGS", str(wgs))
    d, m, T = 512, 768, 40
    L = synth.make_layer(synth.small_config(f"input_side_slots_{wgs}", d, m, dtype, n_outlier=2, heavy_tail=dtype == BF16))
    x = synth.make_activations(L, T, "prompt")
    xt = synth.make_activations(L, 4, "decode")
    for f_cand in (0.1, 0.123):  # 77 and 94 candidates: different remainders of four per workgroup
        n_ret, n_cand, _ = pop.pop_region_counts(m, 0.3, f_cand)
        with GpuLayer(pop, L, max_tokens=T, max_batch=1) as G:
            pop.pop_layer_set_importance(G.handle, pop.POP_IMPORTANCE_INPUT_SIDE)
            scores, region, ret, cand = G.prefill(x, n_ret, n_cand)
            r1, _, cand1 = oracle.partition(scores, n_ret, n_cand)
            assert np.array_equal(region, r1) and np.array_equal(cand, cand1)
            for t, k in enumerate([n_cand // 2, 0, n_cand, 1]):
                out = G.decode(xt[t:t + 1], k, one_call=bool(t % 2))
                assert pop.pop_layer_step_kind(G.handle) == (1, wgs)
                c_ref = oracle.importance_input_side(xt[t:t + 1], L.w_gate, L.w_up, dtype, chan=cand)[cand]
                assert score_rel_err(out["cscore"][0], c_ref, eps=1e-6) <= SCORE_TOL
                mask1, _, act1 = oracle.select(region, out["cscore"][0], cand, k)
                assert np.array_equal(out["mask"][0], mask1)
                assert np.array_equal(out["active_idx"][0][:n_ret + k], act1)
                active = np.flatnonzero(mask1).astype(np.int32)
                H = oracle.hidden(xt[t:t + 1], L.w_gate, L.w_up, dtype, chan=active)
                assert score_rel_err(out["h"][0][active], H[0][active], eps=DECODE_FLOOR[dtype]) <= SCORE_TOL
                assert max_abs_rel(out["y"][0], oracle.down(H, L.w_down, dtype, mask1)[0]) <= Y_TOL[dtype]


@pytest.mark.parametrize("strategy,gamma", [(0, 0.1), (0, 0.2), (1, 0.0), (2, 0.0)])
def test_strategy_as_layer_mode(pop, oracle, strategy, gamma):
    """The ablation's decode strategies as a mode of the layer: after pop_layer_set_strategy the sentinel counts give
    the partition, the prompt's forward pass and the steps of the explicit counts of pop_strategy_counts, bit for
    bit; without a strategy the sentinels are refused."""
    d, m, T, r = 256, 640, 40, 0.4
    L = synth.make_layer(synth.small_config(f"mode_{strategy}_{gamma}", d, m, BF16, n_outlier=2, heavy_tail=True))
    x = synth.make_activations(L, T, "prompt")
    xt = synth.make_activations(L, 3, "decode")
    n_ret, n_cand, k = pop.pop_strategy_counts(strategy, m, r, gamma)
    with GpuLayer(pop, L, max_tokens=T, max_batch=3) as G:
        with pytest.raises(pop.PopError) as e:
            pop.pop_prefill_partition(G.handle, dev(x), T, pop.POP_FROM_STRATEGY, pop.POP_FROM_STRATEGY)
        assert e.value.status == pop.POP_ESTATE
        explicit = G.prefill(x, n_ret, n_cand)
        steps = [G.decode(xt[:1], k), G.decode(xt, k, one_call=True)]
        fwd = G.prefill_forward(x, n_ret, n_cand, k, F32)
        with pytest.raises(pop.PopError) as e:
            G.decode(xt[:1], None)
        assert e.value.status == pop.POP_EINVAL
        with pytest.raises(pop.PopError):
            pop.pop_layer_set_strategy(G.handle, 7, r, gamma)
        pop.pop_layer_set_strategy(G.handle, strategy, r, gamma)
        scores = torch.empty(m, dtype=torch.float32, device="cuda")
        region = torch.empty(m, dtype=torch.uint8, device="cuda")
        pop.pop_prefill_partition(G.handle, dev(x), T, pop.POP_FROM_STRATEGY, pop.POP_FROM_STRATEGY, scores, region)
        assert np.array_equal(host(scores), explicit[0]) and np.array_equal(host(region), explicit[1])
        for ref, (xb, one) in zip(steps, ((xt[:1], False), (xt, True))):
            got = G.decode(xb, None, one_call=one)
            for key in ("mask", "active_idx", "n_active", "cscore", "y"):
                assert np.array_equal(got[key], ref[key]), key
        y = torch.empty((T, d), dtype=torch.float32, device="cuda")
        mask = torch.empty(m, dtype=torch.uint8, device="cuda")
        pop.pop_prefill_forward(G.handle, dev(x), T, pop.POP_FROM_STRATEGY, pop.POP_FROM_STRATEGY, pop.POP_FROM_STRATEGY,
                                y, F32, None, None, None, None, mask)
        assert np.array_equal(host(mask), fwd[4]) and np.array_equal(host(y).astype(np.float64), fwd[5])
        # and against the oracle: the mode's steps are the method's steps with those counts
        _check_decode(oracle, G, L, explicit[1], explicit[3], xt[:1], k)


def test_large_candidate_sets(pop, oracle, monkeypatch):
    """Candidate sets beyond the selection's own key buffer (4096 keys): a layer of many channels and a short hidden
    size, most channels candidates.  One sequence and a batch of three with different k (the separate top-k launch with
    its keys and decisions in launch-provided LDS; the batch also through the selection inside the gate/up launch),
    and the input-side reading of the same layer."""
    d, m, T = 128, 6000, 24
    L = synth.make_layer(synth.small_config("large_cand", d, m, BF16, n_outlier=2, heavy_tail=True))
    x = synth.make_activations(L, T, "prompt")
    xt = synth.make_activations(L, 4, "decode")
    n_ret, n_cand = 700, 5000
    with GpuLayer(pop, L, max_tokens=T, max_batch=3) as G:
        scores, region, ret, cand, _ = _check_prefill(oracle, G, L, x, n_ret, n_cand)
        for k in (2500, 1, n_cand):
            _check_decode(oracle, G, L, region, cand, xt[:1], k)
        _check_decode(oracle, G, L, region, cand, xt[1:4], [2500, 0, 4999])
        pop.pop_layer_set_importance(G.handle, pop.POP_IMPORTANCE_INPUT_SIDE)
        scores, region, ret, cand = G.prefill(x, n_ret, n_cand)
        out = G.decode(xt[1:4], [2500, 7, n_cand])
        for b, k in enumerate([2500, 7, n_cand]):
            c_ref = oracle.importance_input_side(xt[1 + b:2 + b], L.w_gate, L.w_up, BF16, chan=cand)[cand]
            assert score_rel_err(out["cscore"][b], c_ref, eps=1e-6) <= SCORE_TOL
            mask1, _, act1 = oracle.select(region, out["cscore"][b], cand, k)
            assert np.array_equal(out["mask"][b], mask1)
            assert np.array_equal(out["active_idx"][b][:n_ret + k], act1)
            active = np.flatnonzero(mask1).astype(np.int32)
            H = oracle.hidden(xt[1 + b:2 + b], L.w_gate, L.w_up, BF16, chan=active)
            assert max_abs_rel(out["y"][b], oracle.down(H, L.w_down, BF16, mask1)[0]) <= Y_TOL[BF16]


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_degenerate_partitions(pop, oracle, dtype):
    d, m, T = 128, 90, 20
    L = synth.make_layer(synth.small_config("degenerate", d, m, dtype))
    x = synth.make_activations(L, T, "prompt")
    xt = synth.make_activations(L, 2, "decode")
    with GpuLayer(pop, L, max_tokens=T, max_batch=2) as G:
        for n_ret, n_cand, k in ((0, m, 30), (m, 0, 0), (0, 0, 0), (10, 0, 0), (0, 17, 17), (89, 1, 1)):
            scores, region, ret, cand, _ = _check_prefill(oracle, G, L, x, n_ret, n_cand)
            _check_decode(oracle, G, L, region, cand, xt[:1], k)
            _check_decode(oracle, G, L, region, cand, xt, [k, 0])


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_pruned_ffn_standalone(pop, oracle, dtype):
    """Stand-alone masks: all ones (= dense FFN), a shared random mask, per-token masks, token chunks with a tail."""
    d, m, T = 264 if dtype == BF16 else 260, 301, 19
    L = synth.make_layer(synth.small_config("standalone", d, m, dtype))
    x = synth.make_activations(L, T, "tokens")
    g = synth.rng("standalone_masks", dtype)
    with GpuLayer(pop, L, max_tokens=T, max_batch=8) as G:
        for mask in (np.ones(m, np.uint8), (g.random(m) < 0.4).astype(np.uint8), np.zeros(m, np.uint8),
                     (g.random((T, m)) < 0.5).astype(np.uint8)):
            for ydtype in (F32, dtype):
                y = G.ffn(x, mask, ydtype)
                y_ref = oracle.pruned_ffn(x, L.w_gate, L.w_up, L.w_down, dtype, mask)
                if not y_ref.any():
                    assert not y.any()
                else:
                    assert max_abs_rel(y, y_ref) <= (Y_TOL[dtype] if ydtype == BF16 else 1e-4)
        # a stand-alone call invalidates the cached decode step
        with pytest.raises(pop.PopError) as e:
            y = torch.empty((1, d), dtype=torch.float32, device="cuda")
            pop.pop_pruned_ffn(G.handle, None, 1, None, 0, y, F32)
        assert e.value.status == pop.POP_ESTATE


# From 32 tokens on a bf16 layer's stand-alone pruned FFN runs on the matrix cores and rounds H to bf16 before the
# down projection (relative error 2^-9 per term, adding in quadrature over the active channels): float32 outputs of
# that path are held to 4e-3 of max|y|, well inside the 2e-2 allowed for bf16 layers; bf16 outputs to the 2e-2.
FFN_MFMA_TOL_F32 = 4e-3


@pytest.mark.parametrize("T", [32, 150, 300])
def test_pruned_ffn_prompt_sized_bf16(pop, oracle, T):
    """Stand-alone pruned FFN of many tokens (forward pass of a prompt under a mask; Sec. 3.4): token tiles with
    a ragged tail, channel counts that are no multiple of the k-step, an empty mask, per-token masks."""
    d, m = 264, 301
    L = synth.make_layer(synth.small_config("ffn_prompt", d, m, BF16))
    x = synth.make_activations(L, T, "tokens")
    g = synth.rng("ffn_prompt_masks", T)
    one = np.zeros(m, np.uint8)
    one[17] = 1
    with GpuLayer(pop, L, max_tokens=T, max_batch=1) as G:
        for mask in (np.ones(m, np.uint8), (g.random(m) < 0.4).astype(np.uint8), np.zeros(m, np.uint8), one,
                     (g.random((T, m)) < 0.5).astype(np.uint8)):
            y_ref = oracle.pruned_ffn(x, L.w_gate, L.w_up, L.w_down, BF16, mask)
            for ydtype in (F32, BF16):
                y = G.ffn(x, mask, ydtype)
                if not y_ref.any():
                    assert not y.any()
                else:
                    err = max_abs_rel(y, y_ref)
                    assert err <= (Y_TOL[BF16] if ydtype == BF16 else FFN_MFMA_TOL_F32), f"T={T} err {err:.3e}"
        # a second, smaller prompt on the same handle reuses the scratch
        y = G.ffn(x[:40], np.ones(m, np.uint8), F32)
        y_ref = oracle.pruned_ffn(x[:40], L.w_gate, L.w_up, L.w_down, BF16, np.ones(m, np.uint8))
        assert max_abs_rel(y, y_ref) <= FFN_MFMA_TOL_F32


@pytest.mark.parametrize("T", [70, 300])
def test_pruned_ffn_direct_load_gemm_step_counts(pop, oracle, T):
    """The down-projection GEMM whose operands go straight into a ring of LDS buffers (d a multiple of 128): numbers
    of active channels that give every split 0, 1, 2, 3 and more k-steps of 64 channels (the ring's first requests
    and its one- and two-step remainders), whole and ragged last k-steps, prompts of one ragged and of two token
    tiles; then a short list after a long one on the same handle (the columns behind a list's end hold the longer
    list's values, which meet rows of zeros)."""
    d, m = 256, 2000
    L = synth.make_layer(synth.small_config("ffn_direct_gemm", d, m, BF16))
    x = synth.make_activations(L, T, "tokens")
    g = synth.rng("ffn_direct_gemm_masks", T)
    with GpuLayer(pop, L, max_tokens=T, max_batch=1) as G:
        for a in (2000, 1, 64, 130, 700, 1100, 1500, 1536, 65):
            mask = np.zeros(m, np.uint8)
            mask[g.choice(m, size=a, replace=False)] = 1
            y_ref = oracle.pruned_ffn(x, L.w_gate, L.w_up, L.w_down, BF16, mask)
            y = G.ffn(x, mask, F32)
            err = max_abs_rel(y, y_ref)
            assert err <= FFN_MFMA_TOL_F32, f"T={T} a={a} err {err:.3e}"


def test_pruned_ffn_prompt_full_size(pop, oracle):
    """Llama-2-7B-shaped layer: the prompt's forward pass under the prefill mask (retained channels plus the best
    k candidates by prefill score), checked on a sample of tokens; and wider-than-one-tile shapes of the split
    contraction (T = 512: 4 splits; T = 2048: none)."""
    cfg, r, f_cand = synth.CFG2, 0.35, 0.10
    L = synth.make_layer(cfg, layer_id=0)
    m = cfg.m
    n_ret, n_cand, _ = pop.pop_region_counts(m, 1.0 - r - f_cand / 2, f_cand)
    k = pop.pop_k_for_ratio(m, r, n_ret, n_cand)
    for T in (512, 2048):
        x = synth.make_activations(L, T, "prompt")
        with GpuLayer(pop, L, max_tokens=T, max_batch=1) as G:
            scores, region, ret, cand = G.prefill(x, n_ret, n_cand)
            mask, sel, _ = oracle.select(region, scores[cand], cand, k)
            assert int(mask.sum()) == n_ret + k
            y = G.ffn(x, mask, F32)
            rows = np.sort(synth.rng("ffn_rows", T).choice(T, size=6, replace=False))
            y_ref = oracle.pruned_ffn(x[rows], L.w_gate, L.w_up, L.w_down, BF16, mask)
            err = max_abs_rel(y[rows], y_ref)
            assert err <= FFN_MFMA_TOL_F32, f"T={T} err {err:.3e}"


def _check_prefill_forward(oracle, G, L, x, n_ret, n_cand, k0, ydtype, y_tol, rows=None):
    """Whole prefilling stage in one call: scores and partition as in the two-call form; the prefill mask must be
    the oracle's selection on the GPU's own scores (retained + best k0 candidates by prefill score); y against the
    oracle's pruned FFN under that mask."""
    dtype = L.cfg.dtype
    scores, region, ret, cand, mask, y = G.prefill_forward(x, n_ret, n_cand, k0, ydtype)
    r1, ret1, cand1 = oracle.partition(scores, n_ret, n_cand)
    assert np.array_equal(region, r1) and np.array_equal(ret, ret1) and np.array_equal(cand, cand1)
    mask1, _, _ = oracle.select(region, scores[cand], cand, k0)
    assert np.array_equal(mask, mask1)
    assert int(mask.sum()) == n_ret + k0
    rows = np.arange(x.shape[0]) if rows is None else rows
    y_ref = oracle.pruned_ffn(x[rows], L.w_gate, L.w_up, L.w_down, dtype, mask)
    if not y_ref.any():
        assert not y[rows].any()
    else:
        err = max_abs_rel(y[rows], y_ref)
        assert err <= y_tol, f"prefill forward y error {err:.3e}"
    return scores, region, ret, cand


@pytest.mark.parametrize("dtype,T", [(F32, 40), (BF16, 20), (BF16, 150), (BF16, 290)])
def test_prefill_forward_small(pop, oracle, dtype, T):
    """Partition + pruned output of the prompt in one call: float32 and short prompts (decode kernels), bf16
    prompts of 32 tokens and more (kept H, gathered columns, matrix-core GEMM); degenerate region sizes; the
    partition it leaves serves the decode steps that follow."""
    d, m = (264, 301) if dtype == BF16 else (260, 301)
    L = synth.make_layer(synth.small_config("prefill_forward", d, m, dtype))
    x = synth.make_activations(L, T, "prompt")
    xt = synth.make_activations(L, 1, "decode")
    mfma = dtype == BF16 and T >= 32
    with GpuLayer(pop, L, max_tokens=T, max_batch=1) as G:
        for n_ret, n_cand, k0 in ((150, 60, 25), (150, 60, 0), (150, 60, 60), (0, 301, 100), (301, 0, 0), (0, 0, 0),
                                  (0, 40, 1)):
            for ydtype in (F32, dtype):
                tol = Y_TOL[BF16] if ydtype == BF16 else (FFN_MFMA_TOL_F32 if mfma else 1e-4)
                scores, region, ret, cand = _check_prefill_forward(oracle, G, L, x, n_ret, n_cand, k0, ydtype, tol)
            # same scores as the two-call form, bit for bit (the contraction is the same kernel)
            s2, region2, _, _ = G.prefill(x, n_ret, n_cand)
            assert np.array_equal(scores, s2) and np.array_equal(region, region2)
            _check_decode(oracle, G, L, region, cand, xt, min(k0, n_cand))


@pytest.mark.parametrize("cfg_name,T,r", [("CFG4", 1024, 0.50), ("CFG5", 300, 0.35)])
def test_prefill_forward_other_shapes(pop, oracle, cfg_name, T, r):
    """The prompt's forward pass on the Llama-2-13B-shaped layer (d = 5120: 40 column tiles, 4 token tiles, no
    split) and on a Mixtral-shaped expert with a ragged share of the prompt (128-token tiles, the last one short)."""
    cfg = getattr(synth, cfg_name)
    L = synth.make_layer(cfg, layer_id=0)
    m = cfg.m
    x = synth.make_activations(L, T, "prompt")
    n_ret, n_cand, k = pop.pop_strategy_counts(pop.POP_STRATEGY_POP, m, r, 0.10)
    rows = np.sort(synth.rng("prefill_forward_rows", cfg_name).choice(T, size=5, replace=False))
    rows[-1] = T - 1
    with GpuLayer(pop, L, max_tokens=T, max_batch=1) as G:
        _check_prefill_forward(oracle, G, L, x, n_ret, n_cand, k, BF16, Y_TOL[BF16], rows=rows)


@pytest.mark.parametrize("d,m,T", [(192, 301, 20), (128, 130, 150), (192, 301, 300), (320, 97, 257)])
def test_prefill_rows_of_whole_k_steps(pop, oracle, d, m, T):
    """bf16 layers whose rows are a whole number of 64-element k-steps take the prefill kernel's direct global -> LDS
    staging: every score against the oracle, with ragged token tiles, channel chunks that do not fill a tile, both
    tile forms and both token-tile sizes; then the forward pass (kept H, list form) and a decode step."""
    L = synth.make_layer(synth.small_config("whole_k_steps", d, m, BF16))
    x = synth.make_activations(L, T, "prompt")
    xt = synth.make_activations(L, 1, "decode")
    n_ret, n_cand, k = m // 2, m // 4, m // 8
    with GpuLayer(pop, L, max_tokens=T, max_batch=1) as G:
        scores, region, ret, cand, _ = _check_prefill(oracle, G, L, x, n_ret, n_cand)
        tol = FFN_MFMA_TOL_F32 if T >= 32 else 1e-4
        _check_prefill_forward(oracle, G, L, x, n_ret, n_cand, k, F32, tol)
        mask = (synth.rng("whole_k_steps_mask", d, m).random(m) < 0.5).astype(np.uint8)
        y = G.ffn(x, mask, F32)
        y_ref = oracle.pruned_ffn(x, L.w_gate, L.w_up, L.w_down, BF16, mask)
        assert max_abs_rel(y, y_ref) <= tol
        _check_decode(oracle, G, L, region, cand, xt, k)


def test_prefill_forward_full_size(pop, oracle):
    """Llama-2-7B-shaped layer, prompt 512: prefill scores on a sample of channels, partition and prefill mask
    on all channels, the prompt's output on a sample of tokens, then a decode step on the partition."""
    cfg, r, f_cand, T = synth.CFG2, 0.35, 0.10, 512
    L = synth.make_layer(cfg, layer_id=0)
    m = cfg.m
    x = synth.make_activations(L, T, "prompt")
    n_ret, n_cand, _ = pop.pop_region_counts(m, 1.0 - r - f_cand / 2, f_cand)
    k = pop.pop_k_for_ratio(m, r, n_ret, n_cand)
    rows = np.sort(synth.rng("prefill_forward_rows").choice(T, size=6, replace=False))
    with GpuLayer(pop, L, max_tokens=T, max_batch=1) as G:
        scores, region, ret, cand = _check_prefill_forward(oracle, G, L, x, n_ret, n_cand, k, F32, FFN_MFMA_TOL_F32,
                                                           rows=rows)
        sample = np.sort(synth.rng("full_size_sample", cfg.name).choice(m, size=64, replace=False)).astype(np.int32)
        H = oracle.hidden(x, L.w_gate, L.w_up, cfg.dtype, chan=sample)
        s_ref = oracle.importance(L.w_down, cfg.dtype, H, chan=sample)[sample]
        assert score_rel_err(scores[sample], s_ref, eps=1e-6) <= SCORE_TOL
        _check_decode(oracle, G, L, region, cand, synth.make_activations(L, 1, "decode_b1"), [k])


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_shared_batch_mask(pop, oracle, dtype):
    """B > 1 with one mask for the batch: candidate scores are Eq. 3 over the step's B activations (the literal
    double sum of the oracle), one selection, every sequence's output under that mask."""
    d, m, T, B = 264 if dtype == BF16 else 260, 301, 24, 5
    L = synth.make_layer(synth.small_config("shared_mask", d, m, dtype))
    x = synth.make_activations(L, T, "prompt")
    xt = synth.make_activations(L, B, "decode")
    n_ret, n_cand, k = 140, 90, 37
    with GpuLayer(pop, L, max_tokens=T, max_batch=8) as G:
        scores, region, ret, cand, _ = _check_prefill(oracle, G, L, x, n_ret, n_cand)
        pop.pop_layer_set_shared_batch_mask(G.handle, True)
        for one_call in (False, True):
            out = G.decode(xt, k, one_call=one_call)
            H = oracle.hidden(xt, L.w_gate, L.w_up, dtype)
            s_ref = oracle.importance(L.w_down, dtype, H)[cand]
            mask1, sel1, act1 = oracle.select(region, out["cscore"][0], cand, k)
            rc = region != 2
            for b in range(B):
                assert score_rel_err(out["cscore"][b], s_ref, eps=DECODE_FLOOR[dtype]) <= SCORE_TOL
                assert np.array_equal(out["cscore"][b], out["cscore"][0])
                assert score_rel_err(out["h"][b][rc], H[b][rc], eps=DECODE_FLOOR[dtype]) <= SCORE_TOL
                assert np.array_equal(out["mask"][b], mask1)
                assert out["n_active"][b] == n_ret + k
                assert np.array_equal(out["active_idx"][b][:n_ret + k], act1)
                y_ref = oracle.down(H[b:b + 1], L.w_down, dtype, mask1)[0]
                assert max_abs_rel(out["y"][b], y_ref) <= Y_TOL[dtype]
        # the aggregated score is not any single sequence's score
        per_seq = oracle.decode(xt[0], L.w_gate, L.w_up, L.w_down, dtype, region, cand, k, want_y=False)["cscore"]
        assert not np.allclose(per_seq, s_ref, rtol=1e-3)
        with pytest.raises(pop.PopError) as e:
            G.decode(xt, [k, k, k + 1, k, k])
        assert e.value.status == pop.POP_ESHAPE
        # one sequence: nothing to aggregate, the usual step
        _check_decode(oracle, G, L, region, cand, xt[:1], k)
        pop.pop_layer_set_shared_batch_mask(G.handle, False)
        _check_decode(oracle, G, L, region, cand, xt, k)


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_input_side_importance(pop, oracle, dtype):
    """The other reading of Eq. 1-2 (first projections and the FFN input): prefill scores and partition, decode
    steps that select first and then run the forward pass over retained + selected channels, per-sequence masks
    at B > 1, the prompt's pruned output; and back to the default reading on the same handle."""
    d, m, T = 264 if dtype == BF16 else 260, 301, 45
    L = synth.make_layer(synth.small_config("input_side", d, m, dtype))
    x = synth.make_activations(L, T, "prompt")
    xt = synth.make_activations(L, 3, "decode")
    n_ret, n_cand, k = 140, 90, 37
    with GpuLayer(pop, L, max_tokens=T, max_batch=4) as G:
        pop.pop_layer_set_importance(G.handle, pop.POP_IMPORTANCE_INPUT_SIDE)
        with pytest.raises(pop.PopError) as e:  # the partition of another reading is gone
            G.n_ret, G.n_cand = n_ret, n_cand
            G.decode(xt[:1], k)
        assert e.value.status == pop.POP_ESTATE
        scores, region, ret, cand = G.prefill(x, n_ret, n_cand)
        s_ref = oracle.importance_input_side(x, L.w_gate, L.w_up, dtype)
        assert score_rel_err(scores, s_ref, eps=1e-6) <= SCORE_TOL
        r1, ret1, cand1 = oracle.partition(scores, n_ret, n_cand)
        assert np.array_equal(region, r1) and np.array_equal(ret, ret1) and np.array_equal(cand, cand1)
        for xb, ks in ((xt[:1], [k]), (xt, [k, 0, n_cand])):
            for one_call in (False, True):
                out = G.decode(xb, ks, one_call=one_call)
                # one sequence: the fused kernel (it scores the candidates from the rows it reads for h); else launches
                kind, wgs = pop.pop_layer_step_kind(G.handle)  # (wgs: 0 where the fused kernel does not take the shape)
                assert kind == (1 if xb.shape[0] == 1 and wgs > 0 else 2)
                for b in range(xb.shape[0]):
                    c_ref = oracle.importance_input_side(xb[b:b + 1], L.w_gate, L.w_up, dtype, chan=cand)[cand]
                    assert score_rel_err(out["cscore"][b], c_ref, eps=1e-6) <= SCORE_TOL
                    mask1, sel1, act1 = oracle.select(region, out["cscore"][b], cand, ks[b])
                    assert np.array_equal(out["mask"][b], mask1)
                    assert out["n_active"][b] == n_ret + ks[b]
                    assert np.array_equal(out["active_idx"][b][:n_ret + ks[b]], act1)
                    active = np.flatnonzero(mask1).astype(np.int32)
                    H = oracle.hidden(xb[b:b + 1], L.w_gate, L.w_up, dtype, chan=active)
                    assert score_rel_err(out["h"][b][active], H[0][active], eps=DECODE_FLOOR[dtype]) <= SCORE_TOL
                    y_ref = oracle.down(H, L.w_down, dtype, mask1)[0]
                    assert max_abs_rel(out["y"][b], y_ref) <= Y_TOL[dtype]
        # the prompt's own forward pass under this reading's prefill mask
        tol = Y_TOL[BF16] if dtype == BF16 else 1e-4
        sc2, region2, _, cand2, mask, y = G.prefill_forward(x, n_ret, n_cand, 20, F32)
        assert np.array_equal(sc2, scores) and np.array_equal(region2, region)
        mask1, _, _ = oracle.select(region, scores[cand], cand, 20)
        assert np.array_equal(mask, mask1)
        y_ref = oracle.pruned_ffn(x, L.w_gate, L.w_up, L.w_down, dtype, mask)
        assert max_abs_rel(y, y_ref) <= (FFN_MFMA_TOL_F32 if dtype == BF16 else tol)
        # one mask for the batch: this reading's importance over the step's rows (s_k over tokens and samples)
        pop.pop_layer_set_shared_batch_mask(G.handle, True)
        with pytest.raises(pop.PopError) as e:
            G.decode(xt, [k, 0, n_cand])
        assert e.value.status == pop.POP_ESHAPE
        out = G.decode(xt, [k] * 3)
        c_ref = oracle.importance_input_side(xt, L.w_gate, L.w_up, dtype, chan=cand)[cand]
        mask1, _, act1 = oracle.select(region, out["cscore"][0], cand, k)
        for b in range(3):
            assert score_rel_err(out["cscore"][b], c_ref, eps=1e-6) <= SCORE_TOL
            assert np.array_equal(out["cscore"][b], out["cscore"][0])
            assert np.array_equal(out["mask"][b], mask1)
            assert np.array_equal(out["active_idx"][b][:n_ret + k], act1)
            active = np.flatnonzero(mask1).astype(np.int32)
            H = oracle.hidden(xt[b:b + 1], L.w_gate, L.w_up, dtype, chan=active)
            assert max_abs_rel(out["y"][b], oracle.down(H, L.w_down, dtype, mask1)[0]) <= Y_TOL[dtype]
        pop.pop_layer_set_shared_batch_mask(G.handle, False)
        # back to the default reading
        pop.pop_layer_set_importance(G.handle, pop.POP_IMPORTANCE_OUTPUT_SIDE)
        _, region_b, _, cand_b, _ = _check_prefill(oracle, G, L, x, n_ret, n_cand)
        assert not np.array_equal(region_b, region)
        _check_decode(oracle, G, L, region_b, cand_b, xt[:1], k)


def test_importance_reduce_standalone(pop, oracle):
    T, m = 77, 1000
    g = synth.rng("impred")
    H = g.standard_normal((T, m), dtype=np.float32)
    nrm = np.abs(g.standard_normal(m, dtype=np.float32)) + np.float32(0.1)
    ref = nrm.astype(np.float64) * np.sqrt((H.astype(np.float64) ** 2).sum(axis=0))
    # the oracle's importance with a one-row "down projection" holding the norms reproduces nrm_j * ||H[:,j]||
    ref2 = oracle.importance(nrm.reshape(1, m), F32, H.astype(np.float64))
    np.testing.assert_allclose(ref, ref2, rtol=1e-13)
    out = torch.empty(m, dtype=torch.float32, device="cuda")
    pop.pop_importance_reduce(dev(H), F32, T, m, dev(nrm), out)
    assert score_rel_err(host(out), ref2, eps=1e-9) <= SCORE_TOL
    Hb = synth.f32_to_bf16_bits(H)
    refb = oracle.importance(nrm.reshape(1, m), F32, synth.storage_to_f64(Hb, BF16))
    pop.pop_importance_reduce(dev(Hb), BF16, T, m, dev(nrm), out)
    assert score_rel_err(host(out), refb, eps=1e-9) <= SCORE_TOL


def test_importance_reduce_long_prompt_with_outliers(pop, oracle):
    """2048 tokens with a few columns a thousand times larger than the rest and a few tokens that dominate their
    column: the column sums must keep the 1e-5 of the scores (a float32 running sum would not)."""
    T, m = 2048, 1536
    g = synth.rng("impred_long")
    H = g.standard_normal((T, m), dtype=np.float32)
    H[:, ::97] *= np.float32(1000.0)
    H[5, ::13] *= np.float32(300.0)
    nrm = np.abs(g.standard_normal(m, dtype=np.float32)) + np.float32(0.1)
    out = torch.empty(m, dtype=torch.float32, device="cuda")
    ref = oracle.importance(nrm.reshape(1, m), F32, H.astype(np.float64))
    pop.pop_importance_reduce(dev(H), F32, T, m, dev(nrm), out)
    assert score_rel_err(host(out), ref, eps=1e-9) <= SCORE_TOL
    Hb = synth.f32_to_bf16_bits(H)
    refb = oracle.importance(nrm.reshape(1, m), F32, synth.storage_to_f64(Hb, BF16))
    pop.pop_importance_reduce(dev(Hb), BF16, T, m, dev(nrm), out)
    assert score_rel_err(host(out), refb, eps=1e-9) <= SCORE_TOL


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_prefill_without_tokens(pop, oracle, dtype):
    """T = 0 (an expert no prompt token was routed to): all scores zero, so the one total order falls back on the
    channel index: the first n_ret channels are retained, the next n_cand are candidates; decode steps then run on
    that partition as on any other.  The forward-pass form gives the same partition and the index-order mask."""
    d, m = (264, 301) if dtype == BF16 else (260, 301)
    L = synth.make_layer(synth.small_config("no_tokens", d, m, dtype))
    xt = synth.make_activations(L, 2, "decode")
    n_ret, n_cand, k = 120, 80, 33
    with GpuLayer(pop, L, max_tokens=8, max_batch=2) as G:
        scores, region, ret, cand = G.prefill(np.zeros((0, d), xt.dtype), n_ret, n_cand)
        assert not scores.any()
        r0, ret0, cand0 = oracle.partition(np.zeros(m, np.float32), n_ret, n_cand)
        assert np.array_equal(region, r0) and np.array_equal(ret, ret0) and np.array_equal(cand, cand0)
        assert np.array_equal(ret, np.arange(n_ret)) and np.array_equal(cand, n_ret + np.arange(n_cand))
        _check_decode(oracle, G, L, region, cand, xt[:1], k)
        _check_decode(oracle, G, L, region, cand, xt, [k, 0])
        sc2, region2, _, _, mask, _ = G.prefill_forward(np.zeros((0, d), xt.dtype), n_ret, n_cand, k)
        assert not sc2.any() and np.array_equal(region2, region)
        assert np.array_equal(mask, (np.arange(m) < n_ret + k).astype(np.uint8))


def test_forward_pass_scratch_poisoned_and_side_stream(pop, oracle):
    """The prompt-sized forward pass on a non-blocking side stream (scratch reserved ahead, so the calls only enqueue),
    and a short channel list right after a call whose compact H holds non-finite values: the columns the GEMM reads
    beyond the short list's end must not keep them."""
    d, m, T = 256, 2000, 96
    L = synth.make_layer(synth.small_config("ffn_poison", d, m, BF16))
    x = synth.make_activations(L, T, "tokens")
    xbad = x.copy()
    xbad[:, ::3] = 0x7F80  # +inf in bf16: H of every channel becomes non-finite
    g = synth.rng("ffn_poison_masks")
    side = torch.cuda.Stream()
    with GpuLayer(pop, L, max_tokens=T, max_batch=1) as G:
        with torch.cuda.stream(side):
            pop.pop_layer_reserve_prompt(G.handle, T, stream=side)
            G.ffn(xbad, np.ones(m, np.uint8), F32)  # fills compact H with inf / nan over all 2000 columns
            for a in (65, 1, 130, 1999):
                mask = np.zeros(m, np.uint8)
                mask[g.choice(m, size=a, replace=False)] = 1
                y = G.ffn(x, mask, F32)
                y_ref = oracle.pruned_ffn(x, L.w_gate, L.w_up, L.w_down, BF16, mask)
                assert np.isfinite(y).all(), a
                assert max_abs_rel(y, y_ref) <= FFN_MFMA_TOL_F32, a
            # the one-call prefilling stage on the same stream, after a poisoned one
            n_ret, n_cand, k0 = 900, 300, 77
            G.prefill_forward(xbad, n_ret, n_cand, k0, F32)
            _check_prefill_forward(oracle, G, L, x, n_ret, n_cand, k0, F32, FFN_MFMA_TOL_F32)
            side.synchronize()


@pytest.mark.parametrize("B", [1, 4])
def test_one_call_step_replays_from_a_graph(pop, B):
    """The one-call step keeps no per-launch state on the host (B = 1: fused kernel and tail kernel; B = 4: the
    gate/up launch with the selection inside, whose counters are never rewound, the down projection and its
    reduction): a captured step is replayed several times, with eager steps in between, and every replay must
    reproduce the eager result bit for bit."""
    d, m, T = 512, 1024, 32
    L = synth.make_layer(synth.small_config("graph_replay", d, m, BF16, n_outlier=2, heavy_tail=True))
    x = synth.make_activations(L, T, "prompt")
    xt = synth.make_activations(L, 3 * B, "decode")
    n_ret, n_cand, _ = pop.pop_region_counts(m, 0.55, 0.1)
    k = [n_cand // 2, n_cand // 3, n_cand // 2 + 1, n_cand // 4][:B]
    with GpuLayer(pop, L, max_tokens=T, max_batch=B) as G:
        G.prefill(x, n_ret, n_cand)
        side = torch.cuda.Stream()
        xs = [dev(xt[i * B:(i + 1) * B]) for i in range(3)]
        y_eager = [torch.zeros((B, d), dtype=torch.int16, device="cuda") for _ in range(3)]
        y_graph = torch.zeros((B, d), dtype=torch.int16, device="cuda")
        with torch.cuda.stream(side):
            for i in range(3):
                pop.pop_decode_step(G.handle, xs[i], B, k, y_eager[i], BF16, stream=side)
            side.synchronize()
            assert pop.pop_layer_step_kind(G.handle)[0] == (1 if B == 1 else 2)
            x_in = xs[0].clone()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                pop.pop_decode_step(G.handle, x_in, B, k, y_graph, BF16, stream=torch.cuda.current_stream())
            for rep in range(6):
                i = rep % 3
                x_in.copy_(xs[i])
                y_graph.fill_(777)
                g.replay()
                torch.cuda.synchronize()
                assert torch.equal(y_graph, y_eager[i]), f"replay {rep}"
                # the program's own eager work between replays
                y_tmp = torch.zeros((B, d), dtype=torch.int16, device="cuda")
                pop.pop_decode_step(G.handle, xs[(i + 1) % 3], B, k, y_tmp, BF16, stream=torch.cuda.current_stream())
                torch.cuda.synchronize()
                assert torch.equal(y_tmp, y_eager[(i + 1) % 3])
            pop.pop_layer_sync_status(G.handle)


@pytest.mark.parametrize("dtype", [BF16, F32])
def test_expired_waits_flag_the_step_and_leave_the_next_one_alone(pop, oracle, dtype):
    """Every bounded wait of the fused step gives up at once (wait limit 0, set from the host): all kernels still
    exit, the step is reported as invalid (POP_EDEVICE), the report clears the record, and with the limit restored
    the following steps are bit-identical to the steps of a fresh layer: nothing of the abandoned step (candidate
    words, selection words, partial rows, counters) is taken for valid later."""
    d, m, T = 512, 768, 40
    L = synth.make_layer(synth.small_config("expired_waits", d, m, dtype, n_outlier=2, heavy_tail=dtype == BF16))
    x = synth.make_activations(L, T, "prompt")
    xt = synth.make_activations(L, 4, "decode")
    n_ret, n_cand, _ = pop.pop_region_counts(m, 0.6, 0.1)
    k = n_cand // 2
    with GpuLayer(pop, L, max_tokens=T, max_batch=1) as G:
        scores, region, ret, cand, _ = _check_prefill(oracle, G, L, x, n_ret, n_cand)
        fresh = [G.decode(xt[t:t + 1], k) for t in range(4)]
        assert pop.pop_layer_step_kind(G.handle)[0] == 1
    with GpuLayer(pop, L, max_tokens=T, max_batch=1) as G:
        G.prefill(x, n_ret, n_cand)
        assert np.array_equal(G.decode(xt[:1], k)["y"], fresh[0]["y"])
        pop.pop_layer_set_wait_limit(G.handle, 0)
        y = torch.zeros(d, dtype=torch.float32, device="cuda")
        flagged = 0
        for t in (1, 2):  # steps whose waits all give up at once (some may find their data in time: also fine)
            pop.pop_decode_step(G.handle, dev(xt[t:t + 1]), 1, [k], y, F32)
            torch.cuda.synchronize()  # the kernels came back
            try:
                pop.pop_layer_sync_status(G.handle)
            except pop.PopError as e:
                assert e.status == pop.POP_EDEVICE
                flagged += 1
                pop.pop_layer_sync_status(G.handle)  # reported once
        assert flagged >= 1, "with no patience at all, at least one of the steps has to miss a hand-over"
        pop.pop_layer_set_wait_limit(G.handle, 1 << 16)
        for t in range(4):
            again = G.decode(xt[t:t + 1], k)  # (raises if the step was flagged)
            for key in ("mask", "n_active", "cscore", "y"):
                assert np.array_equal(again[key], fresh[t][key]), (t, key)
            assert np.array_equal(again["active_idx"][:, :n_ret + k], fresh[t]["active_idx"][:, :n_ret + k]), t
        _check_decode(oracle, G, L, region, cand, xt[3:4], k)
        with pytest.raises(pop.PopError) as e:
            pop.pop_layer_set_wait_limit(G.handle, -1)
        assert e.value.status == pop.POP_EINVAL


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_expired_wait_of_a_batched_step_leaves_the_next_one_alone(pop, oracle, dtype):
    """B > 1: the selecting workgroups of the step's first launch wait for the candidates' scores.  With a wait limit
    of 0 (set from the host) they give up at once: every kernel still exits, the step is reported as invalid
    (POP_EDEVICE, once), and with the limit restored the following steps - same and other batch sizes - are
    bit-identical to those of a fresh layer: the arrival counters agree again without anybody rewinding them."""
    d, m, T, B = 512, 768, 40, 4
    L = synth.make_layer(synth.small_config("expired_batch", d, m, dtype, n_outlier=2, heavy_tail=dtype == BF16))
    x = synth.make_activations(L, T, "prompt")
    xt = synth.make_activations(L, 4 * B, "decode")
    n_ret, n_cand, _ = pop.pop_region_counts(m, 0.6, 0.1)
    k = [n_cand // 2, n_cand // 3, n_cand, 0]
    steps = [(0, B), (B, B), (2 * B, 3), (3 * B, B)]  # (first row of xt, sequences)
    with GpuLayer(pop, L, max_tokens=T, max_batch=B) as G:
        scores, region, ret, cand, _ = _check_prefill(oracle, G, L, x, n_ret, n_cand)
        fresh = [G.decode(xt[t0:t0 + b], k[:b], one_call=True) for t0, b in steps]
    with GpuLayer(pop, L, max_tokens=T, max_batch=B) as G:
        G.prefill(x, n_ret, n_cand)
        pop.pop_layer_set_wait_limit(G.handle, 0)
        y = torch.zeros((B, d), dtype=torch.float32, device="cuda")
        flagged = 0
        for t in (1, 2):
            pop.pop_decode_step(G.handle, dev(xt[t * B:(t + 1) * B]), B, k, y, F32)
            torch.cuda.synchronize()  # the kernels came back
            try:
                pop.pop_layer_sync_status(G.handle)
            except pop.PopError as e:
                assert e.status == pop.POP_EDEVICE
                flagged += 1
                pop.pop_layer_sync_status(G.handle)  # reported once
        assert flagged >= 1, "with no patience at all a selector cannot have found every score in place"
        pop.pop_layer_set_wait_limit(G.handle, 1 << 16)
        for (t0, b), ref in zip(steps, fresh):
            again = G.decode(xt[t0:t0 + b], k[:b], one_call=True)  # (raises if the step was flagged)
            for key in ("mask", "n_active", "cscore", "y"):
                assert np.array_equal(again[key], ref[key]), (t0, key)
            for q in range(b):
                assert np.array_equal(again["active_idx"][q, :n_ret + k[q]], ref["active_idx"][q, :n_ret + k[q]])
        _check_decode(oracle, G, L, region, cand, xt[:B], k)


def test_determinism_and_poisoned_scratch(pop, oracle):
    """Two identical step sequences give bit-identical outputs, also after other work dirtied the scratch."""
    d, m, T = 512, 700, 64
    L = synth.make_layer(synth.small_config("determinism", d, m, BF16))
    x = synth.make_activations(L, T, "prompt")
    xt = synth.make_activations(L, 4, "decode")
    n_ret, n_cand, _ = pop.pop_region_counts(m, 0.55, 0.1)
    k = pop.pop_k_for_ratio(m, 0.4, n_ret, n_cand)
    with GpuLayer(pop, L, max_tokens=T, max_batch=4) as G:
        a = G.prefill(x, n_ret, n_cand)
        o1 = G.decode(xt, k)
        # dirty the scratch with a different call pattern, then repeat
        G.ffn(xt, (synth.rng("dirty").random((4, m)) < 0.9).astype(np.uint8))
        G.prefill(synth.make_activations(L, T, "other_prompt"), n_ret // 2, n_cand)
        b = G.prefill(x, n_ret, n_cand)
        o2 = G.decode(xt, k)
        for u, v in zip(a, b):
            assert np.array_equal(u, v)
        rc = a[1] != 2  # h is defined on retained and candidate channels only
        for key in o1:
            if key == "h":
                assert np.array_equal(o1[key][:, rc], o2[key][:, rc]), key
            else:
                assert np.array_equal(o1[key], o2[key]), key
        # single-sequence steps (fused kernel): bit-identical y as well
        s1 = G.decode(xt[:1], k)
        G.ffn(xt, (synth.rng("dirty2").random((4, m)) < 0.5).astype(np.uint8))
        G.prefill(x, n_ret, n_cand)
        s2 = G.decode(xt[:1], k)
        for key in s1:
            sel = (slice(None), rc) if key == "h" else slice(None)
            assert np.array_equal(s1[key][sel], s2[key][sel]), key


def test_error_paths(pop):
    d, m = 64, 40
    L = synth.make_layer(synth.small_config("errors", d, m, F32))
    E = pop.PopError

    def status(fn, *a, **kw):
        with pytest.raises(E) as e:
            fn(*a, **kw)
        return e.value.status

    wg, wu, wd = dev(L.w_gate), dev(L.w_up), dev(L.w_down)
    assert status(pop.pop_layer_create, d, m, 7, wg, wu, wd, 8, 1) == pop.POP_EINVAL
    assert status(pop.pop_layer_create, d, m, F32, None, wu, wd, 8, 1) == pop.POP_EINVAL
    assert status(pop.pop_layer_create, d, m, F32, wg, wu, wd, 8, 9) == pop.POP_ESHAPE
    assert status(pop.pop_layer_create, d, m, F32, wg, wu, wd, 0, 1) == pop.POP_ESHAPE
    assert status(pop.pop_layer_create, 62, m, F32, wg, wu, wd, 8, 1) == pop.POP_EUNSUPPORTED
    assert status(pop.pop_layer_create, 68, m, BF16, wg, wu, wd, 8, 1) == pop.POP_EUNSUPPORTED
    with GpuLayer(pop, L, max_tokens=8, max_batch=2) as G:
        x = dev(synth.make_activations(L, 8, "p"))
        y = torch.empty((2, d), dtype=torch.float32, device="cuda")
        assert status(pop.pop_decode_mask, G.handle, x, 1, 1) == pop.POP_ESTATE
        assert status(pop.pop_pruned_ffn, G.handle, None, 1, None, 0, y, F32) == pop.POP_ESTATE
        assert status(pop.pop_prefill_partition, G.handle, x, 9, 10, 10) == pop.POP_ESHAPE
        assert status(pop.pop_prefill_partition, G.handle, x, -1, 10, 10) == pop.POP_ESHAPE
        assert status(pop.pop_layer_reserve_prompt, G.handle, 9) == pop.POP_ESHAPE
        assert status(pop.pop_layer_reserve_prompt, None, 4) == pop.POP_EINVAL
        assert status(pop.pop_prefill_partition, G.handle, x, 8, 30, 11) == pop.POP_ESHAPE
        assert status(pop.pop_prefill_partition, G.handle, x, 8, -1, 11) == pop.POP_ESHAPE
        assert status(pop.pop_prefill_partition, G.handle, None, 8, 10, 10) == pop.POP_EINVAL
        pop.pop_prefill_partition(G.handle, x, 8, 10, 10)
        assert status(pop.pop_decode_mask, G.handle, x, 3, 1) == pop.POP_ESHAPE
        assert status(pop.pop_decode_mask, G.handle, x, 1, 11) == pop.POP_ESHAPE
        assert status(pop.pop_decode_mask, G.handle, x, 2, [1, -1]) == pop.POP_ESHAPE
        pop.pop_decode_mask(G.handle, x, 2, [3, 4])
        assert status(pop.pop_pruned_ffn, G.handle, None, 1, None, 0, y, F32) == pop.POP_ESHAPE
        assert status(pop.pop_pruned_ffn, G.handle, None, 2, None, 0, y, 5) == pop.POP_EINVAL
        pop.pop_pruned_ffn(G.handle, None, 2, None, 0, y, F32)
        mask = torch.ones((2, m), dtype=torch.uint8, device="cuda")
        assert status(pop.pop_pruned_ffn, G.handle, x, 4, mask, 2, y, F32) == pop.POP_ESHAPE
        assert status(pop.pop_pruned_ffn, G.handle, None, 2, mask, 2, y, F32) == pop.POP_EINVAL
        y8 = torch.empty((8, d), dtype=torch.float32, device="cuda")
        assert status(pop.pop_prefill_forward, G.handle, x, 8, 10, 10, 11, y8, F32) == pop.POP_ESHAPE
        assert status(pop.pop_prefill_forward, G.handle, x, 8, 10, 10, -1, y8, F32) == pop.POP_ESHAPE
        assert status(pop.pop_prefill_forward, G.handle, x, 9, 10, 10, 5, y8, F32) == pop.POP_ESHAPE
        assert status(pop.pop_prefill_forward, G.handle, x, 8, 10, 10, 5, None, F32) == pop.POP_EINVAL
        assert status(pop.pop_prefill_forward, G.handle, x, 8, 10, 10, 5, y8, 3) == pop.POP_EINVAL
        # misaligned activations or outputs are rejected on the host (the kernels use 16-byte accesses)
        xb = torch.zeros(8 * d + 4, dtype=torch.float32, device="cuda")
        assert status(pop.pop_prefill_partition, G.handle, xb.data_ptr() + 4, 8, 10, 10) == pop.POP_EINVAL
        assert status(pop.pop_decode_mask, G.handle, xb.data_ptr() + 8, 1, 1) == pop.POP_EINVAL
        assert status(pop.pop_pruned_ffn, G.handle, None, 2, None, 0, y.data_ptr() + 4, F32) == pop.POP_EINVAL
        assert status(pop.pop_layer_set_importance, G.handle, 2) == pop.POP_EINVAL
        assert status(pop.pop_layer_set_importance, None, 0) == pop.POP_EINVAL
        assert status(pop.pop_layer_set_shared_batch_mask, None, 1) == pop.POP_EINVAL
        # a failed call leaves the earlier partition usable
        pop.pop_decode_mask(G.handle, x, 2, [3, 4])
        torch.cuda.synchronize()
    s = torch.zeros(10, dtype=torch.float32, device="cuda")
    assert status(pop.pop_partition_from_scores, s, 10, 6, 5) == pop.POP_ESHAPE
    assert status(pop.pop_partition_from_scores, None, 10, 6, 4) == pop.POP_EINVAL
    assert status(pop.pop_partition_top_from_scores, s, 10, 6, 4, 11, None, None, None, None, s) == pop.POP_ESHAPE
    assert status(pop.pop_partition_top_from_scores, s, 10, 6, 4, 5, None, None, None, None, None) == pop.POP_EINVAL
    assert status(pop.pop_topk_from_scores, s, None, 10, 3, None, 10) == pop.POP_EINVAL
    assert status(pop.pop_topk_from_scores, s, s, 10, 11, None, 10) == pop.POP_ESHAPE


# ---------------------------------------------------------------- benchmark configurations

def test_config1_small_fp32(pop, oracle):
    """d=512, m=1376, float32, prompt 64, regions .3/.4/.3, top-k keeps half the candidates, 16 decode steps."""
    cfg = synth.CFG1
    L = synth.make_layer(cfg)
    x = synth.make_activations(L, 64, "prompt")
    xt = synth.make_activations(L, 16, "decode")
    n_ret, n_cand, n_prn = pop.pop_region_counts(cfg.m, 0.3, 0.4)
    assert (n_ret, n_cand, n_prn) == (413, 550, 413)
    k = n_cand // 2
    with GpuLayer(pop, L, max_tokens=64, max_batch=1) as G:
        scores, region, ret, cand, _ = _check_prefill(oracle, G, L, x, n_ret, n_cand)
        for t in range(16):
            out = _check_decode(oracle, G, L, region, cand, xt[t:t + 1], k)
            assert out["mask"].sum() == n_ret + k
        # 0 % pruning reproduces the dense FFN
        y = G.ffn(xt, np.ones(cfg.m, np.uint8))
        dense = oracle.pruned_ffn(xt, L.w_gate, L.w_up, L.w_down, F32, np.ones(cfg.m, np.uint8))
        assert max_abs_rel(y, dense) <= 1e-4


# ---------------------------------------------------------------- full-size shapes, sampled against the oracle

def _full_size_case(pop, oracle, cfg, T, r, batches, n_sample=192, f_cand=0.10):
    """Layer of a benchmark shape at full size, in the launch configuration bench.py uses.  Prefill scores are
    checked on a sample of channels (the oracle computes them one by one), the partition on all channels (GPU
    scores through the oracle's selector), decode steps completely (one token of the oracle is cheap)."""
    L = synth.make_layer(cfg, layer_id=0)
    dtype, m = cfg.dtype, cfg.m
    x = synth.make_activations(L, T, "prompt")
    n_ret, n_cand, _ = pop.pop_region_counts(m, 1.0 - r - f_cand / 2, f_cand)
    k = pop.pop_k_for_ratio(m, r, n_ret, n_cand)
    with GpuLayer(pop, L, max_tokens=T, max_batch=max(batches)) as G:
        scores, region, ret, cand = G.prefill(x, n_ret, n_cand)
        sample = np.sort(synth.rng("full_size_sample", cfg.name).choice(m, size=n_sample, replace=False)).astype(np.int32)
        H = oracle.hidden(x, L.w_gate, L.w_up, dtype, chan=sample)
        s_ref = oracle.importance(L.w_down, dtype, H, chan=sample)[sample]
        err = score_rel_err(scores[sample], s_ref, eps=1e-6)
        assert err <= SCORE_TOL, f"prefill score error {err:.3e}"
        r1, ret1, cand1 = oracle.partition(scores, n_ret, n_cand)
        assert np.array_equal(region, r1) and np.array_equal(ret, ret1) and np.array_equal(cand, cand1)
        for B in batches:
            xt = synth.make_activations(L, B, f"decode_b{B}")
            ks = [k] * B if B == 1 else [max(0, min(n_cand, k + 7 * b - 11)) for b in range(B)]
            _check_decode(oracle, G, L, region, cand, xt, ks)


def test_config2_llama7b_layer_full_size(pop, oracle):
    """Llama-2-7B-shaped layer, bf16, prompt 512, B = 1, sparsity .20 / .35 / .50 (fused decode kernel)."""
    for r in (0.35, 0.20, 0.50):
        _full_size_case(pop, oracle, synth.CFG2, 512, r, [1], n_sample=128)


def test_config3_long_prompt_full_size(pop, oracle):
    """Same shape with the 2048-token prompt of the 32-layer stack configuration (one layer of it)."""
    _full_size_case(pop, oracle, synth.CFG3, 2048, 0.35, [1], n_sample=48)


def test_config4_llama13b_layer_batched_full_size(pop, oracle):
    """Llama-2-13B-shaped layer, bf16, prompt 1024, decode at B = 1, 4, 8 with per-sequence masks."""
    _full_size_case(pop, oracle, synth.CFG4, 1024, 0.50, [1, 4, 8], n_sample=64)


def test_config5_mixtral_expert_full_size(pop, oracle):
    """One Mixtral-shaped expert (d 4096, m 14336), bf16, a ragged share of the prompt tokens, sparsity .35."""
    _full_size_case(pop, oracle, synth.CFG5, 300, 0.35, [1], n_sample=128)


# ---------------------------------------------------------------- mixture-of-experts layer (harness-side routing)

def _route_top2(logits: np.ndarray):
    """Top-2 experts per token (ties to the lower index) and the softmax over those two logits.  The router is
    not part of the pruned-FFN path: it lives in the harness, on both sides of the comparison."""
    order = np.argsort(-logits.astype(np.float64), axis=1, kind="stable")[:, :2]
    top = np.take_along_axis(logits.astype(np.float64), order, axis=1)
    e = np.exp(top - top.max(axis=1, keepdims=True))
    return order, e / e.sum(axis=1, keepdims=True)


def _moe_case(pop, oracle, cfg, n_experts, T, steps, r, n_sample, f_cand=0.10):
    """One MoE layer: every expert is an independent pruned FFN with its own partition, made from the prompt
    tokens routed to it (not weighted by the router); a decode token runs its two experts' steps and the outputs
    are combined with the router weights.  Each expert step is checked as in the single-layer tests, the combined
    output against the oracle's combined output."""
    dtype, m, d = cfg.dtype, cfg.m, cfg.d
    experts = [synth.make_layer(cfg, layer_id=100 + e) for e in range(n_experts)]
    x = synth.make_activations(experts[0], T, "moe_prompt")
    xt = synth.make_activations(experts[0], steps, "moe_decode")
    route_p, _ = _route_top2(synth.make_router_logits(cfg, T, n_experts, "prompt"))
    route_d, prob_d = _route_top2(synth.make_router_logits(cfg, steps, n_experts, "decode"))
    n_ret, n_cand, _ = pop.pop_region_counts(m, 1.0 - r - f_cand / 2, f_cand)
    k = pop.pop_k_for_ratio(m, r, n_ret, n_cand)
    layers, parts = [], []
    try:
        for e, L in enumerate(experts):
            tok = np.flatnonzero((route_p == e).any(axis=1))
            G = GpuLayer(pop, L, max_tokens=max(len(tok), 1), max_batch=1)
            layers.append(G)
            if len(tok) == 0:  # an expert nobody was routed to: all-zero scores, partition by channel order
                scores, region, ret, cand = G.prefill(np.zeros((0, d), x.dtype), n_ret, n_cand)
                assert not scores.any()
                assert np.array_equal(ret, np.arange(n_ret)) and np.array_equal(cand, n_ret + np.arange(n_cand))
                parts.append((region, cand))
                continue
            xe = np.ascontiguousarray(x[tok])
            scores, region, ret, cand = G.prefill(xe, n_ret, n_cand)
            sample = np.sort(synth.rng("moe_sample", e).choice(m, size=n_sample, replace=False)).astype(np.int32)
            H = oracle.hidden(xe, L.w_gate, L.w_up, dtype, chan=sample)
            s_ref = oracle.importance(L.w_down, dtype, H, chan=sample)[sample]
            assert score_rel_err(scores[sample], s_ref, eps=1e-6) <= SCORE_TOL
            r1, ret1, cand1 = oracle.partition(scores, n_ret, n_cand)
            assert np.array_equal(region, r1) and np.array_equal(ret, ret1) and np.array_equal(cand, cand1)
            parts.append((region, cand))
        assert len({p[0].tobytes() for p in parts}) == n_experts  # the experts' partitions really differ
        for t in range(steps):
            y_gpu = np.zeros(d)
            y_ref = np.zeros(d)
            for slot in range(2):
                e = int(route_d[t, slot])
                region, cand = parts[e]
                out = _check_decode(oracle, layers[e], experts[e], region, cand, xt[t:t + 1], k, ydtype=F32)
                ref = oracle.decode(xt[t], experts[e].w_gate, experts[e].w_up, experts[e].w_down, dtype, region, cand,
                                    k, want_y=False)
                y_e = oracle.down(ref["h"].reshape(1, -1), experts[e].w_down, dtype, out["mask"][0])[0]
                y_gpu += prob_d[t, slot] * out["y"][0]
                y_ref += prob_d[t, slot] * y_e
            assert max_abs_rel(y_gpu, y_ref) <= Y_TOL[dtype]
    finally:
        for G in layers:
            G.close()


def test_moe_layer_small(pop, oracle):
    """Four small experts, top-2 routing: every expert gets its own partition from its own tokens."""
    _moe_case(pop, oracle, synth.small_config("moe_small", 512, 640, BF16, n_outlier=2, heavy_tail=True), 4, 96, 4,
              0.35, n_sample=40)


def test_config5_mixtral_moe_layer_full_size(pop, oracle):
    """Mixtral-shaped MoE layer: 8 experts (d 4096, m 14336, bf16), top-2 softmax router over random logits, prompt
    1024, sparsity .35 per expert; a few of the 128 decode steps."""
    _moe_case(pop, oracle, synth.CFG5, 8, 1024, 4, 0.35, n_sample=24)


def test_config3_stack_of_layers(pop, oracle):
    """A stack of Llama-2-7B-shaped layers with independent weights, inputs and partitions, run back to back on one
    stream as the decode loop of the 32-layer configuration does (4 layers here; the layers are independent, so
    more of them add time, not coverage).  Every layer's step is checked against the oracle."""
    cfg = synth.CFG3
    r, f_cand, T = 0.35, 0.10, 256
    n_ret, n_cand, _ = pop.pop_region_counts(cfg.m, 1.0 - r - f_cand / 2, f_cand)
    k = pop.pop_k_for_ratio(cfg.m, r, n_ret, n_cand)
    stack = []
    try:
        for li in range(4):
            L = synth.make_layer(cfg, layer_id=li)
            G = GpuLayer(pop, L, max_tokens=T, max_batch=1)
            stack.append((L, G))
            scores, region, ret, cand = G.prefill(synth.make_activations(L, T, "prompt", li), n_ret, n_cand)
            r1, ret1, cand1 = oracle.partition(scores, n_ret, n_cand)
            assert np.array_equal(region, r1) and np.array_equal(ret, ret1) and np.array_equal(cand, cand1)
            G.part = (region, cand)
        assert len({G.part[0].tobytes() for _, G in stack}) == len(stack)  # per-layer independent partitions
        for t in range(2):
            for li, (L, G) in enumerate(stack):
                xt = synth.make_activations(L, 2, "decode", li)[t:t + 1]
                _check_decode(oracle, G, L, G.part[0], G.part[1], xt, k)
    finally:
        for _, G in stack:
            G.close()
