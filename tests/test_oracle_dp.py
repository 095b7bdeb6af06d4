"""Pins of the oracle's layer-skip dynamic program and of the decode loops (CPU only).

What the paper fixes and these tests check (Eq. 2, Algorithm 1, Sec. 3.1, the lossless claim of the abstract):
  * a direct top-down evaluation of the recurrence, without any table, reproduces every score and choice;
  * the backtracked skip set has exactly M layers, and replaying it layer by layer from x_0 reproduces g(L, M);
  * structural facts: g(i,i) = x_0, choice(1,1) = skip, M = 0 gives the empty set and g = x_L, M = L skips all;
  * degenerate models: identity layers tie every comparison (ties skip) so the last M layers are skipped; a single
    active layer is never skipped;
  * brute force over all C(L, M) skip sets is an upper bound on D(L, M);
  * greedy speculative decoding emits exactly the tokens of plain greedy decoding.
"""
import itertools

import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import clasp_oracle as oc
from tests.helpers import oracle_model, prompt, torch_model


def _np_cos(a, b):
    return float(a @ b / (max(np.sqrt(a @ a), 1e-12) * max(np.sqrt(b @ b), 1e-12)))


def _setup(name, T, resid_scale=1.0, seed=1):
    om = oracle_model(name, seed, resid_scale)
    shape = om.shape
    cache = oc.KVCache(shape, T + 2)
    states, _ = om.prefill(prompt(shape, T), cache)
    return om, shape, cache, states


def _replay(om, cache, x0, mask, pos):
    """Run x_0 through the layers a skip set keeps, in the DP's context (prefix 0..pos-1 plus own k/v)."""
    h = x0.copy()
    for l in range(om.shape.n_layers):
        if not mask[l]:
            h, _, _ = om.layer(l, h, pos, pos, cache.K[l], cache.V[l])
    return h


@pytest.mark.parametrize("resid_scale", [1.0, 0.05])
def test_recursive_evaluation_reproduces_the_table(resid_scale):
    T, M = 9, 3
    om, shape, cache, X = _setup("tiny-f32", T, resid_scale)
    L, pos = shape.n_layers, T - 1
    res = om.dp(X, pos, cache, M)

    def g(i, j):
        """g(i, j) by Eq. 2 taken literally: returns (state, score of computed, score of skip, choice)."""
        if j == 0:
            return X[i], None, None, None
        if j == i:  # every one of the first i layers skipped
            return X[0], None, _np_cos(X[0], X[i]), 1
        comp, _, _ = om.layer(i - 1, g(i - 1, j)[0], pos, pos, cache.K[i - 1], cache.V[i - 1])
        skip = g(i - 1, j - 1)[0]
        sc, ss = _np_cos(comp, X[i]), _np_cos(skip, X[i])
        return (comp, sc, ss, 0) if sc > ss else (skip, sc, ss, 1)

    for i in range(1, L + 1):
        for j in range(1, min(i, M) + 1):
            _, sc, ss, ch = g(i, j)
            assert res["choice"][i, j] == ch, (i, j)
            assert res["sigma_s"][i, j] == pytest.approx(ss, abs=1e-12)
            if j < i:
                assert res["sigma_c"][i, j] == pytest.approx(sc, abs=1e-12)
            else:
                assert np.isnan(res["sigma_c"][i, j])
    np.testing.assert_allclose(res["g_final"], g(L, M)[0], rtol=0, atol=1e-12)
    # cells outside the table
    assert (res["choice"][:, 0] == 255).all() and res["choice"][2, 3] == 255


@pytest.mark.parametrize("name,M,resid_scale", [("tiny-f32", 3, 1.0), ("tiny-f32", 5, 0.05), ("small-bf16", 2, 0.05),
                                               ("small-bf16", 4, 1.0)])
def test_backtracked_set_has_M_layers_and_replays_to_g(name, M, resid_scale):
    T = 7
    om, shape, cache, X = _setup(name, T, resid_scale)
    L, pos = shape.n_layers, T - 1
    res = om.dp(X, pos, cache, M)
    assert int(res["mask"].sum()) == M
    rep = _replay(om, cache, X[0], res["mask"], pos)
    assert np.array_equal(rep, res["g_final"])
    d_lm = np.nanmax([res["sigma_c"][L, M], res["sigma_s"][L, M]])
    assert _np_cos(rep, X[L]) == pytest.approx(d_lm, abs=1e-12)


def test_structural_facts():
    T = 6
    om, shape, cache, X = _setup("tiny-f32", T)
    L, pos = shape.n_layers, T - 1
    r0 = om.dp(X, pos, cache, 0)
    assert not r0["mask"].any() and np.array_equal(r0["g_final"], X[L])
    rL = om.dp(X, pos, cache, L)
    assert rL["mask"].all() and np.array_equal(rL["g_final"], X[0])
    for i in range(1, L + 1):
        assert rL["choice"][i, i] == 1
        assert rL["sigma_s"][i, i] == pytest.approx(_np_cos(X[0], X[i]), abs=1e-12)
    assert rL["choice"][1, 1] == 1 and np.isnan(rL["sigma_c"][1, 1])  # layer 0 is never evaluated at i = 1
    # the stored states are the full model's own trajectory: x_{l+1} = f_l(x_l) in the DP's context
    for l in range(L):
        out, _, _ = om.layer(l, X[l], pos, pos, cache.K[l], cache.V[l])
        np.testing.assert_allclose(out, X[l + 1], rtol=1e-12, atol=1e-13)
    with pytest.raises(ValueError):
        om.dp(X, pos, cache, L + 1)
    with pytest.raises(ValueError):
        om.dp(X, pos, cache, -1)


def _model_with_active_layers(name, active):
    shape = si.SHAPES[name]
    tm = torch_model(name)
    m = {k: v for k, v in tm.items() if k != "layers"}
    m["layers"] = []
    for l, lw in enumerate(tm["layers"]):
        lw = dict(lw)
        if l not in active:
            lw["wo"] = torch.zeros_like(lw["wo"])
            lw["w_down"] = torch.zeros_like(lw["w_down"])
        m["layers"].append(lw)
    return oc.OracleModel(shape, si.model_to_numpy(m))


def test_identity_layers_tie_and_ties_skip_so_the_last_M_layers_go():
    om = _model_with_active_layers("tiny-f32", active=())
    shape = om.shape
    cache = oc.KVCache(shape, 8)
    X, _ = om.prefill(prompt(shape, 5), cache)
    for M in (1, 3, 7):
        res = om.dp(X, 4, cache, M)
        assert res["mask"].tolist() == [0] * (shape.n_layers - M) + [1] * M


@pytest.mark.parametrize("k", [0, 3, 7])
def test_the_only_active_layer_is_never_skipped(k):
    om = _model_with_active_layers("tiny-f32", active=(k,))
    shape = om.shape
    cache = oc.KVCache(shape, 8)
    X, _ = om.prefill(prompt(shape, 5), cache)
    for M in (1, 4, 7):
        res = om.dp(X, 4, cache, M)
        assert res["mask"][k] == 0 and res["mask"].sum() == M
        np.testing.assert_allclose(res["g_final"], X[shape.n_layers], rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("resid_scale", [1.0, 0.05])
def test_brute_force_bounds_the_dp_from_above(resid_scale):
    T, M = 6, 3
    om, shape, cache, X = _setup("tiny-f32", T, resid_scale)
    L, pos = shape.n_layers, T - 1
    res = om.dp(X, pos, cache, M)
    d_lm = np.nanmax([res["sigma_c"][L, M], res["sigma_s"][L, M]])
    best = -2.0
    for comb in itertools.combinations(range(L), M):
        mask = np.zeros(L, dtype=np.uint8)
        mask[list(comb)] = 1
        best = max(best, _np_cos(_replay(om, cache, X[0], mask, pos), X[L]))
    assert best >= d_lm - 1e-12
    assert d_lm > -1.0


def test_override_forces_a_cell():
    T, M = 6, 2
    om, shape, cache, X = _setup("tiny-f32", T, 0.05)
    L = shape.n_layers
    base = om.dp(X, T - 1, cache, M)
    ov = np.full((L + 1, M + 1), -1, dtype=np.int8)
    i, j = 4, 1
    ov[i, j] = 1 - base["choice"][i, j]
    forced = om.dp(X, T - 1, cache, M, override=ov)
    assert forced["choice"][i, j] == 1 - base["choice"][i, j]
    assert np.array_equal(forced["sigma_c"][: i + 1], base["sigma_c"][: i + 1], equal_nan=True)
    rep = _replay(om, cache, X[0], forced["mask"], T - 1)
    assert np.array_equal(rep, forced["g_final"]) and forced["mask"].sum() == M


@pytest.mark.parametrize("name,M,K,resid_scale,n_gen", [("tiny-f32", 3, 4, 1.0, 32), ("tiny-f32", 3, 4, 0.05, 32),
                                                       ("tiny-f32", 0, 4, 1.0, 17), ("small-bf16", 2, 3, 0.05, 16)])
def test_speculative_greedy_is_lossless(name, M, K, resid_scale, n_gen):
    om = oracle_model(name, 1, resid_scale)
    pr = prompt(om.shape, 24)
    plain, _ = om.greedy_decode(pr, n_gen)
    spec = om.spec_decode(pr, n_gen, M, K)
    assert spec["tokens"] == plain
    for r in spec["rounds"]:
        assert 0 <= r["accepted"] <= K and r["mask"].sum() == M
        if M == 0:  # the draft model is the full model: every draft is accepted
            assert r["accepted"] == K


def test_slow_drift_model_accepts_drafts():
    """With small residual writers the hidden state drifts slowly (the regime of Sec. 3.5) and layer-skipped
    drafts get accepted; this keeps the accept > 0 paths of the loop exercised."""
    om = oracle_model("tiny-f32", 1, 0.05)
    spec = om.spec_decode(prompt(om.shape, 24), 32, 3, 4)
    assert sum(r["accepted"] for r in spec["rounds"]) > 0


def test_dp_interval_keeps_the_mask_between_updates():
    om = oracle_model("tiny-f32", 1, 0.05)
    pr = prompt(om.shape, 24)
    plain, _ = om.greedy_decode(pr, 20)
    spec = om.spec_decode(pr, 20, 3, 2, dp_interval=3)
    assert spec["tokens"] == plain
    masks = [r["mask"].tolist() for r in spec["rounds"]]
    for a, b, c in zip(masks[0::3], masks[1::3], masks[2::3]):
        assert a == b == c


def test_top1_prob_closed_forms():
    """Equal logits give 1/V; one logit far above the rest gives 1; shifting all logits changes nothing."""
    assert oc.top1_prob(np.zeros(50)) == pytest.approx(1.0 / 50, rel=1e-12)
    lg = np.array([0.0, np.log(3.0)])
    assert oc.top1_prob(lg) == pytest.approx(0.75, rel=1e-12)
    assert oc.top1_prob(lg + 1000.0) == pytest.approx(0.75, rel=1e-12)
    assert oc.top1_prob(np.array([100.0, 0.0, 0.0])) == pytest.approx(1.0, abs=1e-40)


@pytest.mark.parametrize("thr", [0.0, 0.0026, 0.3, 1.5])
def test_draft_exiting_threshold_shortens_rounds_and_stays_lossless(thr):
    """Sec. 5.3.3: a round stops drafting after the first token whose draft confidence is below the threshold.
    The output must still be plain greedy decoding; threshold 0 never exits early; a threshold above 1 drafts one
    token per round; in between, every round ends exactly at its first low-confidence draft."""
    om = oracle_model("tiny-f32", 1, 0.05)
    pr = prompt(om.shape, 24)
    K = 4
    plain, _ = om.greedy_decode(pr, 24)
    spec = om.spec_decode(pr, 24, 3, K, det_threshold=thr)
    assert spec["tokens"] == plain
    base = om.spec_decode(pr, 24, 3, K)
    if thr == 0.0:
        assert [r["drafts"] for r in spec["rounds"]] == [r["drafts"] for r in base["rounds"]]
    for r in spec["rounds"]:
        n = len(r["drafts"])
        assert 1 <= n <= K and len(r["verify"]) == n + 1 and r["accepted"] <= n
        assert all(c >= thr for c in r["draft_conf"][:-1])
        assert n == K or r["draft_conf"][-1] < thr
        if thr > 1.0:
            assert n == 1
    if thr == 0.0026:  # about the median confidence of this random-init model (vocab 1024): rounds of mixed length
        lens = [len(r["drafts"]) for r in spec["rounds"]]
        assert min(lens) < K and max(lens) > 1


# ---- the search restricted to a window of layers, and the objective of a given skip set (Sec. 3.5) -------------------
def test_window_over_all_layers_is_the_plain_search():
    T, M = 7, 3
    om, shape, cache, X = _setup("tiny-f32", T, 0.05)
    a = om.dp(X, T - 1, cache, M)
    b = om.window(0, shape.n_layers).dp(X, T - 1, cache.window(0, shape.n_layers), M)
    for k in ("sigma_c", "sigma_s", "choice", "g_final", "mask"):
        assert np.array_equal(a[k], b[k], equal_nan=True), k


@pytest.mark.parametrize("resid_scale", [1.0, 0.05])
def test_window_search_replays_and_is_bounded_by_brute_force(resid_scale):
    """Window 2..6 of the 8 layers: the window's skip set replayed from x_2 reproduces g; pushing it on through the
    kept layers 6, 7 gives the state whose cosine with x_L brute force over the window's C(4, 2) sets can only beat
    when it is evaluated on the same objective (cosine at the end of the window)."""
    T, M, lo, hi = 6, 2, 2, 6
    om, shape, cache, X = _setup("tiny-f32", T, resid_scale)
    L, pos = shape.n_layers, T - 1
    res = om.window(lo, hi).dp(X[lo:hi + 1], pos, cache.window(lo, hi), M)
    assert int(res["mask"].sum()) == M and res["mask"].shape == (hi - lo,)
    full_mask = np.zeros(L, dtype=np.uint8)
    full_mask[lo:hi] = res["mask"]
    h = X[lo].copy()
    for l in range(lo, hi):
        if not full_mask[l]:
            h, _, _ = om.layer(l, h, pos, pos, cache.K[l], cache.V[l])
    assert np.array_equal(h, res["g_final"])
    d_win = np.nanmax([res["sigma_c"][hi - lo, M], res["sigma_s"][hi - lo, M]])
    assert _np_cos(h, X[hi]) == pytest.approx(d_win, abs=1e-12)
    # masked_state from x_0 passes through the kept layers 0, 1 (reproducing x_2), the window, then 6, 7
    end = om.masked_state(X[0], pos, cache, full_mask)
    tail = h.copy()
    for l in range(hi, L):
        tail, _, _ = om.layer(l, tail, pos, pos, cache.K[l], cache.V[l])
    np.testing.assert_allclose(end, tail, rtol=1e-12, atol=1e-13)
    assert om.skip_cosine(X[0], pos, cache, full_mask, X[L]) == pytest.approx(_np_cos(end, X[L]), abs=1e-12)
    best = -2.0
    for comb in itertools.combinations(range(lo, hi), M):
        m = np.zeros(L, dtype=np.uint8)
        m[list(comb)] = 1
        g = X[lo].copy()
        for l in range(lo, hi):
            if not m[l]:
                g, _, _ = om.layer(l, g, pos, pos, cache.K[l], cache.V[l])
        best = max(best, _np_cos(g, X[hi]))
    assert best >= d_win - 1e-12


def test_skip_cosine_closed_forms():
    T = 5
    om, shape, cache, X = _setup("tiny-f32", T)
    L, pos = shape.n_layers, T - 1
    none, every = np.zeros(L, dtype=np.uint8), np.ones(L, dtype=np.uint8)
    assert om.skip_cosine(X[0], pos, cache, none, X[L]) == pytest.approx(1.0, abs=1e-12)   # nothing skipped: x_L itself
    assert om.skip_cosine(X[0], pos, cache, every, X[L]) == pytest.approx(_np_cos(X[0], X[L]), abs=1e-12)
    np.testing.assert_allclose(om.masked_state(X[0], pos, cache, none), X[L], rtol=1e-12, atol=1e-13)
