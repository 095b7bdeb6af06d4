"""Pins of the oracle's stochastic decoding pieces (CPU only): inverse-CDF draws, the speculative-sampling
acceptance rule, and the sampling loop.

What fixes them (Sec. 4.1 of the paper calls the method "still speculative sampling", lossless by the result it
cites): whatever the draft distribution q, the first token a round emits must be distributed exactly as the full
model's p. The tests check that on a small vocabulary by exhaustive integration over the uniform numbers' cells and by
a seeded Monte-Carlo run, plus closed forms of the draw itself.
"""
import numpy as np
import pytest

import synth_inputs as si
from oracle import clasp_oracle as oc
from tests.helpers import oracle_model, prompt


def test_inverse_cdf_closed_forms():
    w = [1.0, 1.0, 2.0]
    assert oc.sample_cdf(w, 0.0)[0] == 0 and oc.sample_cdf(w, 0.2499)[0] == 0
    assert oc.sample_cdf(w, 0.25)[0] == 1 and oc.sample_cdf(w, 0.4999)[0] == 1
    assert oc.sample_cdf(w, 0.5)[0] == 2 and oc.sample_cdf(w, 0.9999999)[0] == 2
    assert oc.sample_cdf([0.0, 3.0, 0.0], 0.7)[0] == 1  # zero-weight entries are never drawn
    v, margin = oc.sample_cdf(w, 0.3)
    assert v == 1 and margin == pytest.approx(0.05)
    # scale invariance and the frequency of each index over a fine grid of u
    grid = (np.arange(4000) + 0.5) / 4000
    counts = np.bincount([oc.sample_cdf(np.array(w) * 7.0, u)[0] for u in grid], minlength=3)
    assert counts.tolist() == [1000, 1000, 2000]


def test_softmax_temperature():
    lg = np.array([0.0, np.log(4.0)])
    assert oc.softmax_t(lg, 1.0) == pytest.approx([0.2, 0.8])
    assert oc.softmax_t(lg, 2.0) == pytest.approx([1 / 3, 2 / 3])
    assert oc.softmax_t(lg + 500.0, 1.0) == pytest.approx([0.2, 0.8])


def test_identical_models_accept_every_draft():
    rng = np.random.default_rng(5)
    lg = rng.normal(size=(4, 11))
    drafts = [3, 7, 0]
    a, tok, _ = oc.spec_accept(lg, lg[:3], drafts, [0.0, 0.5, 0.999999], 0.37)
    assert a == 3 and tok == oc.sample_cdf(oc.softmax_t(lg[3]), 0.37)[0]


def test_rejection_draws_only_where_p_exceeds_q():
    p_lg = np.log(np.array([[0.5, 0.3, 0.2], [1 / 3, 1 / 3, 1 / 3]]))
    q_lg = np.log(np.array([[0.1, 0.2, 0.7]]))
    # draft token 2: p/q = 2/7; u = 0.9 rejects; residual max(0, p - q) = (0.4, 0.1, 0) -> token 0 w.p. 0.8
    for u_fin, want in [(0.0, 0), (0.79, 0), (0.81, 1), (0.999, 1)]:
        a, tok, _ = oc.spec_accept(p_lg, q_lg, [2], [0.9], u_fin)
        assert (a, tok) == (0, want)
    a, tok, _ = oc.spec_accept(p_lg, q_lg, [2], [0.2], 0.5)  # 0.2 * 0.7 < 0.2: kept, bonus from p_1
    assert (a, tok) == (1, 1)
    a, _, _ = oc.spec_accept(p_lg, q_lg, [0], [0.999999], 0.5)  # p >= q: always kept
    assert a == 1


def _first_token_distribution_exact(p, q):
    """P(first emitted token = t) by integrating the rule over (draft draw, u_accept, u_final) analytically from
    what the oracle functions return on a grid: u_accept and u_final enter only through thresholds, so a fine
    midpoint grid is exact up to its resolution."""
    V = p.size
    p_lg, q_lg = np.log(np.stack([p, p])), np.log(q[None, :])
    G = 400
    grid = (np.arange(G) + 0.5) / G
    dist = np.zeros(V)
    for x in range(V):
        if q[x] == 0:
            continue
        for ua in grid:
            a, _, _ = oc.spec_accept(p_lg, q_lg, [x], [ua], 0.5)
            if a == 1:
                dist[x] += q[x] / G
            else:
                for uf in grid[::8]:
                    _, tok, _ = oc.spec_accept(p_lg, q_lg, [x], [ua], uf)
                    dist[tok] += q[x] / G / len(grid[::8])
    return dist


def test_first_token_follows_the_full_model_exactly_on_a_grid():
    p = np.array([0.40, 0.25, 0.20, 0.10, 0.05])
    q = np.array([0.05, 0.45, 0.10, 0.30, 0.10])
    dist = _first_token_distribution_exact(p, q)
    assert dist.sum() == pytest.approx(1.0, abs=1e-9)
    assert np.abs(dist - p).max() < 6e-3  # grid resolution: 1/400 in u_accept, 1/50 in u_final


def test_first_token_follows_the_full_model_monte_carlo():
    rng = np.random.default_rng(11)
    V, N = 7, 30000
    p_lg, q_lg = rng.normal(size=V) * 1.5, rng.normal(size=V) * 1.5
    p, q = oc.softmax_t(p_lg), oc.softmax_t(q_lg)
    u = si.gen_uniform(3, 3 * N, 7).numpy().astype(np.float64).reshape(N, 3)
    counts = np.zeros(V)
    for u_d, u_a, u_f in u:
        x, _ = oc.sample_cdf(q, u_d)
        a, tok, _ = oc.spec_accept(np.stack([p_lg, p_lg]), q_lg[None, :], [x], [u_a], u_f)
        counts[x if a == 1 else tok] += 1
    chi2 = float(((counts - N * p) ** 2 / (N * p)).sum())
    assert chi2 < 22.5  # 6 degrees of freedom: P(chi2 > 22.5) ~ 1e-3; the run is seeded, so this is a fixed check
    # and it is NOT distributed as q (the test would be blind if p and q were close)
    assert float(((counts - N * q) ** 2 / (N * q)).sum()) > 200


def test_uniform_generator_range_and_mean():
    u = si.gen_uniform(1, 100000, 0).numpy()
    assert u.min() >= 0.0 and u.max() < 1.0 and abs(u.mean() - 0.5) < 5e-3
    assert np.all(u * (1 << 24) == np.round(u * (1 << 24)))
    assert not np.array_equal(u[:1000], si.gen_uniform(1, 1000, 1).numpy())


def _uniforms(seed, rounds, K):
    return {"first": si.gen_uniform(seed, 1, 10).numpy(), "draft": si.gen_uniform(seed, rounds * K, 11).numpy(),
            "accept": si.gen_uniform(seed, rounds * K, 12).numpy(), "final": si.gen_uniform(seed, rounds, 13).numpy()}


def test_sampling_loop_structure():
    """M = 0: the draft model is the full model, p = q, every draft is kept. M > 0: rounds stay consistent."""
    om = oracle_model("tiny-f32", 1, 0.05)
    pr = prompt(om.shape, 16)
    K, n_gen = 3, 14
    un = _uniforms(4, n_gen, K)
    full = om.spec_sample_decode(pr, n_gen, 0, K, un)
    assert all(r["accepted"] == K for r in full["rounds"]) and len(full["tokens"]) == n_gen
    spec = om.spec_sample_decode(pr, n_gen, 3, K, un)
    assert spec["tokens"][0] == full["tokens"][0]  # same prefill, same first draw
    emitted = 1
    for r in spec["rounds"]:
        assert 0 <= r["accepted"] <= K and r["mask"].sum() == 3 and r["pos"] == len(pr) + emitted - 1
        emitted += r["accepted"] + 1
    assert emitted >= n_gen


def test_argmax_margin_closed_forms():
    """argmax_margin: lowest index of the maximum, and the gap to the runner-up (0 on a tie, inf for one entry)."""
    assert oc.argmax_margin(np.array([1.0, 5.0, 3.0])) == (1, 2.0)
    assert oc.argmax_margin(np.array([2.0, 7.0, 7.0, 1.0])) == (1, 0.0)
    assert oc.argmax_margin(np.array([-4.0, -9.5, -4.25])) == (0, 0.25)
    i, m = oc.argmax_margin(np.array([3.0]))
    assert i == 0 and m == float("inf")
    lg = np.array([0.5, -1.0, 0.25, 0.5 - 1e-9])
    i, m = oc.argmax_margin(lg)
    assert i == 0 and abs(m - 1e-9) < 1e-15
    # shifting every logit moves neither the index nor the margin; scaling scales the margin
    assert oc.argmax_margin(lg + 11.0)[0] == 0 and abs(oc.argmax_margin(3.0 * lg)[1] - 3e-9) < 1e-14


def test_sampling_loop_with_no_skipped_layer_is_plain_ancestral_sampling():
    """M = 0: draft model = full model, so p = q, every draft is kept, and the loop must emit exactly what sampling the
    full model token by token emits when it is handed the same uniform numbers in the order the loop consumes them:
    first, then per round K draft numbers and the round's final number. This pins the loop's bookkeeping (positions,
    cache rows, which uniform number feeds which draw) to the textbook procedure, written here without any rounds."""
    om = oracle_model("tiny-f32", 1, 0.05)
    pr = prompt(om.shape, 12)
    K, n_gen, temp = 3, 13, 0.8
    un = _uniforms(9, n_gen, K)
    spec = om.spec_sample_decode(pr, n_gen, 0, K, un, temperature=temp)
    order = [un["first"][0]]
    for r in range(n_gen):
        order += list(un["draft"][r * K:(r + 1) * K]) + [un["final"][r]]
    cache = oc.KVCache(om.shape, len(pr) + n_gen + 2)
    _, lg = om.prefill(pr, cache)
    plain = []
    for t in range(n_gen):
        tok, _ = oc.sample_cdf(oc.softmax_t(lg, temp), order[t])
        plain.append(tok)
        _, lg = om.token(tok, len(pr) + t, cache)
    assert spec["tokens"] == plain
    assert all(r["accepted"] == K for r in spec["rounds"])


def test_sampling_loop_keeps_every_draft_when_the_acceptance_numbers_are_zero():
    """u * q(x) < p(x) holds for u = 0 wherever p(x) > 0: with all acceptance numbers zero every round keeps its K
    drafts whatever the skip set, emits K + 1 tokens, and the next round starts K + 1 positions further on."""
    om = oracle_model("tiny-f32", 1, 1.0)
    pr = prompt(om.shape, 10)
    K, n_gen = 2, 10
    un = _uniforms(5, n_gen, K)
    un["accept"] = np.zeros_like(un["accept"])
    spec = om.spec_sample_decode(pr, n_gen, 3, K, un)
    assert all(r["accepted"] == K for r in spec["rounds"])
    assert [r["pos"] for r in spec["rounds"]] == [len(pr) + (K + 1) * i for i in range(len(spec["rounds"]))]
    flat = [spec["tokens"][0]]
    for r in spec["rounds"]:
        flat += r["drafts"] + [r["next"]]
    assert flat[:n_gen] == spec["tokens"]
    # and with acceptance numbers just below one, a model whose draft differs from the full model rejects early
    # (a draft x drawn from q is rejected exactly when q(x) > p(x) then: about every other one on this model)
    n_gen = 30
    un = _uniforms(5, n_gen, K)
    un["accept"] = np.full_like(un["accept"], 1.0 - 2.0 ** -24)
    spec = om.spec_sample_decode(pr, n_gen, 3, K, un)
    kept = sum(r["accepted"] for r in spec["rounds"])
    assert 0 < kept < K * len(spec["rounds"]) and len(spec["rounds"]) >= n_gen // (K + 1)
