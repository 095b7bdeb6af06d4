"""GPU parity of stochastic decoding: inverse-CDF draws, the speculative-sampling acceptance rule and the sampling
loop, called through the C ABI, against the fp64 oracle on the same logits and the same uniform numbers.

Tokens and accepted counts are integers decided by floating-point comparisons (a running sum against u * total, a
probability ratio against u): they must be equal wherever the oracle's own margin of that comparison exceeds what fp32
sums over the vocabulary can move it (1e-5 of the total for the running sums, 1e-4 relative for the ratio); below
that margin either side of the boundary is a correct draw and the case is skipped (and counted, so that a test cannot
pass by skipping everything).
"""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import clasp_oracle as oc
from tests.helpers import oracle_model
from tests.test_gpu_parity import dev, engine

pytestmark = pytest.mark.gpu

CDF_MARGIN = 1e-5
RATIO_MARGIN = 1e-4


def _logits(seed, rows, vocab, scale):
    return si.gen_matrix(seed, 900 + rows, rows, vocab, scale, "f32").numpy().astype(np.float32)


@pytest.mark.parametrize("name,temperature", [("tiny-f32", 1.0), ("small-bf16", 1.0), ("small-bf16", 0.7)])
def test_sample_token_matches_oracle(name, temperature):
    eng = engine(name)
    V = si.SHAPES[name].vocab  # 1024, and 2064 (not a multiple of the workgroup size: ragged chunks)
    lg = _logits(5, 3, V, 2.0)
    lg[1, V // 3: V // 3 + 400] = -1e30  # a long run of zero-probability tokens (whole chunks of zero weight)
    lg[2] = 0.0
    lg[2, -1] = 30.0  # nearly all mass on the last index
    us = np.concatenate([si.gen_uniform(9, 60, 0).numpy(), [0.0, 1.0 - 2.0 ** -24, 0.5]]).astype(np.float32)
    d_u, d_tok = dev(us), torch.zeros(1, dtype=torch.int32, device="cuda")
    checked = 0
    for row in range(3):
        d_lg = dev(lg[row])
        w = oc.softmax_t(lg[row], temperature)
        for i, u in enumerate(us):
            eng.clasp_sample_token(d_lg, temperature, d_u[i:i + 1], d_tok)
            ref, margin = oc.sample_cdf(w, float(u))
            got = int(d_tok)
            assert 0 <= got < V and w[got] > 0
            if margin > CDF_MARGIN:
                assert got == ref, (row, i, u, got, ref, margin)
                checked += 1
    assert checked > 150


def _accept_case(seed, n, V, noise):
    p_lg = _logits(seed, n + 1, V, 2.0)
    q_lg = (p_lg[:n] + noise * _logits(seed + 1, n, V, 2.0)).astype(np.float32)
    u = si.gen_uniform(seed, 2 * n + 1, 3).numpy()
    drafts = [oc.sample_cdf(oc.softmax_t(q_lg[i]), float(u[i]))[0] for i in range(n)]
    return p_lg, q_lg, drafts, u[n:2 * n].astype(np.float32), u[2 * n:].astype(np.float32)


@pytest.mark.parametrize("name,temperature", [("tiny-f32", 1.0), ("small-bf16", 1.0), ("small-bf16", 0.6)])
def test_spec_accept_matches_oracle(name, temperature):
    eng = engine(name)
    V = si.SHAPES[name].vocab
    n_acc = torch.zeros(1, dtype=torch.int32, device="cuda")
    nxt = torch.zeros(1, dtype=torch.int32, device="cuda")
    checked, seen = 0, set()
    for seed in range(40):
        n = 1 + seed % 4
        noise = [0.0, 0.05, 0.3, 1.0][(seed // 4) % 4]
        p_lg, q_lg, drafts, u_acc, u_fin = _accept_case(100 + seed, n, V, noise)
        a_ref, tok_ref, info = oc.spec_accept(p_lg, q_lg, drafts, u_acc, float(u_fin[0]), temperature)
        eng.clasp_spec_accept(dev(p_lg), dev(q_lg), dev([7] + drafts, torch.int32), n, temperature, dev(u_acc),
                              dev(u_fin), n_acc, nxt)
        a, tok = int(n_acc), int(nxt)
        assert 0 <= a <= n and 0 <= tok < V
        if noise == 0.0:
            assert a == n  # identical distributions: every draft is kept
        if min(info["ratio_margin"]) > RATIO_MARGIN:
            assert a == a_ref, (seed, a, a_ref, info)
            if info["cdf_margin"] > CDF_MARGIN:
                assert tok == tok_ref, (seed, tok, tok_ref, info)
                checked += 1
                seen.add(a == n)
    assert checked > 25 and seen == {True, False}  # both full acceptance and rejections were compared


def test_invalid_sampling_arguments_are_rejected_on_the_host():
    import paper_2505_24196_amd as clasp
    eng = engine("tiny-f32")
    V = si.SHAPES["tiny-f32"].vocab
    lg, u = torch.zeros(V, device="cuda"), torch.zeros(1, device="cuda")
    tok = torch.zeros(32, dtype=torch.int32, device="cuda")
    with pytest.raises(clasp.ClaspError):
        eng.clasp_sample_token(lg, 0.0, u, tok[:1])
    with pytest.raises(clasp.ClaspError):
        eng.clasp_draft_sample(None, tok[:1], 10 ** 6, 1.0, u, lg, tok[1:2])
    p = torch.zeros(32, V, device="cuda")
    with pytest.raises(clasp.ClaspError):
        eng.clasp_spec_accept(p, p, tok, 0, 1.0, u, u, tok[:1], tok[1:2])
    with pytest.raises(clasp.ClaspError):
        eng.clasp_spec_accept(p, p, tok, 16, 1.0, torch.zeros(16, device="cuda"), u, tok[:1], tok[1:2])


def _uniforms(seed, rounds, K):
    return {"first": si.gen_uniform(seed, 1, 10), "draft": si.gen_uniform(seed, rounds * K, 11),
            "accept": si.gen_uniform(seed, rounds * K, 12), "final": si.gen_uniform(seed, rounds, 13)}


@pytest.mark.parametrize("M,resid_scale,useed", [(0, 0.05, 7), (3, 1.0, 11)])
def test_sampling_loop_tiny_matches_oracle(M, resid_scale, useed):
    """Closed sampling loop on the tiny fp32 model with shared uniform numbers. M = 0: the draft model is the full
    model, so every draft must be kept. The device trajectory is compared with the oracle's round by round until the
    first decision whose oracle margin is below tolerance (after which the two may legitimately part); the seeds
    of the uniform numbers are chosen so that the oracle's first rounds are clear of such decisions. (Random-init
    models have nearly flat distributions, so almost every draft is kept here; rejections are compared in
    test_spec_accept_matches_oracle.)"""
    import paper_2505_24196_amd as clasp
    name, K, n_gen = "tiny-f32", 3, 20
    shape = si.SHAPES[name]
    om, eng = oracle_model(name, 1, resid_scale), engine(name, 1, resid_scale)
    pr = [int(t) for t in si.gen_tokens(2, 32, shape.vocab)]
    un = _uniforms(useed, n_gen, K)
    gpu = clasp.clasp_sample_generate(eng, pr, n_gen, M, K, {k: v.cuda() for k, v in un.items()})
    ref = om.spec_sample_decode(pr, n_gen, M, K, {k: v.numpy() for k, v in un.items()})
    assert len(gpu["tokens"]) == n_gen and all(0 <= t < shape.vocab for t in gpu["tokens"])
    if M == 0:
        assert all(r["accepted"] == K for r in gpu["rounds"])
    compared = 0
    if ref["first_margin"] > CDF_MARGIN:
        assert gpu["tokens"][0] == ref["tokens"][0]
        for rg, ro in zip(gpu["rounds"], ref["rounds"]):
            if M and np.nanmin(np.abs(ro["dp"]["sigma_c"] - ro["dp"]["sigma_s"])) <= 2e-3:
                break
            if min(ro["draft_margin"]) <= CDF_MARGIN or min(ro["ratio_margin"]) <= RATIO_MARGIN \
                    or ro["cdf_margin"] <= CDF_MARGIN:
                break
            assert rg["mask"] == ro["mask"].tolist() and rg["drafts"] == ro["drafts"]
            assert (rg["accepted"], rg["next"]) == (ro["accepted"], ro["next"])
            compared += 1
    assert compared >= 3
