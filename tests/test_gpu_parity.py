"""GPU parity: the HIP path, called through the C ABI (ctypes binding), against the CPU oracle on the same seeded
inputs. Tolerances (from the benchmark spec): hidden states 1e-4 relative in fp32 and 2e-2 relative in bf16 (max abs
error over the max magnitude of the oracle tensor), cosine scores 1e-3 absolute, skip sets / choices / tokens
bit-exact wherever the oracle's own decision margin exceeds the tolerance; on a sub-margin cell the oracle is re-run
with that cell forced to the device's choice so that everything downstream is still compared.
"""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import clasp_oracle as oc
from tests.helpers import oracle_model, prompt, torch_model

pytestmark = pytest.mark.gpu

HID_TOL = {"f32": 1e-4, "bf16": 2e-2}
COS_TOL = 1e-3
COS_MARGIN = 2e-3


def relerr(a, b):
    """Largest absolute error over the largest magnitude of the oracle tensor."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.abs(a - b).max() / (np.abs(b).max() + 1e-30))


def relerr_rows(a, b):
    """The same figure taken row by row (last axis = one hidden state / one row of logits), largest over the rows:
    no row borrows the scale of a larger one."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    a, b = a.reshape(-1, a.shape[-1]), b.reshape(-1, b.shape[-1])
    return float((np.abs(a - b).max(axis=1) / (np.abs(b).max(axis=1) + 1e-30)).max())


def assert_close(a, b, tol, what=""):
    """Tensor-wide and per-row relative error both within tol."""
    e, er = relerr(a, b), relerr_rows(a, b)
    assert e <= tol and er <= tol, f"{what}: tensor-wide {e:.3e}, per-row {er:.3e} > {tol}"


_ENGINES = {}


def engine(name, seed=1, resid_scale=1.0, max_seq=256, max_rows=16):
    import paper_2505_24196_amd as clasp
    key = (name, seed, resid_scale, max_seq, max_rows)
    if key not in _ENGINES:
        _ENGINES[key] = clasp.Engine(si.SHAPES[name], max_seq=max_seq, max_rows=max_rows).load(
            torch_model(name, seed, resid_scale))
    return _ENGINES[key]


def dev(x, dtype=torch.float32):
    return torch.as_tensor(np.asarray(x), dtype=dtype, device="cuda")


def oracle_prefill(om, toks, t_max):
    cache = oc.KVCache(om.shape, t_max)
    st, lg = [], []
    for t, tk in enumerate(toks):
        s, l = om.token(tk, t, cache, want_states=True)
        st.append(s)
        lg.append(l)
    return cache, np.stack(st, 1), np.stack(lg)


def oracle_dp_following(om, Xw, pos, cache, M, g_choice, stats=None):
    """The oracle's DP, with every cell where it and the device decide differently forced to the device's choice -
    allowed only where the oracle's own margin |sigma_c - sigma_s| is within COS_MARGIN - so that everything
    downstream of a near-tie is still compared. stats (dict) counts the decided cells and the forced ones."""
    L = om.shape.n_layers
    ov = np.full((L + 1, M + 1), -1, dtype=np.int8)
    for _ in range(16):
        ref = om.dp(Xw, pos, cache, M, override=ov)
        diff = np.argwhere(ref["choice"] != g_choice)
        if diff.size == 0:
            break
        for i, j in diff:
            assert ref["choice"][i, j] != 255 and g_choice[i, j] != 255, f"cell ({i},{j}) defined on one side only"
            margin = abs(ref["sigma_c"][i, j] - ref["sigma_s"][i, j])
            assert margin <= COS_MARGIN, f"choice differs at ({i},{j}) with oracle margin {margin}"
            ov[i, j] = g_choice[i, j]
    else:
        raise AssertionError("device and oracle choices do not converge")
    if stats is not None:
        stats["cells"] = stats.get("cells", 0) + int((ref["choice"] != 255).sum())
        stats["forced"] = stats.get("forced", 0) + int((ov >= 0).sum())
    return ref


def check_dp(om, eng, X, pos, cache, M, lo=0, hi=None, X_dev=None, stats=None):
    """Margin-aware comparison of one DP call (restricted to the layers lo..hi-1 when given; X then still holds all
    L+1 states, of which lo..hi are read). X: the oracle's stored states; X_dev: the states the device's own verify pass
    produced for the same row (a device tensor; default: the oracle's, uploaded). Returns (device result, oracle result)."""
    L_all = om.shape.n_layers
    hi = L_all if hi is None else hi
    L = hi - lo
    windowed = (lo, hi) != (0, L_all)
    Xd = dev(X) if X_dev is None else X_dev
    if windowed:
        gpu = eng.clasp_dp_select_window(Xd, pos, M, lo, hi, want_tables=True)
        om, cache, Xw = om.window(lo, hi), cache.window(lo, hi), X[lo:hi + 1]
    else:
        gpu = eng.clasp_dp_select(Xd, pos, M, want_tables=True)
        Xw = X
    g_choice = gpu["choice"].cpu().numpy()
    ref = oracle_dp_following(om, Xw, pos, cache, M, g_choice, stats)
    sc = gpu["scores"].cpu().numpy().astype(np.float64)
    for k, key in enumerate(("sigma_c", "sigma_s")):
        assert np.array_equal(np.isnan(sc[..., k]), np.isnan(ref[key])), key
        if not np.isnan(ref[key]).all():
            assert np.nanmax(np.abs(sc[..., k] - ref[key])) <= COS_TOL, key
    mask = gpu["mask"].cpu().numpy()
    assert mask[lo:hi].tolist() == ref["mask"].tolist()
    assert int(mask.sum()) == M and not mask[:lo].any() and not mask[hi:].any()
    assert relerr(gpu["g_final"].cpu().numpy(), ref["g_final"]) <= HID_TOL[om.shape.dtype]
    return gpu, ref


def replay_against_oracle(om, prompt_toks, spec, M, K, logit_tol, thr=None, dp_interval=1, prefilled=None):  # noqa: C901
    """The oracle driven call by call along a traced device run of the Draft -> Verify -> Layer-Optimisation loop
    (decode.clasp_generate(trace=True)): every DP table, every skip set, every draft and verify token of every round is
    compared. Where the two sides decide differently the oracle's own margin must be within tolerance (COS_MARGIN for a
    DP cell, logit_tol for an argmax), and the oracle then follows the device's decision, so the comparison goes on to
    the end of the run instead of stopping at the first near-tie. prefilled = (cache, states, logits): the oracle's own
    prompt pass when the caller has it already. Returns the counts of what was compared."""
    shape = om.shape
    n_rounds = len(spec["rounds"])
    if prefilled is None:
        cache = oc.KVCache(shape, len(prompt_toks) + sum(r["accepted"] + 1 for r in spec["rounds"]) + K + 2)
        states, logits = om.prefill(prompt_toks, cache)
    else:
        cache, states, logits = prefilled
        assert cache.t_max >= len(prompt_toks) + sum(r["accepted"] + 1 for r in spec["rounds"]) + K + 1
    st = {"rounds": 0, "cells": 0, "forced": 0, "tokens": 0, "tokens_forced": 0}

    def same_token(dev_tok, lg, what):
        ref_tok, margin = oc.argmax_margin(lg)
        st["tokens"] += 1
        if dev_tok != ref_tok:
            assert margin <= logit_tol, f"{what}: device {dev_tok}, oracle {ref_tok} with margin {margin}"
            st["tokens_forced"] += 1

    pending = spec["tokens"][0]
    same_token(pending, logits, "first token")
    pos = len(prompt_toks)
    dp_states, dp_pos = states, pos - 1
    ref = None
    for r, rg in enumerate(spec["rounds"]):
        assert rg["pos"] == pos
        if r % dp_interval == 0:
            ref = oracle_dp_following(om, dp_states, dp_pos, cache, M, rg["dp"]["choice"].numpy(), st)
            sc = rg["dp"]["scores"].numpy().astype(np.float64)
            for k, key in enumerate(("sigma_c", "sigma_s")):
                assert np.array_equal(np.isnan(sc[..., k]), np.isnan(ref[key])), key
                if not np.isnan(ref[key]).all():
                    assert np.nanmax(np.abs(sc[..., k] - ref[key])) <= COS_TOL, f"round {r} {key}"
        assert rg["mask"] == ref["mask"].tolist(), f"round {r}: skip sets differ"
        tok = pending
        for k, d in enumerate(rg["drafts"]):
            _, lg = om.token(tok, pos + k, cache, skip=ref["mask"])
            same_token(d, lg, f"round {r} draft {k}")
            if thr is not None:  # the confidence that decides whether the round goes on (the device's own rule is
                conf = oc.top1_prob(lg)  # checked by the caller on the device's figures)
                assert abs(rg["draft_conf"][k] - conf) <= 5e-3 * conf + 1e-6, f"round {r} draft {k} confidence"
            tok = d
        rows = [pending] + rg["drafts"]
        v_states = []
        for i, tk in enumerate(rows):
            s_i, lg = om.token(tk, pos + i, cache, want_states=True)
            v_states.append(s_i)
            same_token(rg["verify"][i], lg, f"round {r} verify row {i}")
        a = rg["accepted"]
        assert a == next((i for i in range(len(rg["drafts"])) if rg["drafts"][i] != rg["verify"][i]), len(rg["drafts"]))
        if "states" in rg:
            assert relerr(rg["states"].numpy(), v_states[a]) <= HID_TOL[shape.dtype], f"round {r}: states of row {a}"
        dp_states, dp_pos = v_states[a], pos + a
        pending = rg["verify"][a]
        pos += a + 1
        st["rounds"] += 1
    assert st["rounds"] == n_rounds
    return st


@pytest.mark.parametrize("name", ["tiny-f32", "small-bf16", "small-bf16-hd128"])
def test_verify_forward_hidden_states_and_logits(name):
    shape = si.SHAPES[name]
    om, eng = oracle_model(name), engine(name)
    toks = prompt(shape, 21)
    _, ost, olg = oracle_prefill(om, toks, 32)
    tt = dev(toks, torch.int32)
    outs = [eng.clasp_verify_forward(tt[:16], 0, True, True, True), eng.clasp_verify_forward(tt[16:], 16, True, True, True)]
    hid = torch.cat([o["hidden"] for o in outs], 1).cpu().numpy()
    lg = torch.cat([o["logits"] for o in outs]).cpu().numpy()
    am = torch.cat([o["argmax"] for o in outs]).cpu().numpy()
    mg = torch.cat([o["margin"] for o in outs]).cpu().numpy()
    tol = HID_TOL[shape.dtype]
    for l in range(shape.n_layers + 1):
        assert relerr(hid[l], ost[l]) <= tol, f"layer {l}"
    assert relerr(lg, olg) <= tol
    logit_tol = tol * np.abs(olg).max() * 2
    for r in range(len(toks)):
        ref_tok, ref_margin = oc.argmax_margin(olg[r])
        assert am[r] == int(np.argmax(lg[r]))
        if ref_margin > logit_tol:
            assert am[r] == ref_tok
            assert abs(mg[r] - ref_margin) <= logit_tol
    # one row at a time (plain decoding) gives the same states as the 16-row launch, within tolerance
    one = eng.clasp_verify_forward(tt[20:21], 20, True, True)
    assert relerr(one["hidden"][:, 0].cpu().numpy(), ost[:, 20]) <= tol


@pytest.mark.parametrize("name", ["small-bf16", "small-bf16-hd128"])
def test_verify_forward_every_row_count_of_a_launch(name):
    """A prompt of 1 + 2 + .. + 17 + 32 tokens goes through verify passes of 1, 2, .., 17 and 32 rows (every row count
    of one row group, a ragged and a full second group), each on top of the cache the passes before it left: the states
    of every row at every layer against the oracle, tensor-wide and row by row."""
    shape = si.SHAPES[name]
    sizes = list(range(1, 18)) + [32]
    n = sum(sizes)
    om, eng = oracle_model(name), engine(name, max_seq=256, max_rows=32)
    toks = prompt(shape, n)
    _, ost, _ = oracle_prefill(om, toks, 256)
    tt = dev(toks, torch.int32)
    tol, p0 = HID_TOL[shape.dtype], 0
    for k in sizes:
        out = eng.clasp_verify_forward(tt[p0:p0 + k], p0, True)
        hid = out["hidden"].cpu().numpy()
        assert hid.shape[1] == k
        for l in range(shape.n_layers + 1):
            assert_close(hid[l], ost[l, p0:p0 + k], tol, f"{k} rows at position {p0}, layer {l}")
        p0 += k
    assert p0 == n


@pytest.mark.parametrize("name,M", [("tiny-f32", 0), ("tiny-f32", 1), ("tiny-f32", 3), ("tiny-f32", 8),
                                    ("small-bf16", 2), ("small-bf16", 6), ("small-bf16-hd128", 3)])
@pytest.mark.parametrize("resid_scale", [1.0, 0.05])
def test_dp_select_matches_oracle(name, M, resid_scale):
    shape = si.SHAPES[name]
    om, eng = oracle_model(name, 1, resid_scale), engine(name, 1, resid_scale)
    toks = prompt(shape, 19)
    cache, ost, _ = oracle_prefill(om, toks, 32)
    eng.clasp_verify_forward(dev(toks[:16], torch.int32), 0)
    eng.clasp_verify_forward(dev(toks[16:], torch.int32), 16)  # device cache from the device's own prefill
    gpu, ref = check_dp(om, eng, ost[:, -1], 18, cache, M)
    if M == 0:
        assert not gpu["mask"].any()
    if M == shape.n_layers:
        assert gpu["mask"].all()


def test_dp_select_on_device_states_end_to_end():
    """verify -> DP entirely on the device (states never leave HBM) against the oracle's verify -> DP."""
    name = "tiny-f32"
    shape = si.SHAPES[name]
    om, eng = oracle_model(name, 1, 0.05), engine(name, 1, 0.05)
    toks = prompt(shape, 12)
    cache, ost, _ = oracle_prefill(om, toks, 32)
    out = eng.clasp_verify_forward(dev(toks, torch.int32), 0, want_hidden=True)
    for row in (3, 11):
        c = oc.KVCache(shape, 32)
        c.K[:, :row] = cache.K[:, :row]
        c.V[:, :row] = cache.V[:, :row]
        stats = {}
        check_dp(om, eng, ost[:, row], row, c, 3, X_dev=out["hidden"][:, row, :], stats=stats)
        assert stats["cells"] >= 3 * shape.n_layers - 3 and stats["forced"] <= 2, stats


@pytest.mark.parametrize("name", ["tiny-f32", "small-bf16"])
def test_draft_step_chain(name):
    """Two chained draft steps with a skip set (the second reads the first one's cache rows and device token)."""
    shape = si.SHAPES[name]
    om, eng = oracle_model(name, 1, 0.05), engine(name, 1, 0.05)
    toks = prompt(shape, 9)
    cache, _, olg = oracle_prefill(om, toks, 32)
    eng.clasp_verify_forward(dev(toks, torch.int32), 0)
    mask = np.zeros(shape.n_layers, dtype=np.uint8)
    mask[[1, shape.n_layers - 2]] = 1
    buf = torch.zeros(3, dtype=torch.int32, device="cuda")
    prob = torch.zeros(2, dtype=torch.float32, device="cuda")
    buf[0] = int(np.argmax(olg[-1]))
    tok = int(buf[0])
    for k in range(2):
        eng.clasp_draft_step(mask.tolist(), buf[k:k + 1], 9 + k, buf[k + 1:k + 2], prob[k:k + 1])
        _, lg = om.token(tok, 9 + k, cache, skip=mask)
        ref_tok, ref_margin = oc.argmax_margin(lg)
        p = np.exp(lg - lg.max())
        p /= p.sum()
        if ref_margin > HID_TOL[shape.dtype] * np.abs(lg).max() * 2:
            assert int(buf[k + 1]) == ref_tok
            assert abs(float(prob[k]) - p.max()) <= 0.05 * p.max() + 1e-6
        tok = int(buf[k + 1])  # follow the device token so that the second step sees the same input
    # keep-all mask == NULL mask == one-row verify
    a = torch.zeros(1, dtype=torch.int32, device="cuda")
    b = torch.zeros(1, dtype=torch.int32, device="cuda")
    eng.clasp_draft_step(None, buf[0:1], 9, a)
    eng.clasp_draft_step([0] * shape.n_layers, buf[0:1], 9, b)
    v = eng.clasp_verify_forward(buf[0:1], 9)
    assert int(a) == int(b) == int(v["argmax"][0])


@pytest.mark.parametrize("T", [700, 1500, 2601])
def test_long_prefix_split_and_ragged_blocks(T):
    """Synthetic cache: the prefix ends inside a 32-key block; 700 tokens take the latency-oriented single-workgroup
    launch, 1500 and 2601 the split launch (2 and 3 workgroups per KV head and query group) plus the merge kernel."""
    name = "small-bf16"
    shape = si.SHAPES[name]
    om, eng = oracle_model(name), engine(name, max_seq=2688)
    K, V = si.gen_kv(shape, 3, shape.n_layers, T)
    cache = oc.KVCache(shape, T + 8)
    cache.load(K.numpy().astype(np.float64), V.numpy().astype(np.float64))
    for l in range(shape.n_layers):
        eng.clasp_kv_load(l, K[l], V[l])
    toks = prompt(shape, 5, seed=5)
    st, lg = [], []
    for r, tk in enumerate(toks):
        s, l_ = om.token(tk, T + r, cache, want_states=True)
        st.append(s)
        lg.append(l_)
    ost = np.stack(st, 1)
    out = eng.clasp_verify_forward(dev(toks, torch.int32), T, want_hidden=True, want_logits=True)
    for l in range(shape.n_layers + 1):
        assert relerr(out["hidden"][l].cpu().numpy(), ost[l]) <= HID_TOL["bf16"], f"layer {l}"
    c = oc.KVCache(shape, T + 8)
    c.K[:, :T + 2] = cache.K[:, :T + 2]
    c.V[:, :T + 2] = cache.V[:, :T + 2]
    check_dp(om, eng, ost[:, 2], T + 2, c, 3)


@pytest.mark.parametrize("n_rows", [10, 13])
def test_very_long_prefix_three_and_four_query_tiles_per_workgroup(n_rows):
    """head_dim 128 over a 16500-token prefix (516 key blocks): from 512 blocks on, one workgroup of four wavefronts
    carries all query tiles of a KV group (10 rows x 4 heads = 40 queries = 3 tiles, 13 rows = 52 queries = 4 tiles)
    through one pass over the prefix, split 32 ways, merged by the combine kernel. Verify rows (causal among
    themselves) and the DP's candidate rows (own key / value from the self block) against the oracle."""
    name, T = "small-bf16-hd128", 16500
    shape = si.SHAPES[name]
    om, eng = oracle_model(name), engine(name, max_seq=16640)
    K, V = si.gen_kv(shape, 7, shape.n_layers, T)
    cache = oc.KVCache(shape, T + 16)
    cache.load(K.numpy().astype(np.float64), V.numpy().astype(np.float64))
    for l in range(shape.n_layers):
        eng.clasp_kv_load(l, K[l], V[l])
    toks = prompt(shape, n_rows, seed=8)
    st = []
    for r, tk in enumerate(toks):
        s, _ = om.token(tk, T + r, cache, want_states=True, want_logits=False)
        st.append(s)
    ost = np.stack(st, 1)
    out = eng.clasp_verify_forward(dev(toks, torch.int32), T, want_hidden=True)
    for l in range(shape.n_layers + 1):
        assert_close(out["hidden"][l].cpu().numpy(), ost[l], HID_TOL["bf16"], f"layer {l}")
    if n_rows == 10:  # the search with M = L - 1... the model has 4 layers: M = 3 pushes up to 3 rows; its attention
        # launches take one query tile, the verify rows above are what takes three and four
        check_dp(om, eng, ost[:, 1], T + 1, cache, 3, X_dev=out["hidden"][:, 1, :].contiguous())


@pytest.mark.parametrize("name,T", [("small-bf16", 300), ("small-bf16", 700), ("small-bf16", 1500),
                                    ("small-bf16-hd128", 2601)])
def test_single_row_forward_over_long_prefix(name, T):
    """One-row launches (draft steps, plain decoding) split the prefix over several workgroups per KV head and let
    the output projection merge the pieces (2, 3, 2 and 3 pieces here); hidden states and the chained draft token are
    compared with the oracle, and the row must agree with the same row inside a several-row launch."""
    shape = si.SHAPES[name]
    om, eng = oracle_model(name), engine(name, max_seq=2688)
    K, V = si.gen_kv(shape, 4, shape.n_layers, T)
    cache = oc.KVCache(shape, T + 8)
    cache.load(K.numpy().astype(np.float64), V.numpy().astype(np.float64))
    for l in range(shape.n_layers):
        eng.clasp_kv_load(l, K[l], V[l])
    toks = prompt(shape, 2, seed=6)
    st, lg = om.token(toks[0], T, cache, want_states=True)
    one = eng.clasp_verify_forward(dev(toks[:1], torch.int32), T, want_hidden=True, want_logits=True)
    assert relerr(one["hidden"][:, 0].cpu().numpy(), st) <= HID_TOL["bf16"]
    assert relerr(one["logits"][0].cpu().numpy(), lg) <= HID_TOL["bf16"]
    two = eng.clasp_verify_forward(dev(toks, torch.int32), T, want_hidden=True)
    # (the softmax weights enter the MFMA as fp16 and the two launches scale them against different running maxima)
    assert relerr(one["hidden"][:, 0].cpu().numpy(), two["hidden"][:, 0].cpu().numpy()) <= 5e-3
    # a draft step with a skip set at the next position
    mask = np.zeros(shape.n_layers, dtype=np.uint8)
    mask[1] = 1
    nxt = torch.zeros(1, dtype=torch.int32, device="cuda")
    eng.clasp_draft_step(mask.tolist(), dev(toks[1:2], torch.int32), T + 1, nxt)
    _, dl = om.token(toks[1], T + 1, cache, skip=mask)
    ref_tok, ref_margin = oc.argmax_margin(dl)
    if ref_margin > HID_TOL["bf16"] * np.abs(dl).max() * 2:
        assert int(nxt) == ref_tok


def test_two_row_groups_32_rows_and_budget_above_16():
    """max_rows = 32: a 32-row verify launch and a DP with M = 20 use two 16-row MFMA groups."""
    name = "small-bf16-deep"
    shape = si.SHAPES[name]
    om, eng = oracle_model(name, 1, 0.1), engine(name, 1, 0.1, max_seq=128, max_rows=32)
    toks = prompt(shape, 37)
    cache, ost, olg = oracle_prefill(om, toks, 64)
    tt = dev(toks, torch.int32)
    o1 = eng.clasp_verify_forward(tt[:32], 0, want_hidden=True, want_logits=True)
    o2 = eng.clasp_verify_forward(tt[32:], 32, want_hidden=True, want_logits=True)
    hid = torch.cat([o1["hidden"], o2["hidden"]], 1).cpu().numpy()
    for l in range(shape.n_layers + 1):
        assert relerr(hid[l], ost[l]) <= HID_TOL["bf16"], f"layer {l}"
    check_dp(om, eng, ost[:, -1], 36, cache, 20)
    check_dp(om, eng, ost[:, -1], 36, cache, 16)


def test_cache_conversion_saturates_instead_of_overflowing():
    """Keys / values of a bf16 model are cached as fp16: magnitudes beyond 65504 are stored as +-65504, not as
    infinities, and a forward pass over such a cache stays finite."""
    name = "small-bf16"
    shape = si.SHAPES[name]
    eng = engine(name, max_seq=64)
    K, V = si.gen_kv(shape, 5, 1, 40)
    K, V = K[0].clone(), V[0].clone()
    K[3, 0, 5], K[7, 1, 0], V[2, 0, 9], V[11, 1, 63] = 1.0e6, -7.0e4, -3.0e38, 65520.0
    eng.clasp_kv_load(0, K, V)
    Kr, Vr = eng.clasp_kv_read(0, 0, 40)
    assert float(Kr[3, 0, 5]) == 65504.0 and float(Kr[7, 1, 0]) == -65504.0
    assert float(Vr[2, 0, 9]) == -65504.0 and float(Vr[11, 1, 63]) == 65504.0
    assert torch.isfinite(Kr).all() and torch.isfinite(Vr).all()
    ok = K.abs() < 6.0e4
    assert torch.equal(Kr.cpu()[ok], K[ok].to(torch.float16).float())  # bf16-rounded inputs below the limit: exact or fp16-rounded
    out = eng.clasp_verify_forward(dev(prompt(shape, 3), torch.int32), 40, want_hidden=True, want_logits=True)
    assert torch.isfinite(out["hidden"]).all() and torch.isfinite(out["logits"]).all()
    eng.k_cache.zero_()
    eng.v_cache.zero_()


def test_empty_prefix_and_single_row():
    name = "tiny-f32"
    shape = si.SHAPES[name]
    om, eng = oracle_model(name), engine(name)
    cache = oc.KVCache(shape, 8)
    st, lg = om.token(5, 0, cache, want_states=True)
    out = eng.clasp_verify_forward(dev([5], torch.int32), 0, want_hidden=True, want_logits=True)
    assert relerr(out["hidden"][:, 0].cpu().numpy(), st) <= 1e-4
    assert relerr(out["logits"][0].cpu().numpy(), lg) <= 1e-4
    check_dp(om, eng, st, 0, oc.KVCache(shape, 8), 2)  # DP with no cached prefix at all


def test_same_call_twice_is_bit_identical():
    name = "small-bf16"
    shape = si.SHAPES[name]
    eng = engine(name)
    tt = dev(prompt(shape, 13), torch.int32)
    a = eng.clasp_verify_forward(tt, 0, want_hidden=True, want_logits=True)
    b = eng.clasp_verify_forward(tt, 0, want_hidden=True, want_logits=True)
    assert torch.equal(a["hidden"], b["hidden"]) and torch.equal(a["logits"], b["logits"])
    d1 = eng.clasp_dp_select(a["hidden"][:, 12, :], 12, 3, want_tables=True)
    d2 = eng.clasp_dp_select(a["hidden"][:, 12, :], 12, 3, want_tables=True)
    for k in d1:
        assert torch.equal(d1[k].view(torch.uint8), d2[k].view(torch.uint8)), k


def test_invalid_arguments_are_rejected_on_the_host():
    import paper_2505_24196_amd as clasp
    name = "tiny-f32"
    shape = si.SHAPES[name]
    eng = engine(name)
    tt = dev(prompt(shape, 20), torch.int32)
    with pytest.raises(clasp.ClaspError):
        eng.clasp_verify_forward(tt, 0)  # 20 rows > max_rows 16
    with pytest.raises(clasp.ClaspError):
        eng.clasp_verify_forward(tt[:4], 254)  # runs past max_seq
    st = torch.zeros(shape.n_layers + 1, shape.d_model, device="cuda")
    with pytest.raises(clasp.ClaspError):
        eng.clasp_dp_select(st, 3, shape.n_layers + 1)
    with pytest.raises(clasp.ClaspError):
        eng.clasp_dp_select(st, -1, 2)
    with pytest.raises(clasp.ClaspError):
        eng.clasp_draft_step(None, tt[:1], 256, tt[1:2])
    with pytest.raises(clasp.ClaspError):  # 100 rows is not a multiple of the 16-feature tile
        clasp.clasp_pack_matrix(torch.zeros(100, 128, dtype=torch.bfloat16, device="cuda"), "bf16")
    with pytest.raises(clasp.ClaspError):  # head_dim 24 is not one the bf16 kernels are built for
        clasp.Engine(si.ModelShape("bad", 2, 96, 4, 4, 24, 64, 1024, "bf16"), max_seq=64)


@pytest.mark.parametrize("resid_scale,M", [(1.0, 3), (0.05, 3), (1.0, 0)])
def test_closed_loop_tiny_matches_oracle_and_is_lossless(resid_scale, M):
    """Benchmark configuration 1: 64 random context tokens, M = 3, draft length 4, 32 generated tokens."""
    import paper_2505_24196_amd as clasp
    name = "tiny-f32"
    shape = si.SHAPES[name]
    om, eng = oracle_model(name, 1, resid_scale), engine(name, 1, resid_scale)
    pr = [int(t) for t in si.gen_tokens(2, 64, shape.vocab)]
    plain_ref, plain_margin = om.greedy_decode(pr, 32)
    plain_gpu, _ = clasp.greedy_generate(eng, pr, 32)
    spec_gpu = clasp.clasp_generate(eng, pr, 32, M, 4, trace=True)
    # lossless on the device: speculative tokens == the device's own plain greedy tokens
    assert spec_gpu["tokens"] == plain_gpu
    # against the oracle: identical up to the first step whose oracle logit margin is below tolerance
    for t, (a, b) in enumerate(zip(plain_gpu, plain_ref)):
        if a != b:
            assert plain_margin[t] < 1e-3, f"token {t} differs with oracle margin {plain_margin[t]}"
            break
    spec_ref = om.spec_decode(pr, 32, M, 4)
    assert spec_ref["tokens"] == plain_ref
    # every round of the device run against the oracle driven along it (near-ties follow the device, and are counted)
    st = replay_against_oracle(om, pr, spec_gpu, M, 4, 1e-3)
    assert st["rounds"] == len(spec_gpu["rounds"]) >= 32 // 5
    assert st["tokens"] >= 1 + 6 * st["rounds"] - 5 and st["tokens_forced"] <= max(2, st["tokens"] // 20), st
    if M:
        assert st["cells"] >= st["rounds"] * (M * shape.n_layers - M * M) and st["forced"] <= st["cells"] // 50 + 2, st
    if M == 0:
        assert all(r["accepted"] == 4 for r in spec_gpu["rounds"])
    if resid_scale == 0.05 and M:
        assert sum(r["accepted"] for r in spec_gpu["rounds"]) > 0


@pytest.mark.parametrize("thr", [0.0026, 1.5])
def test_closed_loop_with_draft_exiting_threshold(thr):
    """Sec. 5.3.3 on the device: rounds end at the first draft whose top-1 probability is below the threshold, the
    output stays the device's own plain greedy decoding, and round lengths follow the oracle's wherever no
    confidence sits within 5 % of the threshold (0.0026 is about the median confidence of this vocab-1024 model)."""
    import paper_2505_24196_amd as clasp
    name, M, K, n_gen = "tiny-f32", 3, 4, 24
    shape = si.SHAPES[name]
    om, eng = oracle_model(name, 1, 0.05), engine(name, 1, 0.05)
    pr = [int(t) for t in si.gen_tokens(2, 64, shape.vocab)]
    plain_gpu, _ = clasp.greedy_generate(eng, pr, n_gen)
    spec_gpu = clasp.clasp_generate(eng, pr, n_gen, M, K, trace=True, det_threshold=thr)
    assert spec_gpu["tokens"] == plain_gpu
    for r in spec_gpu["rounds"]:
        n = len(r["drafts"])
        assert 1 <= n <= K and len(r["verify"]) == n + 1 and r["accepted"] <= n
        assert all(c >= thr for c in r["draft_conf"][:-1]) and (n == K or r["draft_conf"][-1] < thr)
        if thr > 1.0:
            assert n == 1
    plain_ref, plain_margin = om.greedy_decode(pr, n_gen)
    spec_ref = om.spec_decode(pr, n_gen, M, K, det_threshold=thr)
    assert spec_ref["tokens"] == plain_ref
    # the oracle along the device's rounds: tables, skip sets, tokens and the confidences that end the rounds
    st = replay_against_oracle(om, pr, spec_gpu, M, K, 1e-3, thr=thr)
    assert st["rounds"] == len(spec_gpu["rounds"]) and st["tokens"] >= 2 * st["rounds"]
    assert st["tokens_forced"] <= max(2, st["tokens"] // 20) and st["forced"] <= st["cells"] // 50 + 2, st
    # where no confidence sits within 5 % of the threshold the oracle's own run has rounds of the same lengths
    if plain_gpu == plain_ref and not st["tokens_forced"] and not st["forced"]:
        for rg, ro in zip(spec_gpu["rounds"], spec_ref["rounds"]):
            if any(abs(c - thr) <= 0.05 * thr for c in ro["draft_conf"]):
                break
            assert len(rg["drafts"]) == len(ro["drafts"])


def test_two_row_groups_head_dim_128():
    """A 32-row verify launch and a DP with M = 20 on the head_dim-128 model (two 16-row MFMA groups, four column
    tiles per wavefront, 8 query tiles per KV head)."""
    name = "small-bf16-hd128"
    shape = si.SHAPES[name]
    om, eng = oracle_model(name, 1, 0.3), engine(name, 1, 0.3, max_seq=128, max_rows=32)
    toks = prompt(shape, 35)
    cache, ost, olg = oracle_prefill(om, toks, 64)
    tt = dev(toks, torch.int32)
    o1 = eng.clasp_verify_forward(tt[:32], 0, want_hidden=True, want_logits=True)
    o2 = eng.clasp_verify_forward(tt[32:], 32, want_hidden=True, want_logits=True)
    hid = torch.cat([o1["hidden"], o2["hidden"]], 1).cpu().numpy()
    for l in range(shape.n_layers + 1):
        assert relerr(hid[l], ost[l]) <= HID_TOL["bf16"], f"layer {l}"
    lg = torch.cat([o1["logits"], o2["logits"]], 0).cpu().numpy()
    assert relerr(lg, olg) <= HID_TOL["bf16"]
    check_dp(om, eng, ost[:, -1], 34, cache, 4)


def test_lower_optimisation_frequency_on_the_device():
    """dp_interval = 3 (Sec. 3.7): the skip set is kept for three verify steps; output still equals the device's own
    plain greedy decoding, and the masks change only at every third round."""
    import paper_2505_24196_amd as clasp
    name = "tiny-f32"
    shape = si.SHAPES[name]
    eng = engine(name, 1, 0.05)
    pr = [int(t) for t in si.gen_tokens(2, 40, shape.vocab)]
    plain, _ = clasp.greedy_generate(eng, pr, 24)
    spec = clasp.clasp_generate(eng, pr, 24, 3, 2, dp_interval=3)
    assert spec["tokens"] == plain
    masks = [r["mask"] for r in spec["rounds"]]
    for a, b, c in zip(masks[0::3], masks[1::3], masks[2::3]):
        assert a == b == c
    assert all(sum(m) == 3 for m in masks)
    curve = clasp.skip_set_jaccard(masks[::3], 4)
    assert all(0.0 <= x <= 1.0 for x in curve)


def test_budget_equal_to_depth_and_last_cache_position():
    """Degenerate ends of the ranges: M = L skips every layer (the draft model is embedding -> final norm -> lm_head),
    and the last position of the cache (pos = max_seq - 1) is usable by every call."""
    name = "tiny-f32"
    shape = si.SHAPES[name]
    L = shape.n_layers
    om, eng = oracle_model(name), engine(name, max_seq=64, max_rows=16)
    toks = prompt(shape, 63)
    cache, ost, olg = oracle_prefill(om, toks, 64)
    tt = dev(toks, torch.int32)
    for s in range(0, 63, 16):
        out = eng.clasp_verify_forward(tt[s:s + 16], s, want_hidden=True, want_logits=True)
    # rows 48..62: the last one sits at position 62; one more row at position 63 = max_seq - 1
    assert relerr(out["hidden"][:, -1].cpu().numpy(), ost[:, -1]) <= HID_TOL["f32"]
    last_tok = int(np.argmax(olg[-1]))
    st, lg = om.token(last_tok, 63, cache, want_states=True)
    one = eng.clasp_verify_forward(dev([last_tok], torch.int32), 63, want_hidden=True, want_logits=True)
    assert relerr(one["hidden"][:, 0].cpu().numpy(), st) <= HID_TOL["f32"]
    assert relerr(one["logits"][0].cpu().numpy(), lg) <= HID_TOL["f32"]
    # DP at the last position with M = L: every layer skipped, g(L, L) = x_0
    gpu, ref = check_dp(om, eng, st, 63, cache, L)
    assert gpu["mask"].cpu().numpy().tolist() == [1] * L == ref["mask"].tolist()
    assert relerr(gpu["g_final"].cpu().numpy(), st[0]) <= 1e-6
    # draft step that skips everything, at the last position
    nxt = torch.zeros(1, dtype=torch.int32, device="cuda")
    prob = torch.zeros(1, dtype=torch.float32, device="cuda")
    eng.clasp_draft_step([1] * L, dev([last_tok], torch.int32), 63, nxt, prob)
    _, dl = om.token(last_tok, 63, cache, skip=np.ones(L, dtype=np.uint8))
    ref_tok, ref_margin = oc.argmax_margin(dl)
    if ref_margin > 1e-3:
        assert int(nxt) == ref_tok
    assert abs(float(prob) - oc.top1_prob(dl)) <= 1e-3 * oc.top1_prob(dl)
    import paper_2505_24196_amd as clasp
    with pytest.raises(clasp.ClaspError):
        eng.clasp_verify_forward(dev([1, 2], torch.int32), 63)  # second row would sit at max_seq


# ---- window search and the objective of given skip sets (Sec. 3.5) -----------------------------------------------
@pytest.mark.parametrize("name,resid_scale,lo,hi,M", [("tiny-f32", 0.05, 2, 6, 2), ("small-bf16-deep", 0.05, 8, 16, 4),
                                                     ("small-bf16-deep", 1.0, 6, 18, 5)])
def test_window_search_matches_oracle(name, resid_scale, lo, hi, M):
    shape = si.SHAPES[name]
    om, eng = oracle_model(name, 1, resid_scale), engine(name, 1, resid_scale)
    toks = prompt(shape, 12)
    cache, ost, _ = oracle_prefill(om, toks, 16)
    tt = dev(toks, torch.int32)
    eng.clasp_verify_forward(tt, 0)
    pos, X = 11, ost[:, 11]
    check_dp(om, eng, X, pos, cache, M, lo, hi)


@pytest.mark.parametrize("name,resid_scale", [("tiny-f32", 1.0), ("small-bf16", 0.05), ("small-bf16-hd128", 1.0)])
def test_skip_cosine_matches_oracle(name, resid_scale):
    """Every skip set of two layers, the empty set and the full set: cosines of the masked forward's last state."""
    import itertools
    shape = si.SHAPES[name]
    L = shape.n_layers
    om, eng = oracle_model(name, 1, resid_scale), engine(name, 1, resid_scale)
    toks = prompt(shape, 10)
    cache, ost, _ = oracle_prefill(om, toks, 16)
    tt = dev(toks, torch.int32)
    eng.clasp_verify_forward(tt, 0)
    pos, X = 9, ost[:, 9]
    masks = [[0] * L, [1] * L] + [[1 if l in c else 0 for l in range(L)] for c in itertools.combinations(range(L), 2)]
    got = eng.clasp_skip_cosine(masks, tt[9:10], pos, dev(X[L])).cpu().numpy()
    ref = np.array([om.skip_cosine(X[0], pos, cache, m, X[L]) for m in masks])
    assert np.abs(got - ref).max() <= COS_TOL, np.abs(got - ref).max()
    assert abs(got[0] - 1.0) <= COS_TOL
    # the masked forward leaves the full model's cache rows below pos alone: the verify states are reproduced after it
    out = eng.clasp_verify_forward(tt[9:10], pos, want_hidden=True)
    assert relerr(out["hidden"][:, 0].cpu().numpy(), X) <= HID_TOL[shape.dtype]


def test_markov_study_rows_match_oracle():
    """decode.markov_study on a window of 6 layers (M = 2, 15 sets): brute-force optimum, the DP's set and its rank
    against the oracle's own enumeration."""
    import itertools
    from paper_2505_24196_amd import decode
    name, lo, hi, M = "small-bf16-deep", 9, 15, 2
    shape = si.SHAPES[name]
    L = shape.n_layers
    om, eng = oracle_model(name, 1, 0.05), engine(name, 1, 0.05)
    toks = prompt(shape, 10)
    cache, ost, _ = oracle_prefill(om, toks, 16)
    tt = dev(toks, torch.int32)
    eng.clasp_verify_forward(tt, 0)
    pos, X = 9, ost[:, 9]
    row = decode.markov_study(eng, dev(X), tt[9:10], pos, lo, hi, [M], n_random=8)[0]
    combos = list(itertools.combinations(range(lo, hi), M))
    ref = np.array([om.skip_cosine(X[0], pos, cache, [1 if l in c else 0 for l in range(L)], X[L]) for c in combos])
    assert row["sets"] == len(combos) == 15
    assert abs(row["brute_force_cos"] - ref.max()) <= COS_TOL
    order = np.sort(ref)[::-1]
    if order[0] - order[1] > COS_MARGIN:
        assert tuple(row["brute_force_set"]) == combos[int(ref.argmax())]
    dp_ref = om.window(lo, hi).dp(X[lo:hi + 1], pos, cache.window(lo, hi), M)
    margins = np.abs(dp_ref["sigma_c"] - dp_ref["sigma_s"])
    if np.nanmin(margins[1:, 1:]) > COS_MARGIN:
        assert row["dp_set"] == [lo + int(i) for i in np.flatnonzero(dp_ref["mask"])]
        k = combos.index(tuple(row["dp_set"]))
        assert abs(row["dp_cos"] - ref[k]) <= COS_TOL
    assert row["random_min_cos"] <= row["random_mean_cos"] <= row["brute_force_cos"] + 1e-6
    assert row["dp_cos"] <= row["brute_force_cos"] + 1e-6


def test_window_and_skip_cosine_reject_bad_arguments():
    from paper_2505_24196_amd.binding import ClaspError
    name = "small-bf16"
    shape = si.SHAPES[name]
    L = shape.n_layers
    eng = engine(name)
    X = dev(np.zeros((L + 1, shape.d_model)))
    tok = dev([1], torch.int32)
    for lo, hi, M in ((3, 3, 0), (4, 2, 1), (-1, 3, 1), (0, L + 1, 1), (1, 4, 4)):   # empty / reversed / outside / M > window
        with pytest.raises(ClaspError):
            eng.clasp_dp_select_window(X, 5, M, lo, hi)
    with pytest.raises(ClaspError):
        eng.clasp_skip_cosine([[0] * (L - 1)], tok, 5, X[L])          # mask of the wrong length
    with pytest.raises(ClaspError):
        eng.clasp_skip_cosine([[0] * L], tok, 256, X[L])              # position beyond max_seq
    # M = window: every layer of the window skipped, nothing outside it
    res = eng.clasp_dp_select_window(X, 5, 3, 1, 4)
    assert res["mask"].cpu().tolist() == [0, 1, 1, 1] + [0] * (L - 4)


@pytest.mark.parametrize("name,resid_scale,M", [("tiny-f32", 0.05, 3), ("tiny-f32", 1.0, 8), ("small-bf16", 1.0, 1),
                                               ("small-bf16-deep", 0.05, 12), ("small-bf16-deep", 1.0, 16),
                                               ("small-bf16-hd128", 0.05, 2)])
def test_search_without_tables_gives_the_same_set(name, resid_scale, M):
    """Without the tables the library leaves out the cells that cannot reach (L, M); the skip set must not change and
    g(L, M) only by fp32 rounding order (launches with fewer rows may take kernels that slice K differently). Also
    on a window of layers."""
    shape = si.SHAPES[name]
    L = shape.n_layers
    om, eng = oracle_model(name, 1, resid_scale), engine(name, 1, resid_scale, max_rows=32)
    toks = prompt(shape, 12)
    _, ost, _ = oracle_prefill(om, toks, 16)
    tt = dev(toks, torch.int32)
    eng.clasp_verify_forward(tt, 0)
    X = dev(ost[:, 11])
    full = eng.clasp_dp_select(X, 11, M, want_tables=True)
    lean = eng.clasp_dp_select(X, 11, M, want_g_final=True)
    assert torch.equal(full["mask"], lean["mask"]) and int(lean["mask"].sum()) == M
    assert relerr(lean["g_final"].cpu().numpy(), full["g_final"].cpu().numpy()) <= 1e-5
    if L >= 6 and M <= L - 4:
        lo, hi = 2, L - 2
        Mw = min(M, hi - lo)
        full = eng.clasp_dp_select_window(X, 11, Mw, lo, hi, want_tables=True)
        lean = eng.clasp_dp_select_window(X, 11, Mw, lo, hi)
        assert torch.equal(full["mask"], lean["mask"])
