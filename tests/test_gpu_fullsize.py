"""Parity at the benchmark's full size (LLaMA-3-8B shape, bf16, M = 12), in the launch configuration bench.py times.
test_8b_model_made_prefix_* is the setting of Sec. 3.1 / 3.4 as it stands: each side (fp64 oracle, device) runs the
full model over the same prompt itself, and the verify states, the DP on the device's own states and a draft step are
compared on top of each side's own cache, so the rounding of the device's cached keys / values is part of what is
measured. For the long prefixes of the context sweep (T >= 2048; the oracle's prefill would take hours) a seeded
synthetic KV prefix, a shared input, stands in on both sides."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import clasp_oracle as oc
from tests.test_gpu_parity import (COS_TOL, HID_TOL, assert_close, check_dp, dev, relerr, relerr_rows,
                                   replay_against_oracle)

pytestmark = pytest.mark.gpu


MAX_T = 32768


@pytest.fixture(scope="module")
def setup_8b():
    import bench
    shape = si.LLAMA3_8B
    T = 512
    eng, host = bench.build_engine(shape, 1, MAX_T + 64, 16, keep_host=True)
    om = oc.OracleModel(shape, host)
    K, V = si.gen_kv(shape, 3, shape.n_layers, T)
    cache = oc.KVCache(shape, T + 8)
    cache.load(K.numpy().astype(np.float64), V.numpy().astype(np.float64))
    for l in range(shape.n_layers):
        eng.clasp_kv_load(l, K[l], V[l])
    yield shape, T, eng, om, cache
    eng.close()


def verify_dp_draft(shape, T, eng, om, cache, M=12):
    """Two verify rows at positions T, T+1 on top of a T-token prefix, the DP on row 1, one draft step."""
    toks = [int(t) for t in si.gen_tokens(2, 3, shape.vocab, stream=9)]
    st, lg = [], []
    for r, tk in enumerate(toks):
        print(f"oracle verify row {r}", flush=True)
        s, l_ = om.token(tk, T + r, cache, want_states=True)
        st.append(s)
        lg.append(l_)
    ost, olg = np.stack(st, 1), np.stack(lg)
    out = eng.clasp_verify_forward(dev(toks, torch.int32), T, want_hidden=True, want_logits=True)
    for l in range(shape.n_layers + 1):
        assert_close(out["hidden"][l].cpu().numpy(), ost[l], HID_TOL["bf16"], f"layer {l}")
    assert_close(out["logits"].cpu().numpy(), olg, HID_TOL["bf16"], "logits")
    # DP on row 1 (position T+1), the device on the states its own verify pass captured, the oracle on its own;
    # cache rows 0..T are the prefix plus row 0's own k/v on either side
    print("oracle dp", flush=True)
    stats = {}
    X_dev = out["hidden"][:, 1, :].contiguous()
    gpu, ref = check_dp(om, eng, ost[:, 1], T + 1, cache, M, X_dev=X_dev, stats=stats)
    L = shape.n_layers
    assert stats["cells"] == sum(min(i, M) for i in range(1, L + 1)) and stats["forced"] <= stats["cells"] // 25, stats
    # the call as bench.py issues it (no tables: cells that cannot reach (L, M) are left out) selects the same set
    lean = eng.clasp_dp_select(X_dev, T + 1, M)
    assert torch.equal(lean["mask"], gpu["mask"])
    # one draft step with the selected skip set, from row 2's token at position T+2: the draft model's logits (every
    # one of them, whatever the margin), its greedy token where the margin allows, and the top-1 probability
    print("oracle draft", flush=True)
    mask = ref["mask"].tolist()
    nxt = torch.zeros(2, dtype=torch.int32, device="cuda")
    prob = torch.zeros(1, dtype=torch.float32, device="cuda")
    lg_dev = torch.empty(shape.vocab, dtype=torch.float32, device="cuda")
    eng.clasp_draft_sample(mask, dev(toks[2:3], torch.int32), T + 2, 1.0, dev([0.5]), lg_dev, nxt[1:2])
    eng.clasp_draft_step(mask, dev(toks[2:3], torch.int32), T + 2, nxt[0:1], prob)
    _, dl = om.token(toks[2], T + 2, cache, skip=ref["mask"])
    assert_close(lg_dev.cpu().numpy()[None], dl[None], HID_TOL["bf16"], "draft logits")
    assert int(nxt[0]) == int(torch.argmax(lg_dev))
    ref_tok, ref_margin = oc.argmax_margin(dl)
    if ref_margin > HID_TOL["bf16"] * np.abs(dl).max() * 2:
        assert int(nxt[0]) == ref_tok
    assert abs(float(prob) - oc.top1_prob(dl)) <= 0.05 * oc.top1_prob(dl)
    return stats


def test_8b_verify_dp_and_draft(setup_8b):
    shape, T, eng, om, cache = setup_8b
    verify_dp_draft(shape, T, eng, om, cache)


def load_prefix(shape, eng, cache, T, n_layers):
    """Synthetic prefix of T tokens for the first n_layers layers, drawn layer by layer with the shared generator (on
    the device, where a billion draws take seconds) and handed to both sides."""
    for l in range(n_layers):
        K, V = si.gen_kv(shape, 1000 + l, 1, T, "cuda")
        eng.clasp_kv_load(l, K[0], V[0])
        cache.K[l, :T] = K[0].cpu().numpy()
        cache.V[l, :T] = V[0].cpu().numpy()
    print(f"prefix of {T} tokens loaded", flush=True)


def test_8b_long_prefix_verify_dp_and_draft(setup_8b):
    """The same calls on an 8192-token prefix of the benchmark's context sweep (split attention and its merge), with the
    sweep's smaller skip budget M = 8 (the oracle's search costs ~0.2 s per candidate row and layer at this length)."""
    shape, _, eng, om, _ = setup_8b
    T = 8192
    cache = oc.KVCache(shape, T + 8)
    load_prefix(shape, eng, cache, T, shape.n_layers)
    verify_dp_draft(shape, T, eng, om, cache, M=8)


def test_8b_mid_prefix_largest_budget(setup_8b):
    """2048-token prefix with the context sweep's largest skip budget, M = 16: a full 16-row group of candidates from
    level 17 on (the DP, its lean form, and a draft step with 16 of the 32 layers skipped)."""
    shape, _, eng, om, _ = setup_8b
    T = 2048
    cache = oc.KVCache(shape, T + 8)
    load_prefix(shape, eng, cache, T, shape.n_layers)
    verify_dp_draft(shape, T, eng, om, cache, M=16)


def test_8b_longest_prefix_first_layers(setup_8b):
    """32768-token prefix (two query tiles per workgroup, 64-way split, merge kernel). The oracle's plain attention
    loop takes ~0.7 s per row and layer here, so the comparison covers the first 8 layers: two verify rows' states
    0..8 and the search restricted to those layers (M = 6, up to 6 candidate rows per layer)."""
    shape, _, eng, om, _ = setup_8b
    T, Lw, M = MAX_T, 8, 6
    omw = om.window(0, Lw)
    cache = oc.KVCache(omw.shape, T + 8)
    load_prefix(shape, eng, cache, T, Lw)
    toks = [int(t) for t in si.gen_tokens(2, 2, shape.vocab, stream=9)]
    st = []
    for r, tk in enumerate(toks):
        print(f"oracle verify row {r}, {Lw} layers", flush=True)
        s, _ = omw.token(tk, T + r, cache, want_states=True, want_logits=False)
        st.append(s)
    ost = np.stack(st, 1)
    out = eng.clasp_verify_forward(dev(toks, torch.int32), T, want_hidden=True)
    for l in range(Lw + 1):
        assert relerr(out["hidden"][l].cpu().numpy(), ost[l]) <= HID_TOL["bf16"], f"layer {l}"
    print("oracle dp, window of 8 layers", flush=True)
    X = np.zeros((shape.n_layers + 1, shape.d_model))
    X[:Lw + 1] = ost[:, 1]
    check_dp(om, eng, X, T + 1, cache, M, 0, Lw)   # the cache holds exactly the window's layers


def cdf_margin_bound(V, mass=1.0, max_arg=16.0):
    """How far (as a fraction of the total weight) the device's fp32 inverse-CDF draw can sit from the fp64 one, from
    the arithmetic of sample_kernel / spec_accept_kernel: a running sum is reached through at most 2 * ceil(V / 1024)
    additions inside per-thread chunks, 64 + 63 inside a wavefront's 64 chunk sums, 16 over the wavefront totals and a
    couple more, each rounding by at most 2^-24 of a value no larger than the total; every weight is
    exp((logit - max) / T) with the argument (|argument| <= max_arg where it matters) rounded twice (2^-23 relative)
    and expf good to 2 units in the last place (2^-22), and an interval has two ends. Weights that are differences
    max(p - q, 0) carry the errors of p and q, which are fractions of THEIR totals (1), so the bound grows by
    1 / mass when the drawn-from weights only add up to `mass`."""
    adds = 2 * -(-V // 1024) + 64 + 63 + 16 + 2
    weights = 2 * (max_arg * 2.0 ** -23 + 2.0 ** -22)
    return (adds * 2.0 ** -24 + weights) / mass


def test_8b_vocab_sampling_and_acceptance(setup_8b):
    """Inverse-CDF draws and one acceptance round at the full vocabulary (128256 entries, 126 per thread with a ragged
    last chunk), on synthetic logits, against the fp64 oracle. A draw is compared wherever the oracle's distance to
    the nearest interval end exceeds cdf_margin_bound (2.8e-5 of the total for a softmax at this vocabulary)."""
    shape, T, eng, om, cache = setup_8b
    V = shape.vocab
    n = 4
    p_lg = si.gen_matrix(21, 900, n + 1, V, 2.0, "f32").numpy()
    q_lg = (p_lg[:n] + 0.3 * si.gen_matrix(22, 901, n, V, 2.0, "f32").numpy()).astype(np.float32)
    us = si.gen_uniform(23, 128, 0)
    d_tok = torch.zeros(1, dtype=torch.int32, device="cuda")
    d_lg, d_u = dev(p_lg[0]), us.cuda()
    w = oc.softmax_t(p_lg[0])
    bound = cdf_margin_bound(V)
    assert 2e-5 < bound < 4e-5
    checked = 0
    for i in range(128):
        eng.clasp_sample_token(d_lg, 1.0, d_u[i:i + 1], d_tok)
        ref, margin = oc.sample_cdf(w, float(us[i]))
        if margin > bound:
            assert int(d_tok) == ref
            checked += 1
    assert checked >= 40, checked  # about 0.4 of the draws clear the bound at this vocabulary
    res = torch.zeros(2, dtype=torch.int32, device="cuda")
    compared = 0
    for trial in range(24):
        u = si.gen_uniform(30 + trial, 2 * n + 1, 3).numpy()
        drafts = [oc.sample_cdf(oc.softmax_t(q_lg[i]), float(u[i]))[0] for i in range(n)]
        a_ref, tok_ref, info = oc.spec_accept(p_lg, q_lg, drafts, u[n:2 * n], float(u[2 * n]))
        eng.clasp_spec_accept(dev(p_lg), dev(q_lg), dev([1] + drafts, torch.int32), n, 1.0, dev(u[n:2 * n]),
                              dev(u[2 * n:]), res[0:1], res[1:2])
        a, tok = res.cpu().tolist()
        if min(info["ratio_margin"]) > 1e-4:
            assert a == a_ref
            # a rejected round draws from max(p - q, 0), whose weights add up to less than one
            mass = 1.0 if a_ref == n else float(np.maximum(oc.softmax_t(p_lg[a_ref]) - oc.softmax_t(q_lg[a_ref]), 0).sum())
            if info["cdf_margin"] > cdf_margin_bound(V, mass):
                assert tok == tok_ref
                compared += 1
    assert compared >= 6, compared


def test_8b_model_made_prefix_verify_dp_and_draft(setup_8b):
    """Benchmark configuration 2 as the paper defines it (Sec. 3.1, 3.4): the DP runs on states and a cache that the
    verify model itself produced. Oracle and device each run the full model over the same 160 random prompt tokens
    (the device through clasp_prefill in passes of 128 rows, then again through clasp_verify_forward in chunks of
    max_rows: both caches are held to the oracle's, layer by layer, at the stated bf16 bound), then two verify rows
    (all 33 states), the DP with M = 12 on the device's own states, and a draft step, each on the side's own cache."""
    shape, _, eng, om, _ = setup_8b
    T = 160
    toks = [int(t) for t in si.gen_tokens(2, T, shape.vocab, stream=13)]
    cache = oc.KVCache(shape, T + 40)
    for t, tk in enumerate(toks):
        if t % 16 == 0:
            print(f"oracle prompt token {t}", flush=True)
        om.token(tk, t, cache, want_logits=False)
    tt = dev(toks, torch.int32)
    for s in range(0, T, eng.max_rows):
        eng.clasp_verify_forward(tt[s:s + eng.max_rows], s)
    rows = [tuple(x.cpu().numpy() for x in eng.clasp_kv_read(l, 0, T)) for l in range(shape.n_layers)]
    eng.clasp_prefill(tt, 0, 128)
    worst = 0.0
    for l in range(shape.n_layers):
        K, V = (x.cpu().numpy() for x in eng.clasp_kv_read(l, 0, T))
        for name, got, slow, ref in (("K", K, rows[l][0], cache.K[l, :T]), ("V", V, rows[l][1], cache.V[l, :T])):
            assert_close(got.reshape(T, -1), ref.reshape(T, -1), HID_TOL["bf16"], f"{name} layer {l}")
            assert_close(slow.reshape(T, -1), ref.reshape(T, -1), HID_TOL["bf16"], f"{name} layer {l}, row-limited path")
            worst = max(worst, relerr(got, ref), relerr(slow, ref))
    print(f"largest cache error over 32 layers: {worst:.3e}", flush=True)
    stats = verify_dp_draft(shape, T, eng, om, cache)
    print(f"dp cells compared: {stats}", flush=True)
    # benchmark configuration 2's loop (M = 12, K = 4) from this prompt for a few rounds, the oracle driven along the
    # device's trace on the cache it built above (rows beyond the prompt are rewritten by the rounds themselves)
    from paper_2505_24196_amd import decode
    n_gen = 6
    spec = decode.clasp_generate(eng, toks, n_gen, 12, 4, trace=True)
    assert len(spec["tokens"]) == n_gen
    print(f"closed loop: {len(spec['rounds'])} rounds", flush=True)
    st_last, lg_last = om.token(toks[-1], T - 1, cache, want_states=True)
    logit_tol = HID_TOL["bf16"] * float(np.abs(lg_last).max()) * 2
    rs = replay_against_oracle(om, toks, spec, 12, 4, logit_tol, prefilled=(cache, st_last, lg_last))
    print(f"closed loop replay: {rs}", flush=True)
    assert rs["rounds"] == len(spec["rounds"]) >= 1 and rs["cells"] >= 318 * rs["rounds"]
    assert rs["forced"] <= rs["cells"] // 25 and rs["tokens"] >= 1 + 9 * rs["rounds"] - 8


def test_8b_prefill_short_prompt_against_oracle(setup_8b):
    """clasp_prefill at the full layer shapes against the oracle's token-by-token forward: 23 prompt tokens leave the
    cache, the 24th goes through clasp_verify_forward on top of it. The row-limited path on the same prompt is held to
    the same bound (the stated bf16 one, on every layer), and the two device caches to each other."""
    shape, T, eng, om, _ = setup_8b
    n = 24
    toks = [int(t) for t in si.gen_tokens(2, n, shape.vocab, stream=11)]
    cache = oc.KVCache(shape, 32)
    ost = None
    for t, tk in enumerate(toks):
        ost, _ = om.token(tk, t, cache, want_states=(t == n - 1), want_logits=False)
    tt = dev(toks, torch.int32)
    eng.clasp_verify_forward(tt[:16], 0)
    eng.clasp_verify_forward(tt[16:n - 1], 16)
    rows = [tuple(x.cpu().numpy() for x in eng.clasp_kv_read(l, 0, n - 1)) for l in range(shape.n_layers)]
    eng.clasp_prefill(tt[:n - 1], 0, 128)
    for l in range(shape.n_layers):
        K, V = (x.cpu().numpy() for x in eng.clasp_kv_read(l, 0, n - 1))
        for name, got, slow, ref in (("K", K, rows[l][0], cache.K[l, :n - 1]), ("V", V, rows[l][1], cache.V[l, :n - 1])):
            assert relerr(got, ref) <= HID_TOL["bf16"], f"{name} layer {l}"
            assert relerr(slow, ref) <= HID_TOL["bf16"], f"{name} layer {l}, row-limited path"
            assert relerr(got, slow) <= HID_TOL["bf16"], f"{name} layer {l}, between the device paths"
    out = eng.clasp_verify_forward(tt[n - 1:], n - 1, want_hidden=True)
    hid = out["hidden"][:, 0].cpu().numpy()
    for l in range(shape.n_layers + 1):
        assert relerr(hid[l], ost[l]) <= HID_TOL["bf16"], f"layer {l}"


def test_8b_closed_loop_emits_plain_greedy_tokens(setup_8b):
    """Benchmark configuration 5 (4096-token prompt, M = 12, K = 6) for 40 tokens: the draft / verify / optimise loop
    emits exactly what plain greedy decoding with the full model emits. The two runs push different numbers of rows
    through the kernels, which changes rounding order: a difference is only accepted where plain decoding's own top-1
    margin is below what that can move a logit by, and nothing after it is compared."""
    from paper_2505_24196_amd import decode
    shape, _, eng, _, _ = setup_8b
    prompt = [int(t) for t in si.gen_tokens(2, 4096, shape.vocab)]
    n_gen = 40
    plain, margins = decode.greedy_generate(eng, prompt, n_gen)
    spec = decode.clasp_generate(eng, prompt, n_gen, 12, 6)
    assert len(spec["tokens"]) == n_gen and all(1 <= r["accepted"] + 1 <= 7 for r in spec["rounds"])
    assert all(sum(r["mask"]) == 12 for r in spec["rounds"])
    first = next((i for i, (a, b) in enumerate(zip(plain, spec["tokens"])) if a != b), None)
    if first is not None:
        assert margins[first] < 1e-3, f"token {first} differs where plain decoding's margin is {margins[first]}"


@pytest.mark.parametrize("n,chunk", [(700, 1024), (4100, 4096), (8200, 8192)])
def test_8b_prefill_in_the_timed_configuration(setup_8b, n, chunk):
    """Ragged prompts in passes of 1024 rows (256 x 256 tiles for gate|up, 128 x 128 elsewhere), of 4096 rows (the
    timed configuration: 256 x 256 tiles for o_proj, gate|up and down, 256 x 192 for q/k/v, fp16 operands) and of 8192
    rows (the largest pass, what decode.prefill uses for prompts that long). Against the oracle: layer 0's keys / values at
    sampled positions (they need no prefix) and layer 1's at the first 16 positions (they go through all of layer 0:
    attention over a short prefix, o_proj, gate|up, down). Every layer's cache against the one clasp_verify_forward
    leaves for the same prompt in chunks of max_rows, which test_8b_verify_dp_and_draft ties to the oracle."""
    shape, T, eng, om, _ = setup_8b
    toks = si.gen_tokens(2, n, shape.vocab, stream=12)
    tt = toks.to("cuda")
    for s in range(0, n, eng.max_rows):
        eng.clasp_verify_forward(tt[s:s + eng.max_rows], s)
    ref = []
    for l in range(shape.n_layers):
        K, V = eng.clasp_kv_read(l, 0, n)
        ref.append((K.cpu().numpy(), V.cpu().numpy()))
    eng.clasp_prefill(tt, 0, chunk)
    embed = om.w["embed"]
    for pos in (0, 1, 127, 128, 333, n - 1):
        row = (embed[int(toks[pos])].astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        _, kn, vn = om.layer(0, row, pos, 0, np.zeros((1, shape.kv_dim)), np.zeros((1, shape.kv_dim)))
        K, V = eng.clasp_kv_read(0, pos, 1)
        assert relerr(K.cpu().numpy().ravel(), kn) <= HID_TOL["bf16"], f"K position {pos}"
        assert relerr(V.cpu().numpy().ravel(), vn) <= HID_TOL["bf16"], f"V position {pos}"
    om2 = om.window(0, 2)
    c2 = oc.KVCache(om2.shape, 16)
    for pos in range(16):
        om2.token(int(toks[pos]), pos, c2, want_logits=False)
    K, V = eng.clasp_kv_read(1, 0, 16)
    assert relerr(K.cpu().numpy(), c2.K[1]) <= HID_TOL["bf16"]
    assert relerr(V.cpu().numpy(), c2.V[1]) <= HID_TOL["bf16"]
    for l in range(shape.n_layers):
        K, V = eng.clasp_kv_read(l, 0, n)
        assert relerr(K.cpu().numpy(), ref[l][0]) <= HID_TOL["bf16"], f"K layer {l}"
        assert relerr(V.cpu().numpy(), ref[l][1]) <= HID_TOL["bf16"], f"V layer {l}"
