"""GPU parity of the many-row prompt pass (clasp_prefill) against the CPU oracle's token-by-token full-model forward:
the cache it leaves (read back with clasp_kv_read), and the states / logits of the prompt's last token, which
clasp_verify_forward computes on top of that cache. Tolerance as for the other bf16 calls: 2e-2 of the largest
magnitude of the oracle tensor. Prompt lengths are chosen ragged (not multiples of 16, 128 or the chunk), several
chunks long; from 1024 tokens on the attention shares key / value blocks through LDS (head_dim 64 and 128); the
wide-FFN shape (1024 column tiles in gate|up) takes the 256 x 256 tile of that projection: on bf16 hi / lo planes at 500
tokens, on fp16 operands at 800 and 1300. Passes of 640
rows or more run on fp16 operands (one fp16 plane per activation, weights converted per layer): the 1100-, 1300- and
1700-token cases, the 24-layer shape among them, with the 256 x 256 tile in its fp16 form at 1300 tokens; the
many-heads shape (32 query and 32 KV heads of 64: 384 feature tiles in q/k/v, as many as the 8B shape has) sends the
q/k/v projection of its 2000 tokens through the 256 x 192 tile.
"""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import clasp_oracle as oc
from paper_2505_24196_amd import decode
from paper_2505_24196_amd.binding import ClaspError
from tests.helpers import oracle_model, prompt
from tests.test_gpu_parity import HID_TOL, dev, engine, relerr

pytestmark = pytest.mark.gpu

TOL = HID_TOL["bf16"]


def oracle_cache(om, toks, t_max, want_last=True):
    cache = oc.KVCache(om.shape, t_max)
    states = logits = None
    for t, tk in enumerate(toks):
        last = want_last and t == len(toks) - 1
        states, logits = om.token(tk, t, cache, want_states=last, want_logits=last)
    return cache, states, logits


def check_cache(eng, cache, lo, hi, what=""):
    """Device cache positions lo..hi-1 of every layer against the oracle's."""
    for l in range(eng.shape.n_layers):
        K, V = eng.clasp_kv_read(l, lo, hi - lo)
        ek = relerr(K.cpu().numpy(), cache.K[l, lo:hi])
        ev = relerr(V.cpu().numpy(), cache.V[l, lo:hi])
        assert ek <= TOL and ev <= TOL, f"{what} layer {l}: K {ek:.3e} V {ev:.3e}"


@pytest.mark.parametrize("name,T,chunk", [("small-bf16", 203, 128), ("small-bf16-hd128", 333, 256),
                                           ("small-bf16-deep", 150, 128), ("small-bf16", 130, 128), ("small-bf16", 1100, 1152),
                                           ("small-bf16-hd128", 1700, 2048), ("small-bf16-wide-ffn", 800, 1024), ("small-bf16-wide-ffn", 500, 512),
                                           ("small-bf16-wide-ffn", 1300, 1408), ("small-bf16-deep", 1100, 1152),
                                           ("small-bf16-many-heads", 2000, 2048)])
def test_prefill_cache_and_last_token_match_oracle(name, T, chunk):
    shape = si.SHAPES[name]
    max_seq = (T + 31) // 32 * 32
    om, eng = oracle_model(name), engine(name, max_seq=max_seq)
    toks = prompt(shape, T)
    cache, ost, olg = oracle_cache(om, toks, max_seq)
    tt = dev(toks, torch.int32)
    eng.clasp_prefill(tt[:T - 1], 0, chunk)
    check_cache(eng, cache, 0, T - 1, name)
    out = eng.clasp_verify_forward(tt[T - 1:], T - 1, want_hidden=True, want_logits=True)
    hid = out["hidden"][:, 0].cpu().numpy()
    for l in range(shape.n_layers + 1):
        assert relerr(hid[l], ost[l]) <= TOL, f"layer {l}"
    assert relerr(out["logits"][0].cpu().numpy(), olg) <= TOL
    ref_tok, ref_margin = oc.argmax_margin(olg)
    if ref_margin > TOL * np.abs(olg).max() * 2:
        assert int(out["argmax"][0]) == ref_tok


def test_prefill_continues_an_existing_prefix():
    """Rows at pos0 > 0 (not a multiple of 32) attend what earlier calls left in the cache."""
    name, T0, T = "small-bf16", 45, 45 + 140
    shape = si.SHAPES[name]
    om, eng = oracle_model(name), engine(name, max_seq=192)
    toks = prompt(shape, T)
    cache, _, _ = oracle_cache(om, toks, 192, want_last=False)
    tt = dev(toks, torch.int32)
    for s in range(0, T0, eng.max_rows):
        eng.clasp_verify_forward(tt[s:min(s + eng.max_rows, T0)], s)
    eng.clasp_prefill(tt[T0:], T0, 128)
    check_cache(eng, cache, 0, T)


@pytest.mark.parametrize("T0,T,chunk0,chunk1", [(1003, 1303, 1024, 384), (1100, 2301, 1152, 1280)])
def test_prefill_continues_a_long_prefix(T0, T, chunk0, chunk1):
    """T0 tokens in place, the rest on top: the second call's attention walks the whole prefix through the LDS ring,
    starting from a position that is not a multiple of 32. First case: both calls are bf16 passes; second case: both are
    fp16 passes (1100 and 1201 rows)."""
    name = "small-bf16"
    shape = si.SHAPES[name]
    max_seq = (T + 31) // 32 * 32
    om, eng = oracle_model(name), engine(name, max_seq=max_seq)
    toks = prompt(shape, T)
    cache, _, _ = oracle_cache(om, toks, max_seq, want_last=False)
    tt = dev(toks, torch.int32)
    eng.clasp_prefill(tt[:T0], 0, chunk0)
    eng.clasp_prefill(tt[T0:], T0, chunk1)
    check_cache(eng, cache, 0, T)


@pytest.mark.parametrize("T,chunk", [(300, 128), (1100, 1152)])
def test_prefill_twice_is_bit_identical(T, chunk):
    """No atomics, fixed-order sums: the same prompt pass leaves the same bits (bf16 passes and fp16 passes alike)."""
    name = "small-bf16"
    shape = si.SHAPES[name]
    eng = engine(name, max_seq=(T + 31) // 32 * 32)
    tt = dev(prompt(shape, T), torch.int32)
    eng.clasp_prefill(tt, 0, chunk)
    first = [tuple(t.clone() for t in eng.clasp_kv_read(l, 0, T)) for l in range(shape.n_layers)]
    eng.clasp_prefill(tt, 0, chunk)
    for l in range(shape.n_layers):
        K, V = eng.clasp_kv_read(l, 0, T)
        assert torch.equal(K, first[l][0]) and torch.equal(V, first[l][1]), f"layer {l}"


def test_prefill_agrees_with_the_row_limited_path():
    """Same prompt through clasp_verify_forward in chunks of max_rows: the two caches agree to rounding."""
    name, T = "small-bf16-hd128", 300
    shape = si.SHAPES[name]
    eng = engine(name, max_seq=320)
    tt = dev(prompt(shape, T), torch.int32)
    for s in range(0, T, eng.max_rows):
        eng.clasp_verify_forward(tt[s:s + eng.max_rows], s)
    ref = [eng.clasp_kv_read(l, 0, T) for l in range(shape.n_layers)]
    ref = [(k.clone(), v.clone()) for k, v in ref]
    eng.clasp_prefill(tt, 0, 128)
    for l in range(shape.n_layers):
        K, V = eng.clasp_kv_read(l, 0, T)
        assert relerr(K.cpu().numpy(), ref[l][0].cpu().numpy()) <= 1e-2
        assert relerr(V.cpu().numpy(), ref[l][1].cpu().numpy()) <= 1e-2


def test_decode_prefill_routes_long_prompts_through_it():
    name, T = "small-bf16", 130
    shape = si.SHAPES[name]
    om, eng = oracle_model(name), engine(name, max_seq=160)
    toks = prompt(shape, T)
    _, ost, olg = oracle_cache(om, toks, 160)
    states, nxt, _ = decode.prefill(eng, toks)
    assert relerr(states.cpu().numpy(), ost) <= TOL
    slow_states, slow_nxt, _ = decode.prefill(eng, toks, chunk_rows=0)
    assert relerr(states.cpu().numpy(), slow_states.cpu().numpy()) <= 1e-2
    ref_tok, ref_margin = oc.argmax_margin(olg)
    if ref_margin > TOL * np.abs(olg).max() * 2:
        assert int(nxt) == ref_tok == int(slow_nxt)


def test_kv_read_inverts_kv_load():
    name = "small-bf16"
    shape = si.SHAPES[name]
    eng = engine(name, max_seq=160)
    K, V = si.gen_kv(shape, 5, 1, 77, "cuda")
    eng.clasp_kv_load(2, K[0], V[0])
    Kr, Vr = eng.clasp_kv_read(2, 0, 77)
    assert torch.equal(Kr, K[0].to(torch.bfloat16).to(torch.float32))
    assert torch.equal(Vr, V[0].to(torch.bfloat16).to(torch.float32))
    Kp, _ = eng.clasp_kv_read(2, 33, 10)
    assert torch.equal(Kp, Kr[33:43])


def test_prefill_rejects_what_it_cannot_run():
    eng = engine("small-bf16", max_seq=160)
    tt = dev(prompt(si.SHAPES["small-bf16"], 100), torch.int32)
    with pytest.raises(ClaspError):
        eng.clasp_prefill(tt, 0, 100)       # chunk_rows not a multiple of 128
    with pytest.raises(ClaspError):
        eng.clasp_prefill(tt, 100, 128)     # runs past max_seq
    with pytest.raises(ClaspError):
        engine("tiny-f32").clasp_prefill(tt, 0, 128)   # fp32 models take the row-limited path
