"""Pins of the oracle's model forward (CPU only).

The oracle runs one row at a time against a KV cache. It is pinned here against
  * a full-sequence forward assembled from PyTorch library routines (F.rms_norm, F.linear,
    F.scaled_dot_product_attention with a causal mask and grouped queries, F.silu; rotary embedding as a complex
    multiplication) -- a different formulation (batched, masked, no cache) through different code,
  * closed forms and special cases of the layer (Sec. 3.4: h_{l+1} = f_l(h_l); the layer itself is the LLaMA
    decoder block the paper's models use, "Model and Testbed").
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth_inputs as si
from oracle import clasp_oracle as oc
from tests.helpers import oracle_model, prompt, torch_model


def _as64(t):
    return t.to(torch.float64)


def library_forward(shape, model, tokens):
    """Whole-sequence forward from library routines. Returns (states [L+1][T][d], logits [T][V], K, V caches)."""
    T = len(tokens)
    hd, nq, nkv = shape.head_dim, shape.n_heads, shape.n_kv_heads
    h = _as64(model["embed"])[torch.tensor(tokens)]
    pos = torch.arange(T, dtype=torch.float64)
    inv = shape.rope_base ** (-torch.arange(0, hd, 2, dtype=torch.float64) / hd)
    rot = torch.polar(torch.ones(T, hd // 2, dtype=torch.float64), pos[:, None] * inv[None, :])  # e^{i theta}

    def rope(x):  # x [T][heads][hd], pairs (k, k+hd/2) form the complex number
        z = torch.complex(x[..., : hd // 2], x[..., hd // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    states, Ks, Vs = [h], [], []
    for lw in model["layers"]:
        n1 = F.rms_norm(h, (shape.d_model,), _as64(lw["attn_norm"]), shape.rms_eps)
        q = rope(F.linear(n1, _as64(lw["wq"])).view(T, nq, hd))
        k = rope(F.linear(n1, _as64(lw["wk"])).view(T, nkv, hd))
        v = F.linear(n1, _as64(lw["wv"])).view(T, nkv, hd)
        att = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None],
                                             v.transpose(0, 1)[None], is_causal=True, enable_gqa=True)[0]
        a = h + F.linear(att.transpose(0, 1).reshape(T, nq * hd), _as64(lw["wo"]))
        n2 = F.rms_norm(a, (shape.d_model,), _as64(lw["mlp_norm"]), shape.rms_eps)
        h = a + F.linear(F.silu(F.linear(n2, _as64(lw["w_gate"]))) * F.linear(n2, _as64(lw["w_up"])),
                         _as64(lw["w_down"]))
        states.append(h)
        Ks.append(k)
        Vs.append(v)
    logits = F.linear(F.rms_norm(h, (shape.d_model,), _as64(model["final_norm"]), shape.rms_eps),
                      _as64(model["lm_head"]))
    return torch.stack(states).numpy(), logits.numpy(), torch.stack(Ks).numpy(), torch.stack(Vs).numpy()


@pytest.mark.parametrize("name", ["tiny-f32", "small-bf16"])
def test_incremental_oracle_matches_library_full_sequence(name):
    shape = si.SHAPES[name]
    om, tm = oracle_model(name), torch_model(name)
    toks = prompt(shape, 11)
    ref_states, ref_logits, ref_K, ref_V = library_forward(shape, tm, toks)
    cache = oc.KVCache(shape, 16)
    for t, tok in enumerate(toks):
        st, lg = om.token(tok, t, cache, want_states=True)
        np.testing.assert_allclose(st, ref_states[:, t], rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(lg, ref_logits[t], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(cache.K[:, :11], ref_K, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(cache.V[:, :11], ref_V, rtol=1e-10, atol=1e-12)


def _patched(name, **repl):
    """Oracle model whose listed per-layer matrices are replaced (value: callable(layer, tensor) -> tensor)."""
    shape = si.SHAPES[name]
    tm = torch_model(name)
    m = {k: v for k, v in tm.items() if k != "layers"}
    m["layers"] = []
    for l, lw in enumerate(tm["layers"]):
        lw = dict(lw)
        for key, fn in repl.items():
            lw[key] = fn(l, lw[key])
        m["layers"].append(lw)
    return oc.OracleModel(shape, si.model_to_numpy(m)), m


def test_layer_is_identity_when_residual_writers_are_zero():
    om, _ = _patched("tiny-f32", wo=lambda l, w: torch.zeros_like(w), w_down=lambda l, w: torch.zeros_like(w))
    shape = om.shape
    h = si.gen_states(shape, 5, 1).numpy()[0].astype(np.float64)
    cache = oc.KVCache(shape, 4)
    out, _, _ = om.layer(2, h, 3, 0, cache.K[2], cache.V[2])
    assert np.array_equal(out, h)


def test_rmsnorm_constant_vector_rope_at_zero_and_empty_prefix():
    """h = c*ones: RMSNorm gives ones*c/sqrt(c^2+eps), so k at position 0 (no rotation) is that scalar times the
    row sums of Wk; with an empty prefix the softmax has one term, so attention returns the row's own v and
    a = h + Wo . repeat(v) (each query head reads its group's value head)."""
    name = "small-bf16"
    om, tm = oracle_model(name), torch_model(name)
    shape = om.shape
    c = 0.37
    h = np.full(shape.d_model, c)
    r = c / np.sqrt(c * c + shape.rms_eps)
    lw = tm["layers"][1]
    cache = oc.KVCache(shape, 2)
    _, k_new, v_new = om.layer(1, h, 0, 0, cache.K[1], cache.V[1])
    np.testing.assert_allclose(k_new, r * _as64(lw["wk"]).sum(1).numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(v_new, r * _as64(lw["wv"]).sum(1).numpy(), rtol=1e-12, atol=1e-14)
    # mlp off -> out = a
    om2, m2 = _patched(name, w_down=lambda l, w: torch.zeros_like(w))
    out, _, v2 = om2.layer(1, h, 0, 0, cache.K[1], cache.V[1])
    group = shape.n_heads // shape.n_kv_heads
    att = np.repeat(v2.reshape(shape.n_kv_heads, shape.head_dim), group, axis=0).reshape(-1)
    np.testing.assert_allclose(out, h + _as64(lw["wo"]).numpy() @ att, rtol=1e-12, atol=1e-14)


def test_zero_query_gives_mean_of_values():
    name = "small-bf16"
    om, m = _patched(name, wq=lambda l, w: torch.zeros_like(w), w_down=lambda l, w: torch.zeros_like(w))
    shape = om.shape
    T = 7
    K, V = si.gen_kv(shape, 3, 1, T)
    cache = oc.KVCache(shape, T + 1)
    cache.load(K.numpy().astype(np.float64), V.numpy().astype(np.float64), layers=[0])
    h = si.gen_states(shape, 9, 1).numpy()[0].astype(np.float64)
    out, _, v_own = om.layer(0, h, T, T, cache.K[0], cache.V[0])
    mean_v = (cache.V[0, :T].sum(0) + v_own.reshape(shape.n_kv_heads, shape.head_dim)) / (T + 1)
    att = np.repeat(mean_v, shape.n_heads // shape.n_kv_heads, axis=0).reshape(-1)
    np.testing.assert_allclose(out, h + _as64(m["layers"][0]["wo"]).numpy() @ att, rtol=1e-12, atol=1e-13)


def test_rope_scores_depend_on_relative_position_only():
    """Shifting every position by the same offset leaves the layer output unchanged when the cached keys are
    the layer's own rotated keys for the shifted positions (rotary embedding encodes relative offsets)."""
    name = "tiny-f32"
    om = oracle_model(name)
    shape = om.shape
    rows = si.gen_states(shape, 11, 4).numpy().astype(np.float64)
    outs = []
    for shift in (0, 5):
        cache = oc.KVCache(shape, 16)
        for t in range(4):
            out, k, v = om.layer(3, rows[t], t + shift, t, cache.K[3, shift:], cache.V[3, shift:])
            cache.K[3, shift + t] = k.reshape(shape.n_kv_heads, shape.head_dim)
            cache.V[3, shift + t] = v.reshape(shape.n_kv_heads, shape.head_dim)
        outs.append(out)
    np.testing.assert_allclose(outs[0], outs[1], rtol=1e-11, atol=1e-13)


def test_cosine_closed_forms():
    a = np.array([3.0, 0.0, 4.0])
    assert oc.cosine(a, a) == pytest.approx(1.0, abs=1e-15)
    assert oc.cosine(a, -2 * a) == pytest.approx(-1.0, abs=1e-15)
    assert oc.cosine(a, np.array([0.0, 7.0, 0.0])) == 0.0
    assert oc.cosine(a, np.array([1.0, 0.0, 0.0])) == pytest.approx(0.6, abs=1e-15)
    assert oc.cosine(np.zeros(3), a) == 0.0  # zero vector: x / max(|x|, 1e-12) stays zero


def test_draft_with_empty_mask_is_the_full_model_bit_for_bit():
    name = "tiny-f32"
    om = oracle_model(name)
    shape = om.shape
    toks = prompt(shape, 6)
    c1, c2 = oc.KVCache(shape, 8), oc.KVCache(shape, 8)
    for t, tok in enumerate(toks):
        _, l1 = om.token(tok, t, c1)
        _, l2 = om.token(tok, t, c2, skip=np.zeros(shape.n_layers, dtype=np.uint8))
        assert np.array_equal(l1, l2)
    assert np.array_equal(c1.K, c2.K) and np.array_equal(c1.V, c2.V)


def test_skipped_layer_writes_no_kv_and_passes_state_through():
    name = "tiny-f32"
    om = oracle_model(name)
    shape = om.shape
    skip = np.zeros(shape.n_layers, dtype=np.uint8)
    skip[[1, 4]] = 1
    cache = oc.KVCache(shape, 4)
    st, _ = om.token(17, 0, cache, skip=skip, want_states=True)
    assert np.array_equal(st[1], st[2]) and np.array_equal(st[4], st[5])
    assert not cache.K[1].any() and not cache.V[4].any() and cache.K[0, 0].any() and cache.K[2, 0].any()
