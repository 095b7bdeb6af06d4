"""ctypes front end of the C oracle plus the greedy decode loops -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module. It never imports the
HIP package. Arithmetic lives in clasp_oracle.c; this file adds
  * prefill / plain greedy decoding with the full model (the lossless reference of the paper's abstract and
    "Performance Metrics": speculative decoding must not change the generated text),
  * the Draft -> Verify -> Layer-Optimization loop of Sec. 3.1 with greedy acceptance,
  * its stochastic form (Temperature = 1 setting of Sec. 4): inverse-CDF draws and the speculative-sampling
    acceptance rule, in fp64 numpy, with every uniform number passed in,
which are control flow around the C calls.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np

from . import build as _build

_LIB = None


class _Model(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("vocab", C.c_int32),
                ("wdtype", C.c_int32), ("rms_eps", C.c_double), ("rope_base", C.c_double),
                ("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("attn_norm", C.POINTER(C.c_void_p)), ("mlp_norm", C.POINTER(C.c_void_p)),
                ("wq", C.POINTER(C.c_void_p)), ("wk", C.POINTER(C.c_void_p)), ("wv", C.POINTER(C.c_void_p)),
                ("wo", C.POINTER(C.c_void_p)), ("w_gate", C.POINTER(C.c_void_p)),
                ("w_up", C.POINTER(C.c_void_p)), ("w_down", C.POINTER(C.c_void_p))]


def _lib():
    global _LIB
    if _LIB is None:
        path = _build.build()
        lib = C.CDLL(path)
        dp = C.POINTER(C.c_double)
        lib.clasp_oracle_layer.argtypes = [C.POINTER(_Model), C.c_int, dp, C.c_int, C.c_int, dp, dp, dp, dp, dp]
        lib.clasp_oracle_layer.restype = C.c_int
        lib.clasp_oracle_token.argtypes = [C.POINTER(_Model), C.c_int, C.c_int, C.c_void_p, dp, dp, C.c_int, dp, dp]
        lib.clasp_oracle_token.restype = C.c_int
        lib.clasp_oracle_cosine.argtypes = [dp, dp, C.c_int]
        lib.clasp_oracle_cosine.restype = C.c_double
        lib.clasp_oracle_dp.argtypes = [C.POINTER(_Model), dp, C.c_int, dp, dp, C.c_int, C.c_int, C.c_void_p,
                                        dp, dp, C.c_void_p, dp, C.c_void_p]
        lib.clasp_oracle_dp.restype = C.c_int
        lib.clasp_oracle_num_threads.restype = C.c_int
        _LIB = lib
    return _LIB


def _dptr(a: Optional[np.ndarray]):
    if a is None:
        return None
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.POINTER(C.c_double))


def num_threads() -> int:
    return int(_lib().clasp_oracle_num_threads())


def cosine(a: np.ndarray, b: np.ndarray) -> float:
    a = np.ascontiguousarray(a, dtype=np.float64)
    b = np.ascontiguousarray(b, dtype=np.float64)
    return float(_lib().clasp_oracle_cosine(_dptr(a), _dptr(b), a.size))


class KVCache:
    """The full model's keys (rotated) and values: float64 [n_layers][t_max][n_kv_heads][head_dim]."""

    def window(self, lo: int, hi: int) -> "KVCache":
        """View of the layers lo..hi-1 (shares memory), for OracleModel.window."""
        v = KVCache.__new__(KVCache)
        v.K, v.V, v.t_max = self.K[lo:hi], self.V[lo:hi], self.t_max
        return v

    def __init__(self, shape, t_max: int):
        dims = (shape.n_layers, t_max, shape.n_kv_heads, shape.head_dim)
        self.K = np.zeros(dims, dtype=np.float64)
        self.V = np.zeros(dims, dtype=np.float64)
        self.t_max = t_max

    def load(self, K: np.ndarray, V: np.ndarray, layers: Optional[Sequence[int]] = None):
        """Fill rows 0..T-1 from arrays [n][T][n_kv][hd] (synthetic contents or another cache)."""
        layers = range(K.shape[0]) if layers is None else layers
        for src, l in enumerate(layers):
            self.K[l, :K.shape[1]] = K[src]
            self.V[l, :V.shape[1]] = V[src]


class OracleModel:
    """Holds row-major numpy weights (float32, or uint16 bf16 bit patterns) and calls the C oracle."""

    def __init__(self, shape, weights: Dict[str, object]):
        self.shape = shape
        self.w = weights  # keep the arrays alive
        L = shape.n_layers
        layers = weights["layers"]
        assert len(layers) == L
        wd = 0 if shape.dtype == "f32" else 1
        want = np.float32 if wd == 0 else np.uint16

        def p(a: np.ndarray, dt):
            assert a.dtype == dt and a.flags["C_CONTIGUOUS"], (a.dtype, dt)
            return a.ctypes.data

        def arr(name: str, dt):
            return (C.c_void_p * L)(*[p(layers[l][name], dt) for l in range(L)])

        self._arrays = {n: arr(n, want) for n in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")}
        self._arrays["attn_norm"] = arr("attn_norm", np.float32)
        self._arrays["mlp_norm"] = arr("mlp_norm", np.float32)
        m = _Model(shape.n_layers, shape.d_model, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn,
                   shape.vocab, wd, shape.rms_eps, shape.rope_base,
                   p(weights["embed"], want), p(weights["lm_head"], want), p(weights["final_norm"], np.float32))
        for n, a in self._arrays.items():
            setattr(m, n, C.cast(a, C.POINTER(C.c_void_p)))
        self._m = m

    # ---- single calls -------------------------------------------------------------------------------------
    def layer(self, l: int, h: np.ndarray, pos: int, n_prefix: int, Kl: np.ndarray, Vl: np.ndarray):
        """f_l on one row: returns (out[d], k_new[kv_dim], v_new[kv_dim])."""
        s = self.shape
        h = np.ascontiguousarray(h, dtype=np.float64)
        out = np.empty(s.d_model)
        kn = np.empty(s.kv_dim)
        vn = np.empty(s.kv_dim)
        rc = _lib().clasp_oracle_layer(C.byref(self._m), l, _dptr(h), pos, n_prefix, _dptr(Kl), _dptr(Vl),
                                       _dptr(out), _dptr(kn), _dptr(vn))
        if rc:
            raise ValueError("clasp_oracle_layer: bad argument")
        return out, kn, vn

    def token(self, token: int, pos: int, cache: KVCache, skip: Optional[np.ndarray] = None,
              want_states: bool = False, want_logits: bool = True):
        """One token through the (possibly layer-skipped) model; writes the cache row `pos`."""
        s = self.shape
        states = np.empty((s.n_layers + 1, s.d_model)) if want_states else None
        logits = np.empty(s.vocab) if want_logits else None
        sk = None
        if skip is not None:
            sk = np.ascontiguousarray(skip, dtype=np.uint8)
            assert sk.size == s.n_layers
        rc = _lib().clasp_oracle_token(C.byref(self._m), int(token), int(pos),
                                       None if sk is None else sk.ctypes.data, _dptr(cache.K), _dptr(cache.V),
                                       cache.t_max, _dptr(states), _dptr(logits))
        if rc:
            raise ValueError("clasp_oracle_token: bad argument")
        return states, logits

    def dp(self, X: np.ndarray, pos: int, cache: KVCache, M: int, override: Optional[np.ndarray] = None):
        """Algorithm 1 for the token at `pos` with stored states X[(L+1)][d]."""
        s = self.shape
        L = s.n_layers
        if not (0 <= M <= L):
            raise ValueError("M out of range")
        X = np.ascontiguousarray(X, dtype=np.float64)
        assert X.shape == (L + 1, s.d_model)
        sc = np.empty((L + 1, M + 1))
        ss = np.empty((L + 1, M + 1))
        ch = np.empty((L + 1, M + 1), dtype=np.uint8)
        gf = np.empty(s.d_model)
        mask = np.empty(L, dtype=np.uint8)
        ov = None
        if override is not None:
            ov = np.ascontiguousarray(override, dtype=np.int8)
            assert ov.shape == (L + 1, M + 1)
        rc = _lib().clasp_oracle_dp(C.byref(self._m), _dptr(X), int(pos), _dptr(cache.K), _dptr(cache.V),
                                    cache.t_max, int(M), None if ov is None else ov.ctypes.data, _dptr(sc),
                                    _dptr(ss), ch.ctypes.data, _dptr(gf), mask.ctypes.data)
        if rc:
            raise ValueError("clasp_oracle_dp: bad argument")
        return {"sigma_c": sc, "sigma_s": ss, "choice": ch, "g_final": gf, "mask": mask}

    # ---- the search restricted to a window of layers, and the objective of a given skip set (Sec. 3.5) ------------
    def window(self, lo: int, hi: int) -> "OracleModel":
        """The layers lo..hi-1 as a model of their own (same weights): its dp() is Algorithm 1 with every layer outside
        the window kept, on states X[lo..hi] and the cache of those layers (cache_window)."""
        if not (0 <= lo < hi <= self.shape.n_layers):
            raise ValueError("window out of range")
        import dataclasses
        w = dict(self.w)
        w["layers"] = self.w["layers"][lo:hi]
        return OracleModel(dataclasses.replace(self.shape, n_layers=hi - lo), w)

    def masked_state(self, x0: np.ndarray, pos: int, cache: KVCache, mask: Sequence[int]) -> np.ndarray:
        """x_0 through the layers a skip set keeps, each attending the cache rows 0..pos-1 of its layer plus its own
        key/value (the context of the candidates in Algorithm 1): the state the draft model would hand to the head."""
        h = np.array(x0, dtype=np.float64)
        for l in range(self.shape.n_layers):
            if not mask[l]:
                h, _, _ = self.layer(l, h, pos, pos, cache.K[l], cache.V[l])
        return h

    def skip_cosine(self, x0: np.ndarray, pos: int, cache: KVCache, mask: Sequence[int], target: np.ndarray) -> float:
        """Eq. 1's objective for one skip set: cosine of masked_state with the full model's last hidden state."""
        return cosine(self.masked_state(x0, pos, cache, mask), np.asarray(target, dtype=np.float64))

    # ---- loops --------------------------------------------------------------------------------------------
    def prefill(self, tokens: Sequence[int], cache: KVCache, pos0: int = 0):
        """Full model over the prompt, one token at a time. Returns (states, logits) of the last token."""
        states = logits = None
        for t, tok in enumerate(tokens):
            last = t == len(tokens) - 1
            states, logits = self.token(tok, pos0 + t, cache, want_states=last, want_logits=last)
        return states, logits

    def greedy_decode(self, prompt: Sequence[int], n_gen: int, t_max: Optional[int] = None):
        """Plain greedy decoding with the full model. Returns (tokens, margins): top-1 minus top-2 logit."""
        t_max = t_max or len(prompt) + n_gen + 1
        cache = KVCache(self.shape, t_max)
        _, logits = self.prefill(prompt, cache)
        out, margins = [], []
        pos = len(prompt)
        while len(out) < n_gen:
            tok, mg = argmax_margin(logits)
            out.append(tok)
            margins.append(mg)
            if len(out) == n_gen:
                break
            _, logits = self.token(tok, pos, cache)
            pos += 1
        return out, margins

    def spec_decode(self, prompt: Sequence[int], n_gen: int, M: int, K: int, t_max: Optional[int] = None,
                    dp_interval: int = 1, det_threshold: Optional[float] = None):
        """Greedy self-speculative decoding (Sec. 3.1): draft K tokens with the layer-skipped model, verify them
        with the full model, accept the longest matching prefix plus the full model's next token, then re-run the
        layer optimisation on the last accepted token's stored states. dp_interval > 1 re-optimises only every
        that many verify steps (Sec. 3.7). det_threshold (Sec. 5.3.3): drafting stops after the first draft token
        whose softmax probability under the draft model is below the threshold (that token is still proposed), so a
        round holds 1..K drafts. Returns a dict with the tokens and a per-round trace."""
        s = self.shape
        t_max = t_max or len(prompt) + n_gen + K + 2
        cache = KVCache(s, t_max)
        states, logits = self.prefill(prompt, cache)
        pending, _ = argmax_margin(logits)
        out = [pending]
        pos = len(prompt)  # position the pending token will occupy
        dp = self.dp(states, pos - 1, cache, M)  # prefill counts as verification 0
        mask = dp["mask"]
        rounds = []
        n_verify = 0
        while len(out) < n_gen:
            drafts, conf, tok = [], [], pending
            for k in range(K):
                _, lg = self.token(tok, pos + k, cache, skip=mask)
                tok, _ = argmax_margin(lg)
                drafts.append(tok)
                conf.append(top1_prob(lg))
                if det_threshold is not None and conf[-1] < det_threshold:
                    break
            n_draft = len(drafts)
            rows = [pending] + drafts
            v, v_states, v_margin = [], [], []
            for r, tk in enumerate(rows):  # the verify pass: full model, causal over the K+1 rows
                st, lg = self.token(tk, pos + r, cache, want_states=True)
                a_tok, a_mg = argmax_margin(lg)
                v.append(a_tok)
                v_margin.append(a_mg)
                v_states.append(st)
            a = 0
            while a < n_draft and drafts[a] == v[a]:
                a += 1
            out.extend(drafts[:a] + [v[a]])
            n_verify += 1
            rounds.append({"pos": pos, "mask": mask.copy(), "drafts": drafts, "verify": v, "accepted": a,
                           "verify_margin": v_margin, "dp": dp, "draft_conf": conf})
            if n_verify % dp_interval == 0:
                dp = self.dp(v_states[a], pos + a, cache, M)
                mask = dp["mask"]
            pending = v[a]
            pos += a + 1
        return {"tokens": out[:n_gen], "rounds": rounds}

    def spec_sample_decode(self, prompt: Sequence[int], n_gen: int, M: int, K: int, uniforms: Dict[str, np.ndarray],
                           temperature: float = 1.0, t_max: Optional[int] = None):
        """Stochastic self-speculative decoding: as spec_decode, but draft tokens are drawn from the layer-skipped
        model's softmax, verified with the speculative-sampling acceptance rule (spec_accept), and the layer
        optimisation runs on the last accepted row. uniforms: "first" [1], "draft" [rounds*K], "accept"
        [rounds*K], "final" [rounds] numbers in [0, 1), consumed by round r at indices r*K + k (draft, accept) and r
        (final), so that a device run with the same arrays makes the same draws."""
        s = self.shape
        t_max = t_max or len(prompt) + n_gen + K + 2
        cache = KVCache(s, t_max)
        states, logits = self.prefill(prompt, cache)
        pending, first_margin = sample_cdf(softmax_t(logits, temperature), uniforms["first"][0])
        out = [pending]
        pos = len(prompt)
        dp = self.dp(states, pos - 1, cache, M)
        mask = dp["mask"]
        rounds = []
        r = 0
        while len(out) < n_gen:
            drafts, q_logits, draft_margin, tok = [], [], [], pending
            for k in range(K):
                _, lg = self.token(tok, pos + k, cache, skip=mask)
                tok, mg = sample_cdf(softmax_t(lg, temperature), uniforms["draft"][r * K + k])
                drafts.append(tok)
                q_logits.append(lg)
                draft_margin.append(mg)
            rows = [pending] + drafts
            p_logits, v_states = [], []
            for i, tk in enumerate(rows):
                st, lg = self.token(tk, pos + i, cache, want_states=True)
                p_logits.append(lg)
                v_states.append(st)
            a, nxt, info = spec_accept(np.stack(p_logits), np.stack(q_logits), drafts,
                                       uniforms["accept"][r * K:(r + 1) * K], uniforms["final"][r], temperature)
            out.extend(drafts[:a] + [nxt])
            rounds.append({"pos": pos, "mask": mask.copy(), "drafts": drafts, "accepted": a, "next": nxt, "dp": dp,
                           "draft_margin": draft_margin, "ratio_margin": info["ratio_margin"],
                           "cdf_margin": info["cdf_margin"]})
            dp = self.dp(v_states[a], pos + a, cache, M)
            mask = dp["mask"]
            pending = nxt
            pos += a + 1
            r += 1
        return {"tokens": out[:n_gen], "rounds": rounds, "first_margin": first_margin}


def softmax_t(logits: np.ndarray, temperature: float = 1.0) -> np.ndarray:
    """softmax(logits / temperature) in fp64."""
    lg = np.asarray(logits, dtype=np.float64) / float(temperature)
    e = np.exp(lg - lg.max())
    return e / e.sum()


def sample_cdf(weights: np.ndarray, u: float):
    """Inverse-CDF draw from non-negative (not necessarily normalised) weights with one uniform u in [0, 1): the
    smallest index v whose running sum c_v = w_0 + .. + w_v exceeds u * c_last (the last index of positive weight if
    rounding leaves none). Also returns how far u * c_last is from the two ends of the chosen interval, as a
    fraction of c_last: a device result in lower precision may only differ when that distance is tiny."""
    w = np.asarray(weights, dtype=np.float64)
    c = np.cumsum(w)
    target = float(u) * c[-1]
    v = int(np.searchsorted(c, target, side="right"))
    if v >= w.size:
        v = int(np.nonzero(w > 0)[0][-1])
    lo = c[v - 1] if v > 0 else 0.0
    margin = min(target - lo, c[v] - target) / c[-1] if c[-1] > 0 else 0.0
    return v, float(margin)


def spec_accept(p_logits: np.ndarray, q_logits: np.ndarray, drafts: Sequence[int], u_accept: Sequence[float],
                u_final: float, temperature: float = 1.0):
    """Acceptance rule of speculative sampling (the lossless scheme the paper relies on in its Sec. 4.1 and its
    Temperature = 1 results, from the work it cites there): with p_i = softmax of the full model's logits for the
    token after row i and q_i the draft model's, draft x_i is kept when u_i * q_i(x_i) < p_i(x_i); at the first
    rejection the replacement token is drawn from max(0, p_i - q_i) renormalised; when every draft is kept the
    bonus token is drawn from p_n. p_logits [n+1][V], q_logits [n][V].
    Returns (accepted count a, next token, dict of decision margins)."""
    n = len(drafts)
    info = {"ratio_margin": [], "cdf_margin": None}
    a = n
    for i in range(n):
        p, q = softmax_t(p_logits[i], temperature), softmax_t(q_logits[i], temperature)
        x = int(drafts[i])
        lhs, rhs = float(u_accept[i]) * q[x], p[x]
        info["ratio_margin"].append(abs(lhs - rhs) / max(rhs, lhs, 1e-300))
        if not lhs < rhs:
            a = i
            break
    if a < n:
        p, q = softmax_t(p_logits[a], temperature), softmax_t(q_logits[a], temperature)
        w = np.maximum(p - q, 0.0)
        if w.sum() <= 0.0:
            w = p
    else:
        w = softmax_t(p_logits[n], temperature)
    tok, info["cdf_margin"] = sample_cdf(w, u_final)
    return a, tok, info


def top1_prob(logits: np.ndarray) -> float:
    """Largest softmax probability: 1 / sum_v exp(logit_v - max logit), in fp64."""
    lg = np.asarray(logits, dtype=np.float64)
    return float(1.0 / np.exp(lg - lg.max()).sum())


def argmax_margin(logits: np.ndarray):
    """(lowest index of the maximum, top-1 minus top-2 value)."""
    i = int(np.argmax(logits))
    rest = np.delete(logits, i)
    return i, float(logits[i] - rest.max()) if rest.size else float("inf")
