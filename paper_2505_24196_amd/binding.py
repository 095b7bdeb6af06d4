"""ctypes binding of libclasp_hip.so (the C ABI of include/clasp.h). Argument marshalling only.

PyTorch supplies device memory (tensors) and streams; every step of the hot path runs in the library's HIP kernels.
There is no CPU or eager fallback: if the library is missing or no GPU is present the calls raise.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libclasp_hip.so")

CLASP_F32, CLASP_BF16 = 0, 1
EXPORTS = ("clasp_strerror", "clasp_packed_bytes", "clasp_pack_matrix", "clasp_pack_gate_up", "clasp_workspace_bytes",
           "clasp_kv_cache_bytes", "clasp_create", "clasp_destroy", "clasp_verify_forward", "clasp_dp_select",
           "clasp_draft_step", "clasp_sample_token", "clasp_draft_sample", "clasp_spec_accept", "clasp_kv_load",
           "clasp_kv_read", "clasp_prefill_workspace_bytes", "clasp_prefill", "clasp_dp_select_window", "clasp_skip_cosine",
           "clasp_kernel_timer_begin", "clasp_kernel_timer_end", "clasp_prefill_static", "clasp_static_scratch_bytes")

KERNEL_KINDS = {"qkv": 0, "attention": 1, "o_proj": 2, "gate_up": 3, "down": 4, "lm_head": 5}


class ClaspError(RuntimeError):
    pass


class Config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("vocab", C.c_int32), ("max_seq", C.c_int32),
                ("max_rows", C.c_int32), ("dtype", C.c_int32), ("rms_eps", C.c_float), ("rope_base", C.c_float)]


class Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("attn_norm", C.POINTER(C.c_void_p)), ("mlp_norm", C.POINTER(C.c_void_p)),
                ("wq", C.POINTER(C.c_void_p)), ("wk", C.POINTER(C.c_void_p)), ("wv", C.POINTER(C.c_void_p)),
                ("wo", C.POINTER(C.c_void_p)), ("w_gate_up", C.POINTER(C.c_void_p)), ("w_down", C.POINTER(C.c_void_p))]


_lib = None


def lib():
    """Loads the built library (build it first: python -m paper_2505_24196_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ClaspError(f"{LIB_PATH} is missing: build the HIP library first (python -m paper_2505_24196_amd.build)")
        l = C.CDLL(LIB_PATH)
        vp, i32, sz = C.c_void_p, C.c_int, C.c_size_t
        l.clasp_strerror.restype = C.c_char_p
        l.clasp_strerror.argtypes = [i32]
        l.clasp_packed_bytes.restype = sz
        l.clasp_packed_bytes.argtypes = [i32, i32, i32]
        l.clasp_pack_matrix.argtypes = [vp, vp, i32, i32, i32, i32, vp]
        l.clasp_pack_gate_up.argtypes = [vp, vp, vp, i32, i32, i32, vp]
        l.clasp_workspace_bytes.restype = sz
        l.clasp_workspace_bytes.argtypes = [C.POINTER(Config)]
        l.clasp_kv_cache_bytes.restype = sz
        l.clasp_kv_cache_bytes.argtypes = [C.POINTER(Config)]
        l.clasp_create.argtypes = [C.POINTER(Config), C.POINTER(Weights), vp, sz, vp, vp, C.POINTER(vp)]
        l.clasp_destroy.argtypes = [vp]
        l.clasp_verify_forward.argtypes = [vp, vp, i32, i32, vp, vp, vp, vp, vp]
        l.clasp_dp_select.argtypes = [vp, vp, sz, i32, i32, vp, vp, vp, vp, vp]
        l.clasp_dp_select_window.argtypes = [vp, vp, sz, i32, i32, i32, i32, vp, vp, vp, vp, vp]
        l.clasp_skip_cosine.argtypes = [vp, vp, i32, vp, i32, vp, vp, vp]
        l.clasp_draft_step.argtypes = [vp, vp, vp, i32, vp, vp, vp]
        l.clasp_sample_token.argtypes = [vp, vp, C.c_float, vp, vp, vp]
        l.clasp_draft_sample.argtypes = [vp, vp, vp, i32, C.c_float, vp, vp, vp, vp]
        l.clasp_spec_accept.argtypes = [vp, vp, vp, sz, vp, i32, C.c_float, vp, vp, vp, vp, vp]
        l.clasp_kv_load.argtypes = [vp, i32, vp, vp, i32, vp]
        l.clasp_kv_read.argtypes = [vp, i32, i32, i32, vp, vp, vp]
        l.clasp_prefill_workspace_bytes.restype = sz
        l.clasp_prefill_workspace_bytes.argtypes = [C.POINTER(Config), i32]
        l.clasp_prefill.argtypes = [vp, vp, i32, i32, i32, vp, sz, vp]
        l.clasp_prefill_static.argtypes = [vp, vp, i32, i32, i32, vp]
        l.clasp_static_scratch_bytes.restype = sz
        l.clasp_static_scratch_bytes.argtypes = []
        l.clasp_kernel_timer_begin.argtypes = [vp, i32, i32, i32]
        l.clasp_kernel_timer_end.argtypes = [vp, C.POINTER(C.c_float), C.POINTER(C.c_int)]
        _lib = l
    return _lib


def _check(rc: int, what: str):
    if rc != 0:
        raise ClaspError(f"{what}: {lib().clasp_strerror(rc).decode()} ({rc})")


def _ptr(t: Optional[torch.Tensor], dtype=None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ClaspError("expected a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ClaspError(f"expected dtype {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dtype_code(dtype: str) -> int:
    return CLASP_F32 if dtype == "f32" else CLASP_BF16


def clasp_pack_matrix(src: torch.Tensor, dtype: str, rope_head_dim: int = 0) -> torch.Tensor:
    """Returns the packed copy of a row-major [rows][cols] device matrix (see clasp_pack_matrix in clasp.h);
    rope_head_dim = head_dim for wq and wk, 0 otherwise."""
    rows, cols = src.shape
    code = _dtype_code(dtype)
    want = torch.float32 if code == CLASP_F32 else torch.bfloat16
    if lib().clasp_packed_bytes(rows, cols, code) == 0:
        raise ClaspError(f"matrix {rows}x{cols} cannot be packed for dtype {dtype}")
    dst = torch.empty_like(src)
    _check(lib().clasp_pack_matrix(_ptr(src, want), _ptr(dst), rows, cols, code, rope_head_dim, _stream()),
           "clasp_pack_matrix")
    return dst


def clasp_pack_gate_up(gate: torch.Tensor, up: torch.Tensor, dtype: str) -> torch.Tensor:
    """Returns the single packed [2*d_ffn][d_model] matrix of the two MLP input projections (clasp_pack_gate_up)."""
    f, d = gate.shape
    code = _dtype_code(dtype)
    want = torch.float32 if code == CLASP_F32 else torch.bfloat16
    if up.shape != gate.shape or lib().clasp_packed_bytes(f, d, code) == 0:
        raise ClaspError(f"gate/up {tuple(gate.shape)} cannot be packed for dtype {dtype}")
    dst = torch.empty(2 * f, d, dtype=gate.dtype, device=gate.device)
    _check(lib().clasp_pack_gate_up(_ptr(gate, want), _ptr(up, want), _ptr(dst), f, d, code, _stream()),
           "clasp_pack_gate_up")
    return dst


_MATS = ("wq", "wk", "wv", "wo", "w_down")  # packed one by one; gate and up are packed together
_PACKED = ("wq", "wk", "wv", "wo", "w_gate_up", "w_down")


class Engine:
    """Owns the device buffers of one model + KV cache and exposes the calls of clasp.h with the same names."""

    def __init__(self, shape, max_seq: int, max_rows: int = 16, device: str = "cuda:0"):
        if not torch.cuda.is_available():
            raise ClaspError("no GPU: the CLaSp hot path has no CPU fallback")
        self.shape = shape
        self.device = torch.device(device)
        self.cfg = Config(shape.n_layers, shape.d_model, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn,
                          shape.vocab, max_seq, max_rows, _dtype_code(shape.dtype), shape.rms_eps, shape.rope_base)
        self.max_seq, self.max_rows = max_seq, max_rows
        if lib().clasp_workspace_bytes(C.byref(self.cfg)) == 0:
            raise ClaspError("configuration not supported by the kernels (see clasp_create in clasp.h)")
        self._layers: List[Dict[str, torch.Tensor]] = [None] * shape.n_layers
        self._head: Dict[str, torch.Tensor] = {}
        self._ctx = None

    # ---- weights ------------------------------------------------------------------------------------------------
    def set_head(self, embed: torch.Tensor, lm_head: torch.Tensor, final_norm: torch.Tensor):
        dev = self.device
        self._head = {"embed": embed.to(dev).contiguous(), "lm_head": clasp_pack_matrix(lm_head.to(dev).contiguous(), self.shape.dtype),
                      "final_norm": final_norm.to(dev, torch.float32).contiguous()}

    def set_layer(self, l: int, w: Dict[str, torch.Tensor]):
        """Packs one layer's row-major matrices (the row-major copies can be freed by the caller afterwards)."""
        dev = self.device
        out = {m: clasp_pack_matrix(w[m].to(dev).contiguous(), self.shape.dtype,
                                    self.shape.head_dim if m in ("wq", "wk") else 0) for m in _MATS}
        out["w_gate_up"] = clasp_pack_gate_up(w["w_gate"].to(dev).contiguous(), w["w_up"].to(dev).contiguous(),
                                              self.shape.dtype)
        out["attn_norm"] = w["attn_norm"].to(dev, torch.float32).contiguous()
        out["mlp_norm"] = w["mlp_norm"].to(dev, torch.float32).contiguous()
        self._layers[l] = out

    def load(self, model: Dict[str, object]):
        self.set_head(model["embed"], model["lm_head"], model["final_norm"])
        for l, w in enumerate(model["layers"]):
            self.set_layer(l, w)
        return self.create()

    def create(self):
        if self._ctx is not None:
            return self
        if not self._head or any(w is None for w in self._layers):
            raise ClaspError("weights incomplete")
        L = self.shape.n_layers
        self._arrays = {}
        wts = Weights(self._head["embed"].data_ptr(), self._head["lm_head"].data_ptr(), self._head["final_norm"].data_ptr())
        for name in ("attn_norm", "mlp_norm") + _PACKED:
            arr = (C.c_void_p * L)(*[self._layers[l][name].data_ptr() for l in range(L)])
            self._arrays[name] = arr
            setattr(wts, name, C.cast(arr, C.POINTER(C.c_void_p)))
        ws_bytes = lib().clasp_workspace_bytes(C.byref(self.cfg))
        kv_bytes = lib().clasp_kv_cache_bytes(C.byref(self.cfg))
        if ws_bytes == 0 or kv_bytes == 0:
            raise ClaspError("configuration not supported by the kernels")
        self.workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=self.device)
        self.k_cache = torch.empty(kv_bytes, dtype=torch.uint8, device=self.device)
        self.v_cache = torch.empty(kv_bytes, dtype=torch.uint8, device=self.device)
        ctx = C.c_void_p()
        torch.cuda.synchronize()
        _check(lib().clasp_create(C.byref(self.cfg), C.byref(wts), self.workspace.data_ptr(), ws_bytes,
                                  self.k_cache.data_ptr(), self.v_cache.data_ptr(), C.byref(ctx)), "clasp_create")
        self._ctx = ctx
        return self

    def close(self):
        if self._ctx is not None:
            torch.cuda.synchronize()
            lib().clasp_destroy(self._ctx)
            self._ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- the calls of clasp.h -------------------------------------------------------------------------------------
    def clasp_kv_load(self, layer: int, K: torch.Tensor, V: torch.Tensor):
        """K, V: fp32 [T][n_kv_heads][head_dim] (keys already rotated) -> cache positions 0..T-1 of `layer`."""
        K = K.to(self.device, torch.float32).contiguous()
        V = V.to(self.device, torch.float32).contiguous()
        _check(lib().clasp_kv_load(self._ctx, layer, _ptr(K), _ptr(V), K.shape[0], _stream()), "clasp_kv_load")

    def clasp_kv_read(self, layer: int, pos0: int, n_tokens: int):
        """Cache positions pos0..pos0+n_tokens-1 of `layer` as fp32 (K, V), each [n_tokens][n_kv_heads][head_dim]."""
        s = self.shape
        K = torch.empty(n_tokens, s.n_kv_heads, s.head_dim, dtype=torch.float32, device=self.device)
        V = torch.empty_like(K)
        _check(lib().clasp_kv_read(self._ctx, layer, pos0, n_tokens, _ptr(K), _ptr(V), _stream()), "clasp_kv_read")
        return K, V

    def clasp_prefill(self, tokens: torch.Tensor, pos0: int, chunk_rows: int = 4096):
        """tokens: device int32 [n] -> their keys/values in every layer's cache at pos0.. (bf16 models). The workspace
        for `chunk_rows` rows per pass is allocated on first use and kept."""
        need = lib().clasp_prefill_workspace_bytes(C.byref(self.cfg), chunk_rows)
        if need == 0:
            raise ClaspError("clasp_prefill: unsupported model dtype or chunk_rows (multiple of 128 in 128..8192)")
        ws = getattr(self, "_prefill_ws", None)
        if ws is None or ws.numel() < need:
            ws = self._prefill_ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        _check(lib().clasp_prefill(self._ctx, _ptr(tokens, torch.int32), tokens.numel(), pos0, chunk_rows, ws.data_ptr(),
                                   ws.numel(), _stream()), "clasp_prefill")

    def clasp_prefill_static(self, tokens: torch.Tensor, pos0: int, chunk_rows: int = 128):
        """clasp_prefill on the library's static scratch array: no workspace, no allocation."""
        _check(lib().clasp_prefill_static(self._ctx, _ptr(tokens, torch.int32), tokens.numel(), pos0, chunk_rows,
                                          _stream()), "clasp_prefill_static")

    def clasp_verify_forward(self, tokens: torch.Tensor, pos0: int, want_hidden: bool = False, want_logits: bool = False,
                             want_margin: bool = False):
        """tokens: device int32 [n]. Returns dict(argmax, hidden?, logits?, margin?) of device tensors."""
        n = tokens.numel()
        s = self.shape
        out = {"argmax": torch.empty(n, dtype=torch.int32, device=self.device)}
        if want_hidden:
            out["hidden"] = torch.empty(s.n_layers + 1, n, s.d_model, dtype=torch.float32, device=self.device)
        if want_logits:
            out["logits"] = torch.empty(n, s.vocab, dtype=torch.float32, device=self.device)
        if want_margin:
            out["margin"] = torch.empty(n, dtype=torch.float32, device=self.device)
        _check(lib().clasp_verify_forward(self._ctx, _ptr(tokens, torch.int32), n, pos0, _ptr(out.get("hidden")),
                                          _ptr(out["argmax"]), _ptr(out.get("margin")), _ptr(out.get("logits")),
                                          _stream()), "clasp_verify_forward")
        return out

    def clasp_dp_select(self, states: torch.Tensor, pos: int, M: int, want_tables: bool = False,
                        out: Optional[Dict[str, torch.Tensor]] = None, want_g_final: bool = False):
        """states: device fp32 [L+1][d] (may be a strided view along dim 0). Returns dict(mask, scores?, choice?,
        g_final?) of device tensors; `out` lets the caller reuse the output tensors of an earlier call."""
        s = self.shape
        L = s.n_layers
        if states.dtype != torch.float32 or not states.is_cuda or states.stride(1) != 1 or states.shape != (L + 1, s.d_model):
            raise ClaspError("states must be device fp32 [L+1][d] with unit inner stride")
        if out is None:
            out = {"mask": torch.empty(L, dtype=torch.uint8, device=self.device)}
            if want_tables:
                out["scores"] = torch.empty(L + 1, M + 1, 2, dtype=torch.float32, device=self.device)
                out["choice"] = torch.empty(L + 1, M + 1, dtype=torch.uint8, device=self.device)
                out["g_final"] = torch.empty(s.d_model, dtype=torch.float32, device=self.device)
            elif want_g_final:  # g(L, M) without the tables: the library then skips the cells that cannot reach (L, M)
                out["g_final"] = torch.empty(s.d_model, dtype=torch.float32, device=self.device)
        _check(lib().clasp_dp_select(self._ctx, states.data_ptr(), states.stride(0), pos, M, _ptr(out["mask"]),
                                     _ptr(out.get("scores")), _ptr(out.get("choice")), _ptr(out.get("g_final")),
                                     _stream()), "clasp_dp_select")
        return out

    def clasp_dp_select_window(self, states: torch.Tensor, pos: int, M: int, layer_lo: int, layer_hi: int,
                               want_tables: bool = False):
        """clasp_dp_select over the layers layer_lo..layer_hi-1 only. states: device fp32 [L+1][d]. Returns dict(mask
        [L], scores?, choice? ([layer_hi-layer_lo+1][M+1]), g_final?)."""
        s = self.shape
        L, Lw = s.n_layers, layer_hi - layer_lo
        if states.dtype != torch.float32 or not states.is_cuda or states.stride(1) != 1 or states.shape != (L + 1, s.d_model):
            raise ClaspError("states must be device fp32 [L+1][d] with unit inner stride")
        out = {"mask": torch.empty(L, dtype=torch.uint8, device=self.device)}
        if want_tables and Lw > 0:
            out["scores"] = torch.empty(Lw + 1, M + 1, 2, dtype=torch.float32, device=self.device)
            out["choice"] = torch.empty(Lw + 1, M + 1, dtype=torch.uint8, device=self.device)
            out["g_final"] = torch.empty(s.d_model, dtype=torch.float32, device=self.device)
        _check(lib().clasp_dp_select_window(self._ctx, states.data_ptr(), states.stride(0), pos, M, layer_lo, layer_hi,
                                            _ptr(out["mask"]), _ptr(out.get("scores")), _ptr(out.get("choice")),
                                            _ptr(out.get("g_final")), _stream()), "clasp_dp_select_window")
        return out

    def clasp_skip_cosine(self, masks, token: torch.Tensor, pos: int, target: torch.Tensor) -> torch.Tensor:
        """masks: host array-like [n][L] of 0/1 (1 = skip); token: device int32 [1]; target: device fp32 [d]. Returns
        the device fp32 [n] cosines of the masked forwards' last hidden states with target."""
        import numpy as np
        m = np.ascontiguousarray(np.asarray(masks, dtype=np.uint8))
        if m.ndim != 2 or m.shape[1] != self.shape.n_layers or m.shape[0] < 1:
            raise ClaspError("masks must be [n][n_layers]")
        out = torch.empty(m.shape[0], dtype=torch.float32, device=self.device)
        _check(lib().clasp_skip_cosine(self._ctx, m.ctypes.data, m.shape[0], _ptr(token, torch.int32), pos,
                                       _ptr(target, torch.float32), _ptr(out), _stream()), "clasp_skip_cosine")
        return out

    def clasp_draft_step(self, mask: Optional[Sequence[int]], token: torch.Tensor, pos: int,
                         next_token_out: torch.Tensor, top1_prob_out: Optional[torch.Tensor] = None):
        """mask: host sequence of L 0/1 (1 = skip) or None; token / next_token_out: device int32 [1] (views ok)."""
        mp = None
        if mask is not None:
            mb = (C.c_uint8 * self.shape.n_layers)(*[int(x) for x in mask])
            mp = C.cast(mb, C.c_void_p)
        _check(lib().clasp_draft_step(self._ctx, mp, token.data_ptr(), pos, next_token_out.data_ptr(),
                                      None if top1_prob_out is None else top1_prob_out.data_ptr(), _stream()),
               "clasp_draft_step")

    def _mask_ptr(self, mask):
        if mask is None:
            return None
        mb = (C.c_uint8 * self.shape.n_layers)(*[int(x) for x in mask])
        return C.cast(mb, C.c_void_p), mb

    def clasp_sample_token(self, logits: torch.Tensor, temperature: float, u: torch.Tensor, token_out: torch.Tensor):
        """logits device fp32 [vocab] (contiguous), u device fp32 [1], token_out device int32 [1]."""
        assert logits.dtype == torch.float32 and logits.is_contiguous() and logits.numel() == self.shape.vocab
        assert u.dtype == torch.float32 and token_out.dtype == torch.int32
        _check(lib().clasp_sample_token(self._ctx, logits.data_ptr(), float(temperature), u.data_ptr(),
                                        token_out.data_ptr(), _stream()), "clasp_sample_token")

    def clasp_draft_sample(self, mask: Optional[Sequence[int]], token: torch.Tensor, pos: int, temperature: float,
                           u: torch.Tensor, logits_out: torch.Tensor, next_token_out: torch.Tensor):
        """As clasp_draft_step, drawing the next token with u (device fp32 [1]); logits_out device fp32 [vocab]."""
        assert logits_out.dtype == torch.float32 and logits_out.is_contiguous() and logits_out.numel() == self.shape.vocab
        assert u.dtype == torch.float32 and next_token_out.dtype == torch.int32 and token.dtype == torch.int32
        mp = self._mask_ptr(mask)
        _check(lib().clasp_draft_sample(self._ctx, None if mp is None else mp[0], token.data_ptr(), pos,
                                        float(temperature), u.data_ptr(), logits_out.data_ptr(),
                                        next_token_out.data_ptr(), _stream()), "clasp_draft_sample")

    def clasp_spec_accept(self, p_logits: torch.Tensor, q_logits: torch.Tensor, tokens: torch.Tensor, n_draft: int,
                          temperature: float, u_accept: torch.Tensor, u_final: torch.Tensor,
                          n_accepted_out: torch.Tensor, next_token_out: torch.Tensor):
        """p_logits [>= n_draft+1][vocab], q_logits [>= n_draft][vocab] device fp32 with unit inner stride;
        tokens device int32 [n_draft+1]; u_accept device fp32 [n_draft]; u_final device fp32 [1]."""
        V = self.shape.vocab
        for t, rows in ((p_logits, n_draft + 1), (q_logits, n_draft)):
            assert t.dtype == torch.float32 and t.dim() == 2 and t.shape[1] == V and t.stride(1) == 1 and t.shape[0] >= rows
        assert p_logits.stride(0) == q_logits.stride(0)
        assert tokens.dtype == torch.int32 and tokens.numel() >= n_draft + 1 and u_accept.numel() >= n_draft
        assert u_accept.dtype == torch.float32 and u_final.dtype == torch.float32
        assert n_accepted_out.dtype == torch.int32 and next_token_out.dtype == torch.int32
        _check(lib().clasp_spec_accept(self._ctx, p_logits.data_ptr(), q_logits.data_ptr(), p_logits.stride(0),
                                       tokens.data_ptr(), n_draft, float(temperature), u_accept.data_ptr(),
                                       u_final.data_ptr(), n_accepted_out.data_ptr(), next_token_out.data_ptr(),
                                       _stream()), "clasp_spec_accept")

    # ---- measurement aid ------------------------------------------------------------------------------------------
    def kernel_timer_begin(self, kind: str, capacity: int = 1 << 16, every: int = 1):
        _check(lib().clasp_kernel_timer_begin(self._ctx, KERNEL_KINDS[kind], capacity, every),
               "clasp_kernel_timer_begin")

    def kernel_timer_end(self):
        """Returns (summed elapsed ms, launches timed) of the kernel kind chosen at begin."""
        ms, n = C.c_float(), C.c_int()
        _check(lib().clasp_kernel_timer_end(self._ctx, C.byref(ms), C.byref(n)), "clasp_kernel_timer_end")
        return float(ms.value), int(n.value)
