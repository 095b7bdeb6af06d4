"""Seeded synthetic inputs for the CLaSp hot path: model shapes, random-init weights, token ids, KV contents.

This module serves BOTH the CPU oracle and the HIP library and therefore holds none of the method's
arithmetic: it only draws numbers. Every value is a pure function of (seed, tensor id, element index) through a
counter-based hash (splitmix64 finaliser) followed by Box-Muller, so any tensor can be regenerated on demand,
on the CPU or on the GPU, without touching disk. The paper evaluates trained LLaMA checkpoints on Spec-Bench
(Experiments, "Model and Testbed" / "Datasets"); neither is available, so random-init LLaMA-shaped models
(matrices ~ N(0, 0.02^2), RMSNorm gains = 1) and uniform-random token ids stand in for them.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Optional

import numpy as np
import torch


@dataclasses.dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    dtype: str  # "f32" or "bf16"
    rms_eps: float = 1e-5
    rope_base: float = 10000.0

    @property
    def q_dim(self) -> int:
        return self.n_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    def layer_weight_elems(self) -> int:
        d, f = self.d_model, self.d_ffn
        return d * (self.q_dim + 2 * self.kv_dim) + self.q_dim * d + 3 * d * f

    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2


# The benchmark configurations (tiny fp32 case, LLaMA-3-8B shape, LLaMA-3-70B shape) plus small bf16 shapes
# that a CPU oracle finishes in seconds and that still span several MFMA tiles with ragged tails.
TINY_F32 = ModelShape("tiny-f32", 8, 256, 4, 4, 64, 688, 1024, "f32", 1e-5, 10000.0)
SMALL_BF16 = ModelShape("small-bf16", 6, 512, 8, 2, 64, 1408, 2064, "bf16", 1e-5, 500000.0)
SMALL_BF16_HD128 = ModelShape("small-bf16-hd128", 4, 1024, 8, 2, 128, 2816, 4112, "bf16", 1e-5, 500000.0)
SMALL_BF16_DEEP = ModelShape("small-bf16-deep", 24, 256, 4, 2, 64, 512, 1024, "bf16", 1e-5, 500000.0)
SMALL_BF16_WIDE_FFN = ModelShape("small-bf16-wide-ffn", 2, 512, 8, 2, 64, 8192, 2064, "bf16", 1e-5, 500000.0)
SMALL_BF16_MANY_HEADS = ModelShape("small-bf16-many-heads", 2, 512, 32, 32, 64, 1408, 2064, "bf16", 1e-5, 500000.0)
LLAMA3_8B = ModelShape("llama3-8b-shape", 32, 4096, 32, 8, 128, 14336, 128256, "bf16", 1e-5, 500000.0)
LLAMA3_70B = ModelShape("llama3-70b-shape", 80, 8192, 64, 8, 128, 28672, 128256, "bf16", 1e-5, 500000.0)

SHAPES = {s.name: s for s in (TINY_F32, SMALL_BF16, SMALL_BF16_HD128, SMALL_BF16_DEEP, SMALL_BF16_WIDE_FFN,
                              SMALL_BF16_MANY_HEADS, LLAMA3_8B, LLAMA3_70B)}

_MASK64 = (1 << 64) - 1


def _i64(x: int) -> int:
    """Two's-complement view of an unsigned 64-bit constant, as torch int64 needs it."""
    x &= _MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


_GOLDEN = _i64(0x9E3779B97F4A7C15)
_MUL1 = _i64(0xBF58476D1CE4E5B9)
_MUL2 = _i64(0x94D049BB133111EB)


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right of int64 lanes."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _splitmix64(x: torch.Tensor) -> torch.Tensor:
    z = x + _GOLDEN
    z = (z ^ _lsr(z, 30)) * _MUL1
    z = (z ^ _lsr(z, 27)) * _MUL2
    return z ^ _lsr(z, 31)


def _stream_key(seed: int, tensor_id: int) -> int:
    """One 64-bit key per (seed, tensor), itself a splitmix64 of the pair (python ints, exact)."""
    z = (seed * 0x9E3779B97F4A7C15 + tensor_id * 0xD1B54A32D192ED03 + 0x2545F4914F6CDD1D) & _MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
    return _i64(z ^ (z >> 31))


def hash_bits(seed: int, tensor_id: int, start: int, count: int, device="cpu") -> torch.Tensor:
    """int64 hashes of element indices start..start+count-1 of stream (seed, tensor_id)."""
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    return _splitmix64(idx * _GOLDEN + _stream_key(seed, tensor_id))


def hash_normal(seed: int, tensor_id: int, count: int, device="cpu", chunk: int = 1 << 25) -> torch.Tensor:
    """Standard normals (float32) by Box-Muller over two 24-bit uniforms cut from each element's hash."""
    out = torch.empty(count, dtype=torch.float32, device=device)
    for s in range(0, count, chunk):
        c = min(chunk, count - s)
        h = hash_bits(seed, tensor_id, s, c, device)
        u1 = (_lsr(h, 40).to(torch.float32) + 1.0) * (1.0 / 16777216.0)  # (0, 1]
        u2 = ((h >> 16) & 0xFFFFFF).to(torch.float32) * (1.0 / 16777216.0)  # [0, 1)
        out[s:s + c] = torch.sqrt(-2.0 * torch.log(u1)) * torch.cos(6.283185307179586 * u2)
    return out


def gen_matrix(seed: int, tensor_id: int, rows: int, cols: int, std: float, dtype: str, device="cpu") -> torch.Tensor:
    """[rows][cols] matrix ~ N(0, std^2), rounded to the model dtype (round-to-nearest-even for bf16)."""
    z = hash_normal(seed, tensor_id, rows * cols, device).mul_(std).view(rows, cols)
    return z if dtype == "f32" else z.to(torch.bfloat16)


def gen_tokens(seed: int, count: int, vocab: int, stream: int = 0) -> torch.Tensor:
    """Uniform-random token ids in [0, vocab), int32, on the CPU."""
    h = hash_bits(seed, 1 << 20 | stream, 0, count)
    return (_lsr(h, 11) % vocab).to(torch.int32)


def gen_uniform(seed: int, count: int, stream: int = 0) -> torch.Tensor:
    """Uniform numbers k / 2^24, k in [0, 2^24), float32 (exactly representable), on the CPU. These are the random
    draws of stochastic decoding, handed to both the oracle and the device as inputs."""
    h = hash_bits(seed, 2 << 20 | stream, 0, count)
    return (_lsr(h, 40).to(torch.float64) / float(1 << 24)).to(torch.float32)


# tensor ids inside a model's stream
_EMBED, _LM_HEAD, _LAYER0, _PER_LAYER = 0, 1, 16, 8
_MATS = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")


def matrix_dims(shape: ModelShape, name: str):
    d, f = shape.d_model, shape.d_ffn
    return {"wq": (shape.q_dim, d), "wk": (shape.kv_dim, d), "wv": (shape.kv_dim, d), "wo": (d, shape.q_dim),
            "w_gate": (f, d), "w_up": (f, d), "w_down": (d, f), "embed": (shape.vocab, d),
            "lm_head": (shape.vocab, d)}[name]


def gen_layer(shape: ModelShape, seed: int, layer: int, device="cpu", resid_scale: float = 1.0,
              std: float = 0.02) -> Dict[str, torch.Tensor]:
    """Weights of one decoder layer, every matrix row-major [out_features][in_features].

    resid_scale multiplies the std of the two matrices that write into the residual stream (wo, w_down): 1.0 is
    the plain N(0, 0.02^2) init; a small value gives the "slow-drift" variant whose hidden states change little
    from layer to layer, the regime the paper's method relies on (Sec. 3.5).
    """
    out: Dict[str, torch.Tensor] = {}
    for k, name in enumerate(_MATS):
        rows, cols = matrix_dims(shape, name)
        s = std * (resid_scale if name in ("wo", "w_down") else 1.0)
        out[name] = gen_matrix(seed, _LAYER0 + layer * _PER_LAYER + k, rows, cols, s, shape.dtype, device)
    out["attn_norm"] = torch.ones(shape.d_model, dtype=torch.float32, device=device)
    out["mlp_norm"] = torch.ones(shape.d_model, dtype=torch.float32, device=device)
    return out


def gen_head(shape: ModelShape, seed: int, device="cpu", std: float = 0.02) -> Dict[str, torch.Tensor]:
    """Embedding table, untied lm_head and the final norm gains."""
    return {"embed": gen_matrix(seed, _EMBED, shape.vocab, shape.d_model, std, shape.dtype, device),
            "lm_head": gen_matrix(seed, _LM_HEAD, shape.vocab, shape.d_model, std, shape.dtype, device),
            "final_norm": torch.ones(shape.d_model, dtype=torch.float32, device=device)}


def gen_model(shape: ModelShape, seed: int, device="cpu", resid_scale: float = 1.0) -> Dict[str, object]:
    """{'embed','lm_head','final_norm', 'layers': [per-layer dicts]} of torch tensors on `device`."""
    m: Dict[str, object] = dict(gen_head(shape, seed, device))
    m["layers"] = [gen_layer(shape, seed, l, device, resid_scale) for l in range(shape.n_layers)]
    return m


def gen_kv(shape: ModelShape, seed: int, n_layers: int, n_tokens: int, device="cpu"):
    """Synthetic cache contents standing in for a prefill the oracle cannot afford at large shapes.

    Returns (K, V), each float32 [n_layers][n_tokens][n_kv_heads][head_dim] ~ N(0,1), already rounded to the
    model dtype's grid. For bf16 models the device caches fp16: a bf16-grid value of magnitude >= 2^-14 is an fp16
    number too, so the device cache and the fp64 oracle read identical values there (smaller ones move by <= 2^-25).
    """
    n = n_layers * n_tokens * shape.kv_dim
    outs = []
    for tid in (1 << 21, (1 << 21) + 1):
        z = hash_normal(seed, tid, n, device)
        if shape.dtype == "bf16":
            z = z.to(torch.bfloat16).to(torch.float32)
        outs.append(z.view(n_layers, n_tokens, shape.n_kv_heads, shape.head_dim))
    return outs[0], outs[1]


def gen_states(shape: ModelShape, seed: int, n_rows: int, device="cpu", stream: int = 0) -> torch.Tensor:
    """[n_rows][d_model] float32 ~ N(0,1): stand-in hidden states for kernel-level checks."""
    return hash_normal(seed, (1 << 22) + stream, n_rows * shape.d_model, device).view(n_rows, shape.d_model)


def to_numpy(t: torch.Tensor) -> np.ndarray:
    """CPU numpy view of a tensor; bf16 becomes its uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def model_to_numpy(model: Dict[str, object]) -> Dict[str, object]:
    out: Dict[str, object] = {k: to_numpy(v) for k, v in model.items() if k != "layers"}
    out["layers"] = [{k: to_numpy(v) for k, v in layer.items()} for layer in model["layers"]]
    return out
