"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

This module holds no arithmetic of the method itself: it only draws random
numbers (numpy's Philox bit generator) and shapes them into model weights,
prompts, pending speculations and synthetic prefix KV, at the shapes of the
workloads the paper evaluates (a Llama-3.2-1B-shaped draft, a Llama-3.1-70B-shaped
target, K = 5 drafted tokens, batch 1 and 16; paper Sec. 4 "Setup" and
App. B "Experimental Design").  The paper's prompts come from four public
datasets and its weights are trained; here both are replaced by seeded random
content of the same shape.

Everything is returned as numpy arrays.  For bf16 workloads every value is
already rounded to a bf16-representable float32, so the oracle (which widens to
float64) and the HIP path (which narrows to bf16 bit patterns) multiply exactly
the same numbers.
"""
from __future__ import annotations

from dataclasses import dataclass, field, asdict
from typing import Dict, List, Optional

import numpy as np

__all__ = [
    "ModelShape", "RoundShape", "Workload", "WORKLOADS",
    "round_to_bf16", "bf16_bits", "make_weights", "make_prompt",
    "make_pending", "make_prefix_kv", "weight_names",
    "hashed_normal", "make_hashed_weights", "make_hashed_prefix_kv",
]


@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    dtype: str            # "f32" or "bf16": storage type of weights and KV
    rope_theta: float
    rms_eps: float = 1e-5
    tie_embeddings: bool = False

    @property
    def n_params(self) -> int:
        d, hq, hkv, D, f = self.d_model, self.n_q_heads, self.n_kv_heads, self.head_dim, self.d_ffn
        per_layer = d * (hq * D) + 2 * d * (hkv * D) + (hq * D) * d + 3 * d * f + 2 * d
        head = self.vocab * d * (1 if self.tie_embeddings else 2)
        return self.n_layers * per_layer + head + d


@dataclass(frozen=True)
class RoundShape:
    batch: int
    prefix: int           # P: tokens already in the trunk KV at the start of the round
    K: int                # speculative lookahead
    F: int                # uniform fan-out
    temperature: float    # 0 = greedy

    @property
    def rows(self) -> int:
        return self.batch * (self.K + 1) * self.F


@dataclass(frozen=True)
class Workload:
    name: str
    draft: ModelShape
    round: RoundShape
    target: Optional[ModelShape] = None
    seed: int = 0


TINY = ModelShape(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64, d_ffn=1024,
                  vocab=1024, dtype="f32", rope_theta=10000.0, tie_embeddings=False)
LLAMA_1B = ModelShape(n_layers=16, d_model=2048, n_q_heads=32, n_kv_heads=8, head_dim=64, d_ffn=8192,
                      vocab=128256, dtype="bf16", rope_theta=500000.0, tie_embeddings=True)
LLAMA_70B = ModelShape(n_layers=80, d_model=8192, n_q_heads=64, n_kv_heads=8, head_dim=128, d_ffn=28672,
                       vocab=128256, dtype="bf16", rope_theta=500000.0, tie_embeddings=False)

WORKLOADS: Dict[str, Workload] = {
    "tiny_f32": Workload("tiny_f32", TINY, RoundShape(1, 128, 4, 2, 0.0), target=TINY, seed=101),
    "1b_p1024_f4": Workload("1b_p1024_f4", LLAMA_1B, RoundShape(1, 1024, 5, 4, 0.0), seed=202),
    "1b_p8192_f8_t1": Workload("1b_p8192_f8_t1", LLAMA_1B, RoundShape(1, 8192, 5, 8, 1.0), seed=303),
    "1b_b16_p2048_f4": Workload("1b_b16_p2048_f4", LLAMA_1B, RoundShape(16, 2048, 5, 4, 0.0), seed=404),
    "70b_verify_1b_draft": Workload("70b_verify_1b_draft", LLAMA_1B, RoundShape(1, 4096, 5, 4, 1.0),
                                    target=LLAMA_70B, seed=505),
}


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Bit patterns (uint16) of float32 values that are already bf16-representable."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    if np.any(bits & np.uint32(0xFFFF)):
        raise ValueError("values are not bf16-representable")
    return (bits >> np.uint32(16)).astype(np.uint16)


def _rng(seed: int, *stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[(seed * 0x9E3779B1 + 0x55D0) & 0xFFFFFFFFFFFFFFFF,
                                                      sum((s + 1) * 1000003 ** (i + 1) for i, s in enumerate(stream))
                                                      & 0xFFFFFFFFFFFFFFFF]))


def weight_names(shape: ModelShape) -> List[str]:
    names = ["embed"]
    for l in range(shape.n_layers):
        names += [f"l{l}.{n}" for n in ("attn_norm", "wq", "wk", "wv", "wo", "mlp_norm", "w_gate", "w_up", "w_down")]
    names += ["final_norm"]
    if not shape.tie_embeddings:
        names += ["lm_head"]
    return names


def weight_shape(shape: ModelShape, name: str):
    d, hq, hkv, D, f, V = (shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                           shape.d_ffn, shape.vocab)
    leaf = name.split(".")[-1]
    return {
        "embed": (V, d), "lm_head": (V, d), "final_norm": (d,), "attn_norm": (d,), "mlp_norm": (d,),
        "wq": (hq * D, d), "wk": (hkv * D, d), "wv": (hkv * D, d), "wo": (d, hq * D),
        "w_gate": (f, d), "w_up": (f, d), "w_down": (d, f),
    }[leaf]


def make_weights(shape: ModelShape, seed: int, std: float = 0.02,
                 perturb_of: Optional[Dict[str, np.ndarray]] = None, perturb_std: float = 0.0
                 ) -> Dict[str, np.ndarray]:
    """Random-init weights: every matrix N(0, std), every RMSNorm gain 1.0.

    Matrices are stored as the linear layers apply them, [out_features][in_features].
    With `perturb_of`, returns that model plus N(0, perturb_std) noise (a draft
    that is close to, but not equal to, its target).
    """
    out: Dict[str, np.ndarray] = {}
    for idx, name in enumerate(weight_names(shape)):
        shp = weight_shape(shape, name)
        if name.endswith("norm"):
            w = np.ones(shp, dtype=np.float32)
        else:
            g = _rng(seed, 1, idx)
            if perturb_of is None:
                w = g.standard_normal(shp, dtype=np.float32) * np.float32(std)
            else:
                w = perturb_of[name] + g.standard_normal(shp, dtype=np.float32) * np.float32(perturb_std)
        if shape.dtype == "bf16":
            w = round_to_bf16(w)
        out[name] = w
    return out


def make_prompt(shape: ModelShape, batch: int, length: int, seed: int) -> np.ndarray:
    """Uniform-random token ids, int32 [batch][length]."""
    return _rng(seed, 2).integers(0, shape.vocab, size=(batch, length), dtype=np.int32)


def make_pending(shape: ModelShape, batch: int, K: int, seed: int) -> np.ndarray:
    """Uniform-random pending block {last verified token, s_1..s_K}, int32 [batch][K+1]."""
    return _rng(seed, 3).integers(0, shape.vocab, size=(batch, K + 1), dtype=np.int32)


def make_prefix_kv(shape: ModelShape, batch: int, prefix: int, seed: int):
    """Synthetic trunk KV standing in for a prefill that is not on the measured path.

    Returns (k, v), float32 [n_layers][batch][prefix][n_kv_heads][head_dim], unit-variance
    normal, rounded to bf16 for bf16 models.
    """
    shp = (shape.n_layers, batch, prefix, shape.n_kv_heads, shape.head_dim)
    k = _rng(seed, 4).standard_normal(shp, dtype=np.float32)
    v = _rng(seed, 5).standard_normal(shp, dtype=np.float32)
    if shape.dtype == "bf16":
        k, v = round_to_bf16(k), round_to_bf16(v)
    return k, v


def make_logits(rows: int, vocab: int, seed: int, scale: float = 0.9, n_ties: int = 0) -> np.ndarray:
    """Random fp32 logit rows with the spread of a random-init LM head (sigma ~ 0.9).

    `n_ties` copies the row maximum onto that many extra random positions so that
    tie-breaking is exercised.
    """
    g = _rng(seed, 6)
    z = g.standard_normal((rows, vocab), dtype=np.float32) * np.float32(scale)
    for r in range(rows):
        if n_ties:
            pos = g.choice(vocab, size=n_ties, replace=False)
            z[r, pos] = z[r].max()
    return z


# --------------------------------------------------------------------------- hashed content (the device generates the same)
# A second family of synthetic inputs, defined by integer arithmetic alone so that the HIP library can generate the very
# same bits on the device (models too large for a host copy: the 70B-shaped target).  Element i of tensor t:
#   bits = mix64(mix64(seed + GOLD (t + 1)) + i)        mix64 = the SplitMix64 finaliser
#   S    = sum of the four 16-bit lanes of bits          (mean 131070, standard deviation sqrt(4 (65536^2 - 1) / 12))
#   x    = float32(S - 131070) * float32(std / sigma_S)  one exact conversion, one float32 multiplication
# then rounded to bf16 for bf16 tensors.  Tensor ids: 0 embedding, 1 LM head, 16 + 16 l + {0 wq, 1 wk, 2 wv, 3 wo,
# 4 w_gate, 5 w_up, 6 w_down} for layer l, (1 << 20) + 2 l + {0 keys, 1 values} for the synthetic prefix KV of layer l.

_GOLD = np.uint64(0x9E3779B97F4A7C15)
_SIGMA_S = float(np.sqrt(4.0 * (65536.0 ** 2 - 1.0) / 12.0))


def _mix64(x: np.ndarray) -> np.ndarray:
    x = np.asarray(x, dtype=np.uint64).copy()
    with np.errstate(over="ignore"):
        x ^= x >> np.uint64(30)
        x *= np.uint64(0xBF58476D1CE4E5B9)
        x ^= x >> np.uint64(27)
        x *= np.uint64(0x94D049BB133111EB)
        x ^= x >> np.uint64(31)
    return x


def hashed_normal(seed: int, tensor_id: int, index: np.ndarray, std: float, bf16: bool) -> np.ndarray:
    """The hashed N(0, std)-like value of every element index in `index` (uint64 array) of tensor `tensor_id`."""
    with np.errstate(over="ignore"):
        prefix = _mix64(np.array([np.uint64(seed) + _GOLD * np.uint64(tensor_id + 1)], dtype=np.uint64))[0]
        bits = _mix64(prefix + np.asarray(index, dtype=np.uint64))
    m = np.uint64(0xFFFF)
    S = ((bits & m) + ((bits >> np.uint64(16)) & m) + ((bits >> np.uint64(32)) & m) + (bits >> np.uint64(48))).astype(np.int64)
    x = (S - 131070).astype(np.float32) * np.float32(std / _SIGMA_S)
    return round_to_bf16(x) if bf16 else x


_HASHED_LEAF = {"wq": 0, "wk": 1, "wv": 2, "wo": 3, "w_gate": 4, "w_up": 5, "w_down": 6}


def make_hashed_weights(shape: ModelShape, seed: int, std: float = 0.02) -> Dict[str, np.ndarray]:
    """Random-init weights from the integer hash (what ssd_model_create_random generates on the device)."""
    out: Dict[str, np.ndarray] = {}
    for name in weight_names(shape):
        shp = weight_shape(shape, name)
        if name.endswith("norm"):
            out[name] = np.ones(shp, dtype=np.float32)
            continue
        if name == "embed":
            tid = 0
        elif name == "lm_head":
            tid = 1
        else:
            layer, leaf = name.split(".")
            tid = 16 + 16 * int(layer[1:]) + _HASHED_LEAF[leaf]
        n = int(np.prod(shp))
        out[name] = hashed_normal(seed, tid, np.arange(n, dtype=np.uint64), std, shape.dtype == "bf16").reshape(shp)
    return out


def make_hashed_prefix_kv(shape: ModelShape, batch: int, prefix: int, seed: int):
    """Synthetic unit-variance trunk KV from the integer hash (what ssd_ctx_fill_synthetic_kv generates on the device):
    (k, v), float32 [n_layers][batch][prefix][n_kv_heads][head_dim]."""
    per_seq = prefix * shape.n_kv_heads * shape.head_dim
    idx = (np.arange(batch, dtype=np.uint64)[:, None] << np.uint64(40)) + np.arange(per_seq, dtype=np.uint64)[None, :]
    shp = (batch, prefix, shape.n_kv_heads, shape.head_dim)
    k = np.stack([hashed_normal(seed, (1 << 20) + 2 * l, idx, 1.0, shape.dtype == "bf16").reshape(shp) for l in range(shape.n_layers)])
    v = np.stack([hashed_normal(seed, (1 << 20) + 2 * l + 1, idx, 1.0, shape.dtype == "bf16").reshape(shp) for l in range(shape.n_layers)])
    return k, v
