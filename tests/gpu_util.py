"""Helpers shared by the GPU parity tests: tolerances, error metrics, oracle/GPU set-up."""
from __future__ import annotations

import numpy as np
import torch

import ssd_inputs as I
from oracle import ssd_oracle as O

# spec tolerances: relative error of logits / hidden states against the float64 oracle
TOL = {"bf16": 2e-2, "f32": 1e-4}
# decisions that rest on floating point are compared only where the oracle's own margin exceeds this
MARGIN = 1e-4


def row_rel_err(got: np.ndarray, want: np.ndarray) -> float:
    """max over rows of  max|got - want| / max|want|  (rows = all leading axes)."""
    got = np.asarray(got, np.float64).reshape(-1, got.shape[-1])
    want = np.asarray(want, np.float64).reshape(-1, want.shape[-1])
    num = np.abs(got - want).max(axis=1)
    den = np.maximum(np.abs(want).max(axis=1), 1e-30)
    return float((num / den).max())


def rms_rel_err(got: np.ndarray, want: np.ndarray) -> float:
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    return float(np.sqrt(((got - want) ** 2).sum() / max((want ** 2).sum(), 1e-300)))


def dev_i32(a) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def dev_f32(a) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def kv_to_device(k: np.ndarray, dtype: str) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(k, dtype=np.float32))
    return (t.to(torch.bfloat16) if dtype == "bf16" else t).cuda()


def oracle_trunk_from_arrays(m: O.Model, k: np.ndarray, v: np.ndarray, b: int) -> O.KV:
    """Synthetic prefix KV [L][B][P][Hkv][D] -> the oracle's per-layer lists for sequence b."""
    return O.KV([k[l, b].astype(np.float64) for l in range(m.n_layers)],
                [v[l, b].astype(np.float64) for l in range(m.n_layers)])
