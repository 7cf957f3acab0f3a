"""Helpers shared by the GPU parity tests: tolerances, error metrics, oracle/GPU set-up."""
from __future__ import annotations

import numpy as np
import torch

import ssd_inputs as I
from oracle import ssd_oracle as O

# spec tolerances: relative error of logits / hidden states against the float64 oracle
TOL = {"bf16": 2e-2, "f32": 1e-4}
# What the bf16 paths (bf16 weights and KV, fp32 accumulation; between the phases of the fused pass the activations that
# meet the weights as one fp16 plane, queries and probabilities as two bf16 planes) are measured at against the float64
# oracle, with head room of about 2x: a wrongly visible key among thousands shows up here long before it reaches the
# spec figure above.  Measured: up to 2.6e-3 through the 16 layers of the 1B shape when both sides start from the
# same bf16-representable prefix KV (1.1e-3 with SSD_CTX_TWO_PLANES), less on the 2-layer shapes; up to 3.9e-3 when the
# whole trunk comes from a prefill on the GPU, whose KV is rounded to bf16 while the oracle keeps its own in float64.
TOL_FUSED_BF16 = 5e-3
TOL_BF16_OWN_PREFILL = 8e-3
# Wide passes (more than 48 rows in one batched forward) carry every activation between phases as ONE plane, in fp16,
# and multiply fp16 copies of the weights: measured 1.8e-3 (mean) and 2.5e-3 (worst row) through the 16 layers of the 1B
# shape, so they are held to the bound of the narrow pass after its own prefill.
TOL_WIDE_BF16 = 8e-3
# SSD_CTX_ONE_PLANE_ALL (a measurement option): queries and probabilities as one bf16 plane too, 8 significant bits
# where the scores and the attention output are formed: 1.1e-2 at the 1B shape.
TOL_ONE_PLANE_BF16 = 2e-2
# decisions that rest on floating point are compared only where the oracle's own margin exceeds this
MARGIN = 1e-4


def row_rel_err(got: np.ndarray, want: np.ndarray) -> float:
    """max over rows of  max|got - want| / max|want|  (rows = all leading axes)."""
    got = np.asarray(got, np.float64).reshape(-1, got.shape[-1])
    want = np.asarray(want, np.float64).reshape(-1, want.shape[-1])
    num = np.abs(got - want).max(axis=1)
    den = np.maximum(np.abs(want).max(axis=1), 1e-30)
    return float((num / den).max())


def elem_rel_err(got: np.ndarray, want: np.ndarray) -> float:
    """The second metric of the parity protocol: max over elements of |got - want| / (|want| + atol) with
    atol = 1e-2 x the row's RMS, so that entries near zero are held to a fraction of the row's scale."""
    got = np.asarray(got, np.float64).reshape(-1, got.shape[-1])
    want = np.asarray(want, np.float64).reshape(-1, want.shape[-1])
    atol = 1e-2 * np.sqrt((want ** 2).mean(axis=1, keepdims=True))
    return float((np.abs(got - want) / (np.abs(want) + np.maximum(atol, 1e-30))).max())


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
