"""CPU oracle for the pre-speculation round of speculative speculative decoding.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, float64 statement of
what the HIP library must compute.  Nothing in the product path may import it;
only the tests, the smoke check and the benchmark's reported CPU baseline do.
It shares no code with the HIP path.

What each function follows (section / equation / algorithm of the paper):

  softmax_T, sigma_FC          Def. "sampling scheme" and Def. "Saguaro sampling
                               scheme" (Sec. 4.2.1)
  acceptance_rate              Theorem 1 (Sec. 2.1)
  residual                     Sec. 2.1, residual distribution
  verify                       Sec. 2.1 (sequential acceptance, bonus token),
                               Def. "verification outcome"
  fan_out                      Sec. 4.1.1, "Saguaro verification outcome
                               prediction algorithm"
  glue_extend                  App. B, "Glue & Recurrence" extend before each round
  branch_mask, branch_step_dense
                               App. B, custom attention mask figure (B=1,K=3,F=4,i=2)
  prespeculate                 Alg. 1, predict_verify_outcomes + speculate_for_outcomes;
                               Def. "speculation cache"; App. C (token / element counts)
  cache_lookup                 Alg. 1 (lookup of the realised outcome), App. B payload
  cache_hit_rate, geometric_fan_out_real, geometric_fan_out
                               Sec. 4.1.2, Def. "r power-law cache hit rate" and Theorem
                               "Saguaro Cache Shape: Geometric Fan-Out"; closed form of
                               F_0 from its proof in the theory appendix
  ssd_generate                 Alg. 1 (whole loop; backup speculator = primary, just in time, or
                               random tokens: the two ends of the fallback strategy of Sec. 4.3)
  random_speculation           Sec. 4.3, the implementation's random-token backup speculator
  sample_token                 Sec. 4.2.1, Def. "sampling scheme": softmax at temperature T,
                               drawn with the Gumbel-max trick; T = 0 is the argmax
  ar_generate                  ordinary autoregressive decoding (the losslessness reference)

The transformer itself (RMSNorm, rotary embedding with the rotate-half pairing,
grouped-query softmax attention, SwiGLU) is the Llama-style decoder the paper's
models are instances of; the paper does not restate it.  "parity unpinned"
applies to no function here: each has a pin in tests/test_oracle_*.py (the
Gumbel-max draw of sample_token at temperature > 0, alone and through
decode_branch, speculate and the sampled ssd_generate loop, in
tests/test_oracle_sampling.py).

Draws of the method (acceptance uniforms, Gumbel noise) come from the
counter-based generator `draw_u`, defined by integer arithmetic only; the HIP
library implements the same generator on its own.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

F64 = np.float64
_MASK64 = (1 << 64) - 1
_GOLD = 0x9E3779B97F4A7C15

STREAM_ACCEPT = 0      # acceptance uniforms of verification: (seq, position, 0)
STREAM_BONUS = 1       # Gumbel noise of the bonus token: (seq, position k, token)
STREAM_DRAFT = 2       # Gumbel noise of branch decoding: (branch row, step, token)
STREAM_SPEC = 3        # Gumbel noise of just-in-time (non-branch) drafting: (seq, step, token)
STREAM_BACKUP = 4      # tokens of the random-token backup speculator: (seq, step, 0)


# --------------------------------------------------------------------------- draws

def _mix64(x: int) -> int:
    x &= _MASK64
    x ^= x >> 30
    x = (x * 0xBF58476D1CE4E5B9) & _MASK64
    x ^= x >> 27
    x = (x * 0x94D049BB133111EB) & _MASK64
    x ^= x >> 31
    return x


def _mix64_vec(x: np.ndarray) -> np.ndarray:
    x = x.astype(np.uint64)
    x ^= x >> np.uint64(30)
    x *= np.uint64(0xBF58476D1CE4E5B9)
    x ^= x >> np.uint64(27)
    x *= np.uint64(0x94D049BB133111EB)
    x ^= x >> np.uint64(31)
    return x


def draw_bits(seed: int, stream: int, a: int, b: int, c) -> np.ndarray:
    """The 64 bits of the four-level hash of (seed, stream, a, b, c).  `c` may be an integer array."""
    h = _mix64(seed ^ ((_GOLD * (stream + 1)) & _MASK64))
    h = _mix64(h + a)
    h = _mix64(h + b)
    with np.errstate(over="ignore"):
        return _mix64_vec(np.uint64(h) + np.asarray(c, dtype=np.uint64))


def draw_u(seed: int, stream: int, a: int, b: int, c) -> np.ndarray:
    """Uniform draw in the open interval (0,1): (m + 1/2) 2^-23, m = top 23 bits of
    `draw_bits`."""
    m = (draw_bits(seed, stream, a, b, c) >> np.uint64(41)).astype(F64)
    return (m + 0.5) * (2.0 ** -23)


def gumbel(seed: int, stream: int, a: int, b: int, vocab: int) -> np.ndarray:
    u = draw_u(seed, stream, a, b, np.arange(vocab, dtype=np.uint64))
    return -np.log(-np.log(u))


# --------------------------------------------------------------------------- distributions

def softmax_T(z: np.ndarray, T: float) -> np.ndarray:
    """softmax(z / T) in float64; T must be > 0."""
    z = np.asarray(z, dtype=F64) / T
    e = np.exp(z - z.max())
    return e / e.sum()


def top_f_ids(z: np.ndarray, F: int, exclude: Optional[int] = None) -> np.ndarray:
    """First F token ids when sorting by (logit descending, token id ascending),
    skipping `exclude`.  Brute force: a full stable sort of the row.  NaN ranks last."""
    z = np.asarray(z)
    key = np.where(np.isnan(z), -np.inf, z)
    order = np.argsort(-key, kind="stable")          # stable: equal logits keep ascending ids
    if exclude is not None:
        order = order[order != exclude]
    return order[:F].astype(np.int32)


def sigma_FC(z: np.ndarray, F: int, C: float, T: float = 1.0) -> np.ndarray:
    """Saguaro sampling scheme: weights exp(z_t/T), multiplied by C on the top-F tokens of z,
    then normalised."""
    z = np.asarray(z, dtype=F64)
    w = np.exp((z - z.max()) / T)
    w[top_f_ids(z, F)] *= C
    return w / w.sum()


def sigma_FC_logits(z: np.ndarray, F: int, C: float, T: float = 1.0) -> np.ndarray:
    """Logits whose softmax at temperature T equals sigma_FC(z): z_t + T log C on top-F."""
    out = np.array(z, dtype=F64, copy=True)
    if C < 1.0:
        out[top_f_ids(z, F)] += T * np.log(C) if C > 0 else -np.inf
    return out


def acceptance_rate(p_t: np.ndarray, p_d: np.ndarray) -> float:
    return float(np.minimum(p_t, p_d).sum())


def residual(p_t: np.ndarray, p_d: np.ndarray) -> np.ndarray:
    """max(p_t - p_d, 0), normalised; all-zero if there is no residual mass."""
    r = np.maximum(np.asarray(p_t, F64) - np.asarray(p_d, F64), 0.0)
    s = r.sum()
    return r / s if s > 0 else r


# --------------------------------------------------------------------------- verification

@dataclass
class VerifyTrace:
    accept_len: int
    bonus: int
    accept_margin: List[float]        # |u q(s) - p(s)| / max(p(s), tiny) per tested position
    bonus_margin: float               # gap between best and second best perturbed score


def verify(target_logits: np.ndarray, draft_logits: Optional[np.ndarray], spec: Sequence[int],
           T: float, seed: int, seq: int = 0) -> VerifyTrace:
    """Lossless verification of one sequence.

    target_logits [K+1][V]: row i is the target's distribution for the token after
    s_1..s_i.  draft_logits [K][V]: row i is the distribution s_{i+1} was drawn from.
    T == 0: greedy (accept while the target's argmax equals the drafted token; bonus =
    argmax at the first mismatch, or at row K).  T > 0: accept s_{i+1} iff
    u_i q(s) < p(s); bonus from the residual at the first rejection via the Gumbel-max
    trick, or from the target's own distribution when all K are accepted.  If the
    residual has no mass (unreachable in exact arithmetic) the bonus comes from p."""
    zt = np.asarray(target_logits, dtype=F64)
    K = len(spec)
    V = zt.shape[1]
    margins: List[float] = []
    if T == 0.0:
        k = K
        for i in range(K):
            if int(top_f_ids(zt[i], 1)[0]) != int(spec[i]):
                k = i
                break
        order = top_f_ids(zt[k], 2)
        return VerifyTrace(k, int(order[0]), margins, float(zt[k][order[0]] - zt[k][order[1]]))
    zd = np.asarray(draft_logits, dtype=F64)
    k = K
    for i in range(K):
        p = softmax_T(zt[i], T)[spec[i]]
        q = softmax_T(zd[i], T)[spec[i]]
        u = float(draw_u(seed, STREAM_ACCEPT, seq, i, 0))
        margins.append(abs(u * q - p) / max(p, 1e-300))
        if not (u * q < p):
            k = i
            break
    p = softmax_T(zt[k], T)
    if k < K:
        r = np.maximum(p - softmax_T(zd[k], T), 0.0)
        if r.sum() <= 0.0:
            r = p
    else:
        r = p
    with np.errstate(divide="ignore"):
        score = np.log(r) + gumbel(seed, STREAM_BONUS, seq, k, V)
    order = top_f_ids(score, 2)
    return VerifyTrace(k, int(order[0]), margins, float(score[order[0]] - score[order[1]]))


# --------------------------------------------------------------------------- transformer

@dataclass
class Model:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_theta: float
    rms_eps: float
    w: Dict[str, np.ndarray]          # float64

    @staticmethod
    def from_weights(shape, weights: Dict[str, np.ndarray]) -> "Model":
        w = {k: np.asarray(v, dtype=F64) for k, v in weights.items()}
        if "lm_head" not in w:
            w["lm_head"] = w["embed"]
        return Model(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                     shape.d_ffn, shape.vocab, float(shape.rope_theta), float(shape.rms_eps), w)


def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    return x / np.sqrt((x * x).mean(axis=-1, keepdims=True) + eps) * gain


def rope(x: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """x [T][H][D], pos [T].  Pair (i, i + D/2) is rotated by pos * theta^(-2i/D)."""
    D = x.shape[-1]
    half = D // 2
    inv = theta ** (-np.arange(half, dtype=F64) * 2.0 / D)
    ang = np.asarray(pos, dtype=F64)[:, None] * inv[None, :]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def attention(q: np.ndarray, keys: np.ndarray, vals: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """softmax(q k^T / sqrt(D) + mask) v per query head; query head h reads KV head
    h // (Hq / Hkv).  q [T][Hq][D], keys/vals [S][Hkv][D], mask [T][S] bool."""
    T, Hq, D = q.shape
    group = Hq // keys.shape[1]
    att = np.empty((T, Hq, D), F64)
    for hq in range(Hq):
        hk = hq // group
        s = q[:, hq, :] @ keys[:, hk, :].T / np.sqrt(D)
        s = np.where(mask, s, -np.inf)
        s = s - s.max(axis=1, keepdims=True)
        p = np.exp(s)
        p = p / p.sum(axis=1, keepdims=True)
        att[:, hq, :] = p @ vals[:, hk, :]
    return att


def swiglu(x: np.ndarray, w_gate: np.ndarray, w_up: np.ndarray, w_down: np.ndarray) -> np.ndarray:
    """down( silu(gate(x)) * up(x) ), silu(g) = g / (1 + exp(-g))."""
    gate = x @ w_gate.T
    up = x @ w_up.T
    return ((gate / (1.0 + np.exp(-gate))) * up) @ w_down.T


@dataclass
class KV:
    """Keys and values of a run of consecutive positions, per layer: [S][n_kv_heads][head_dim]."""
    k: List[np.ndarray]
    v: List[np.ndarray]

    @property
    def length(self) -> int:
        return self.k[0].shape[0]

    def slice(self, n: int) -> "KV":
        return KV([a[:n] for a in self.k], [a[:n] for a in self.v])

    def concat(self, other: "KV") -> "KV":
        return KV([np.concatenate([a, b]) for a, b in zip(self.k, other.k)],
                  [np.concatenate([a, b]) for a, b in zip(self.v, other.v)])

    @staticmethod
    def empty(m: Model) -> "KV":
        z = [np.zeros((0, m.n_kv_heads, m.head_dim), F64) for _ in range(m.n_layers)]
        return KV(list(z), [a.copy() for a in z])


def forward(m: Model, tokens: Sequence[int], positions: Sequence[int], past: KV,
            mask: np.ndarray) -> Tuple[np.ndarray, np.ndarray, KV]:
    """One pass of the decoder over T new tokens.

    mask [T][S + T] (bool): which of the S past keys followed by the T new keys each
    new token may attend.  Returns (logits [T][V], final-norm hidden states [T][d],
    the new tokens' KV)."""
    tokens = np.asarray(tokens, dtype=np.int64)
    pos = np.asarray(positions, dtype=np.int64)
    T = len(tokens)
    Hq, Hkv, D = m.n_q_heads, m.n_kv_heads, m.head_dim
    h = m.w["embed"][tokens]
    new_k, new_v = [], []
    for l in range(m.n_layers):
        g = lambda n: m.w[f"l{l}.{n}"]
        x = rmsnorm(h, g("attn_norm"), m.rms_eps)
        q = rope((x @ g("wq").T).reshape(T, Hq, D), pos, m.rope_theta)
        k = rope((x @ g("wk").T).reshape(T, Hkv, D), pos, m.rope_theta)
        v = (x @ g("wv").T).reshape(T, Hkv, D)
        new_k.append(k)
        new_v.append(v)
        keys = np.concatenate([past.k[l], k])
        vals = np.concatenate([past.v[l], v])
        att = attention(q, keys, vals, mask)
        h = h + att.reshape(T, Hq * D) @ g("wo").T
        x = rmsnorm(h, g("mlp_norm"), m.rms_eps)
        h = h + swiglu(x, g("w_gate"), g("w_up"), g("w_down"))
    hid = rmsnorm(h, m.w["final_norm"], m.rms_eps)
    logits = hid @ m.w["lm_head"].T
    return logits, hid, KV(new_k, new_v)


def causal_mask(S: int, T: int) -> np.ndarray:
    """T new tokens after S past ones: token t sees all past keys and new keys 0..t."""
    mask = np.zeros((T, S + T), dtype=bool)
    mask[:, :S] = True
    mask[:, S:] = np.tril(np.ones((T, T), dtype=bool))
    return mask


def prefill(m: Model, tokens: Sequence[int]) -> Tuple[np.ndarray, KV]:
    """KV of tokens at positions 0..len-1 (dense causal mask) and their logits."""
    T = len(tokens)
    logits, _, kv = forward(m, tokens, np.arange(T), KV.empty(m), causal_mask(0, T))
    return logits, kv


def sample_token(logits: np.ndarray, T: float, noise: Optional[np.ndarray]) -> Tuple[int, float]:
    """argmax (T == 0) or Gumbel-max sample of softmax(logits / T).  Returns (token,
    margin to the runner-up score)."""
    score = np.asarray(logits, F64) if T == 0.0 else np.asarray(logits, F64) / T + noise
    order = top_f_ids(score, 2)
    return int(order[0]), float(score[order[0]] - score[order[1]])


# --------------------------------------------------------------------------- the round

def glue_extend(m: Model, trunk: KV, pending: Sequence[int]) -> Tuple[np.ndarray, np.ndarray, KV]:
    """Extend the trunk by the pending block {last verified token, s_1..s_K} (causal).
    Returns (logits z_1..z_{K+1} as rows 0..K, hidden states, trunk + glue KV)."""
    P = trunk.length
    G = len(pending)
    logits, hid, kv = forward(m, pending, np.arange(P, P + G), trunk, causal_mask(P, G))
    return logits, hid, trunk.concat(kv)


def fan_of(F, K: int) -> np.ndarray:
    """Fan-out per accept length: F_k, k = 0..K.  A plain integer is the uniform cache shape."""
    fan = np.full(K + 1, F, np.int64) if np.ndim(F) == 0 else np.asarray(F, np.int64)
    assert fan.shape == (K + 1,) and (fan >= 1).all()
    return fan


def fan_out(glue_logits: np.ndarray, pending: Sequence[int], F) -> np.ndarray:
    """keys[k][j], k = 0..K: the F_k most likely bonus tokens if exactly k drafted tokens
    are accepted: top-F_k of the logits s_{k+1} was drawn from, without s_{k+1} itself
    (a rejected token has zero residual mass); for k = K, top-F_K of the logits after s_K.
    With a fan-out that differs per accept length (Sec. 4.1.2) the array is max F_k wide and
    the unused entries hold -1, which no token equals."""
    K = len(pending) - 1
    fan = fan_of(F, K)
    keys = np.full((K + 1, int(fan.max())), -1, dtype=np.int32)
    for k in range(K + 1):
        keys[k, :fan[k]] = top_f_ids(glue_logits[k], int(fan[k]), exclude=int(pending[k + 1]) if k < K else None)
    return keys


# --------------------------------------------------------------------------- cache shape (Sec. 4.1.2)

def cache_hit_rate(fan: Sequence[float], a: float, r: float) -> float:
    """Chance that the verification outcome of a speculation is in the cache, for a speculator
    with acceptance rate a whose miss rate at fan-out F is F^-r: exactly k < K tokens are
    accepted with probability a^k (1 - a), all K with probability a^K, and the outcome at
    accept length k is among the F_k cached ones with probability 1 - F_k^-r."""
    K = len(fan) - 1
    p = a ** K * (1.0 - float(fan[K]) ** -r)
    for k in range(K):
        p += a ** k * (1.0 - a) * (1.0 - float(fan[k]) ** -r)
    return p


def geometric_fan_out_real(budget: float, K: int, a: float, r: float) -> np.ndarray:
    """The real-valued F_0..F_K that maximise `cache_hit_rate` under sum F_k = budget
    (Theorem "Geometric Fan-Out"): F_k = F_0 a^(k/(1+r)) below K, the last one larger by
    (1-a)^(-1/(1+r)), F_0 from the budget."""
    assert 0.0 < a < 1.0 and r > 0.0 and K >= 0
    q = a ** (1.0 / (1.0 + r))
    last = q ** K * (1.0 - a) ** (-1.0 / (1.0 + r))
    f0 = budget / (last + (1.0 - q ** K) / (1.0 - q))
    return np.array([f0 * q ** k for k in range(K)] + [f0 * last], F64)


def geometric_fan_out(budget: int, K: int, a: float, r: float, f_max: Optional[int] = None) -> np.ndarray:
    """Integer cache shape from the theorem's real-valued one.  The paper does not say how the
    F_k become integers; the reading taken here: every accept length keeps at least one
    candidate, none more than f_max; an F_k the real solution puts outside [1, f_max] is fixed
    at that bound and the rest of the budget is shared among the others in the theorem's
    proportions (the stationarity conditions of the bounded problem); the shares are rounded
    down and the units left over go to the largest fractional parts, lower k first on ties,
    so that sum F_k = budget exactly."""
    cap = budget if f_max is None else f_max
    assert K + 1 <= budget <= (K + 1) * cap
    w = geometric_fan_out_real(1.0, K, a, r)            # proportions
    lo = np.zeros(K + 1, bool)
    hi = np.zeros(K + 1, bool)
    while True:
        free = ~(lo | hi)
        left = budget - int(lo.sum()) - cap * int(hi.sum())
        x = np.where(lo, 1.0, np.where(hi, float(cap), 0.0))
        if free.any():
            x[free] = left * w[free] / w[free].sum()
        over = free & (x > cap)
        under = free & (x < 1.0)
        if over.any():                                  # bind one kind at a time, the upper bound first
            hi |= over
        elif under.any():
            lo |= under
        else:
            break
    fan = np.floor(x + 1e-9).astype(np.int64)
    frac = x - fan
    order = sorted(range(K + 1), key=lambda k: (-frac[k], k))
    spare = budget - int(fan.sum())
    i = 0
    while spare > 0:
        k = order[i % (K + 1)]
        if fan[k] < cap:
            fan[k] += 1
            spare -= 1
        i += 1
    return fan


@dataclass
class SpecCache:
    keys: np.ndarray        # int32 [K+1][F]           (F = max F_k; entries j >= F_k are -1 / zero)
    tokens: np.ndarray      # int32 [K+1][F][K]
    logits: np.ndarray      # float64 [K+1][F][K][V]
    hidden: np.ndarray      # float64 [K+1][F][K][d]   (final-norm hidden states, for parity)
    margins: np.ndarray     # float64 [K+1][F][K]      (sampling margin of every decoded token)
    glue_logits: np.ndarray # float64 [K+1][V]
    trunk: KV               # trunk + glue KV after the extend
    fan: Optional[np.ndarray] = None   # int64 [K+1]: F_k


def decode_branch(m: Model, trunk_glue: KV, P: int, k: int, first: int, steps: int, T: float,
                  seed: int, row: int, forced: Optional[Sequence[int]] = None,
                  sigma: Optional[Tuple[int, float]] = None):
    """One branch on its own: feed `first` at position P+1+k on top of trunk[0 .. P+k],
    then its own continuation.  With `forced` (teacher forcing) step i > 0 feeds
    forced[i-1] instead of its own sample.  Returns (tokens, logits, hidden, margins).

    `sigma` = (F, C) drafts with the Saguaro sampling scheme sigma_{F,C} (Sec. 4.2.1): at T > 0
    every token is drawn from the model's logits with the top-F entries downweighted by C, and
    those are the logits returned (the distribution a verifier has to be given).  F is one
    number, or one per step."""
    past = trunk_glue.slice(P + k + 1)
    tok = int(first)
    toks, logs, hids, margs = [], [], [], []
    for i in range(steps):
        S = past.length
        logits, hid, kv = forward(m, [tok], [P + 1 + k + i], past, np.ones((1, S + 1), dtype=bool))
        past = past.concat(kv)
        noise = gumbel(seed, STREAM_DRAFT, row, i, m.vocab) if T > 0 else None
        z = logits[0]
        if sigma is not None and T > 0.0:
            z = sigma_FC_logits(z, int(sigma[0]) if np.ndim(sigma[0]) == 0 else int(sigma[0][i]), sigma[1], T)
        nxt, margin = sample_token(z, T, noise)
        toks.append(nxt)
        logs.append(z)
        hids.append(hid[0])
        margs.append(margin)
        tok = nxt if forced is None else int(forced[i])
    return np.array(toks, np.int32), np.array(logs), np.array(hids), np.array(margs)


def prespeculate(m: Model, trunk: KV, pending: Sequence[int], F, T: float, seed: int,
                 row_base: int = 0,
                 only_rows: Optional[Sequence[int]] = None,
                 forced_tokens: Optional[np.ndarray] = None,
                 C: float = 1.0) -> SpecCache:
    """One pre-speculation round for one sequence: glue extend, fan-out, then every branch
    (k, j) decoded for K tokens, one branch at a time, each with KV of its own.

    F is the uniform fan-out, or F_0..F_K (Sec. 4.1.2).  Branches are numbered accept length
    by accept length, r = F_0 + .. + F_{k-1} + j (k F + j when uniform); `row_base` is the
    global row index of branch (0,0) (a batch numbers its rows sequence after sequence; the
    index keys the draft Gumbel stream).  `only_rows` restricts the decode to a sample of
    branches (the others are left zero).  `forced_tokens` [K+1][max F_k][K] teacher-forces
    every branch's inputs.  C < 1 decodes the branches with the sampling scheme sigma_{F,C}
    (Sec. 4.2.1); the fan-out itself always ranks the model's own logits.  The token drafted at
    depth i is the one whose rejection ends the next round at accept length i, where the
    cache will hold F_i candidates: that is the F its logits are downweighted with."""
    K = len(pending) - 1
    P = trunk.length
    fan = fan_of(F, K)
    Fm = int(fan.max())
    off = np.concatenate([[0], np.cumsum(fan)])
    glue_logits, _, trunk_glue = glue_extend(m, trunk, pending)
    keys = fan_out(glue_logits, pending, fan)
    tokens = np.zeros((K + 1, Fm, K), np.int32)
    logits = np.zeros((K + 1, Fm, K, m.vocab), F64)
    hidden = np.zeros((K + 1, Fm, K, m.d_model), F64)
    margins = np.full((K + 1, Fm, K), np.inf, F64)
    for k in range(K + 1):
        for j in range(int(fan[k])):
            r = int(off[k]) + j
            if only_rows is not None and r not in only_rows:
                continue
            forced = None if forced_tokens is None else forced_tokens[k, j]
            t, l, h, g = decode_branch(m, trunk_glue, P, k, keys[k, j], K, T, seed, row_base + r, forced,
                                       sigma=(fan[:K], C) if C < 1.0 else None)
            tokens[k, j], logits[k, j], hidden[k, j], margins[k, j] = t, l, h, g
    return SpecCache(keys, tokens, logits, hidden, margins, glue_logits, trunk_glue, fan)


def cache_lookup(keys: np.ndarray, accept_len: int, bonus: int) -> int:
    """Branch index j with keys[accept_len][j] == bonus, or -1 (cache miss)."""
    for j, t in enumerate(keys[accept_len]):
        if int(t) == int(bonus):
            return j
    return -1


# --------------------------------------------------------------------------- the mask of App. B

def branch_mask(P: int, K: int, F: int, i: int) -> np.ndarray:
    """Dense mask of one batched branch-decode step at depth i for one sequence.

    Rows: the (K+1) F branches, row = k F + j.  Columns: the P verified prefix positions,
    the K+1 glue positions, then (i+1) blocks of (K+1) F columns, block e holding every
    branch's token at depth e (block i is the step's own new tokens).  Row (k, j) sees
    the whole prefix, glue 0..k, and column (k, j) of every block."""
    M = (K + 1) * F
    mask = np.zeros((M, P + K + 1 + (i + 1) * M), dtype=bool)
    for k in range(K + 1):
        for j in range(F):
            r = k * F + j
            mask[r, :P + k + 1] = True
            for e in range(i + 1):
                mask[r, P + K + 1 + e * M + r] = True
    return mask


def branch_step_dense(m: Model, trunk_glue: KV, P: int, K: int, F: int, i: int,
                      step_tokens: Sequence[int], earlier: KV):
    """All (K+1) F branches at depth i in ONE forward pass under `branch_mask` (the paper's
    formulation).  `earlier` holds the branch tokens' KV of depths 0..i-1, block after block.
    Returns (logits [M][V], the new block's KV)."""
    M = (K + 1) * F
    pos = [P + 1 + (r // F) + i for r in range(M)]
    past = trunk_glue.concat(earlier)
    logits, _, kv = forward(m, step_tokens, pos, past, branch_mask(P, K, F, i))
    return logits, kv


# --------------------------------------------------------------------------- whole loops

def ar_generate(m: Model, prompt: Sequence[int], n_new: int, T: float = 0.0) -> List[int]:
    """Greedy autoregressive decoding by full recomputation (no KV reuse at all)."""
    assert T == 0.0
    seq = list(int(t) for t in prompt)
    for _ in range(n_new):
        logits, _ = prefill(m, seq)
        seq.append(int(top_f_ids(logits[-1], 1)[0]))
    return seq[len(prompt):]


def speculate(m: Model, trunk: KV, last: int, K: int, T: float, seed: int, seq: int = 0):
    """Ordinary (just-in-time) drafting: K tokens after `last`, one at a time.
    Returns (tokens [K], logits [K][V])."""
    past = trunk
    tok = int(last)
    toks, logs = [], []
    for i in range(K):
        S = past.length
        logits, _, kv = forward(m, [tok], [S], past, np.ones((1, S + 1), dtype=bool))
        past = past.concat(kv)
        noise = gumbel(seed, STREAM_SPEC, seq, i, m.vocab) if T > 0 else None
        tok, _ = sample_token(logits[0], T, noise)
        toks.append(tok)
        logs.append(logits[0])
    return toks, np.array(logs)


def random_speculation(seed: int, seq: int, K: int, vocab: int) -> Tuple[List[int], np.ndarray]:
    """The fast backup speculator of Sec. 4.3: K tokens drawn uniformly from the vocabulary, at
    no model cost.  Token i is the hash of (seed, backup stream, seq, i, 0) modulo the vocabulary
    size (all 64 bits, so the draw is uniform to 2^-47).  Returns (tokens, logits): the logits are
    all zero, i.e. the uniform distribution the tokens were drawn from, which is what lossless
    verification at temperature > 0 has to be given (Sec. 2.1)."""
    toks = [int(draw_bits(seed, STREAM_BACKUP, seq, i, 0)) % vocab for i in range(K)]
    return toks, np.zeros((K, vocab), F64)


@dataclass
class SSDStats:
    rounds: int = 0
    hits: int = 0
    accepted: int = 0
    accept_lens: Optional[List[int]] = None


def ssd_generate(target: Model, draft: Model, prompt: Sequence[int], n_new: int, K: int, F,
                 T: float = 0.0, seed: int = 0, backup: str = "primary") -> Tuple[List[int], SSDStats]:
    """Alg. 1 for one sequence, run sequentially: speculate, then per round
    {verify the pending speculation, pre-speculate for predicted outcomes, look the realised
    outcome up, fall back on a miss}.  The fallback (Sec. 4.3) is just-in-time drafting with the
    same draft (backup = "primary", the low-batch choice) or K random tokens (backup =
    "random", the low-latency choice for large batches)."""
    assert backup in ("primary", "random")
    X = [int(t) for t in prompt]
    n0 = len(X)
    stats = SSDStats(accept_lens=[])
    _, d_trunk = prefill(draft, X[:-1])
    spec, spec_logits = speculate(draft, d_trunk, X[-1], K, T, seed)
    rnd = 0
    while len(X) - n0 < n_new:
        rnd += 1
        rseed = seed + 1000003 * rnd
        # verifier: target logits over {X[-1], s_1..s_K} by full recomputation
        full, _ = prefill(target, X + list(spec))
        zt = full[len(X) - 1:]
        out = verify(zt, spec_logits, spec, T, rseed)
        # speculator, concurrently: pre-speculate for the outcomes of the pending speculation
        pending = [X[-1]] + list(spec)
        cache = prespeculate(draft, d_trunk, pending, F, T, rseed)
        k, bonus = out.accept_len, out.bonus
        X += list(spec[:k]) + [bonus]
        stats.rounds += 1
        stats.accepted += k
        stats.accept_lens.append(k)
        d_trunk = cache.trunk.slice(d_trunk.length + k + 1)
        j = cache_lookup(cache.keys, k, bonus)
        if j >= 0:
            stats.hits += 1
            spec, spec_logits = list(cache.tokens[k, j]), cache.logits[k, j]
        elif backup == "primary":
            spec, spec_logits = speculate(draft, d_trunk, bonus, K, T, rseed)
        else:
            spec, spec_logits = random_speculation(rseed, 0, K, draft.vocab)
    return X[n0:n0 + n_new], stats
