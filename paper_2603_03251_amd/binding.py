"""ctypes binding of libssd_hip.so: the same names as include/ssd.h, argument marshalling only.

PyTorch is used for device memory and streams; every step of the path runs in the library's
kernels.  There is no CPU fallback: if the library is missing, importing this module fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch  # imported before the library so that both share one HIP runtime

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libssd_hip.so")

SSD_OK, SSD_EINVAL, SSD_ESTATE, SSD_EHIP, SSD_ENOMEM = 0, -1, -2, -3, -4
SSD_F32, SSD_BF16 = 0, 1
SSD_MAX_F, SSD_MAX_K = 16, 15
SSD_CTX_PER_OPERATOR, SSD_CTX_FUSED_PHASES, SSD_CTX_NARROW_PASSES = 1, 2, 4
SSD_CTX_ONE_PLANE_ALL = 0x1f00
SSD_CTX_TWO_PLANES = 0x2000
SSD_DEBUG_BARRIER_EPOCH, SSD_DEBUG_SPIN_LIMIT = 1, 2


class SsdError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"ssd status {status}: {message}")
        self.status = status


class ssd_model_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn",
                                         "vocab", "dtype")] + \
               [("rope_theta", C.c_float), ("rms_eps", C.c_float), ("tie_embeddings", C.c_int32)]


class ssd_model_weights(C.Structure):
    _fields_ = [("d_embed", C.c_void_p), ("d_lm_head", C.c_void_p), ("d_final_norm", C.c_void_p)] + \
               [(n, C.POINTER(C.c_void_p)) for n in ("h_attn_norm", "h_wq", "h_wk", "h_wv", "h_wo", "h_mlp_norm",
                                                     "h_w_gate", "h_w_up", "h_w_down")]


class ssd_round_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("batch", "K", "F", "max_trunk", "flags", "kv_pages")]


class ssd_views(C.Structure):
    _fields_ = [("d_trunk_len", C.c_void_p), ("d_keys", C.c_void_p), ("d_tokens", C.c_void_p),
                ("d_logits", C.c_void_p), ("d_hidden", C.c_void_p), ("d_glue_logits", C.c_void_p),
                ("d_glue_hidden", C.c_void_p), ("h_trunk_k", C.POINTER(C.c_void_p)),
                ("h_trunk_v", C.POINTER(C.c_void_p))] + \
               [(n, C.c_int32) for n in ("batch", "K", "F", "vocab", "d_model", "max_trunk", "fused_pass", "pass_rows")]


EXPORTS = {
    "ssd_last_error": (C.c_char_p, []),
    "ssd_model_create": (C.c_int, [C.POINTER(ssd_model_config), C.POINTER(ssd_model_weights), C.c_void_p,
                                   C.POINTER(C.c_void_p)]),
    "ssd_model_create_random": (C.c_int, [C.POINTER(ssd_model_config), C.c_uint64, C.c_void_p, C.POINTER(C.c_void_p)]),
    "ssd_model_destroy": (C.c_int, [C.c_void_p]),
    "ssd_model_release_operator_weights": (C.c_int, [C.c_void_p]),
    "ssd_ctx_create": (C.c_int, [C.c_void_p, C.POINTER(ssd_round_config), C.POINTER(C.c_void_p)]),
    "ssd_ctx_destroy": (C.c_int, [C.c_void_p]),
    "ssd_ctx_prefill": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.c_void_p]),
    "ssd_ctx_fill_synthetic_kv": (C.c_int, [C.c_void_p, C.POINTER(C.c_int32), C.c_uint64, C.c_void_p]),
    "ssd_ctx_kv_pages": (C.c_int, [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
    "ssd_ctx_release_sequence": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p]),
    "ssd_ctx_prefill_sequence": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p]),
    "ssd_ctx_load_trunk": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]),
    "ssd_prespeculate": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p]),
    "ssd_ctx_set_forced": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "ssd_ctx_set_saguaro": (C.c_int, [C.c_void_p, C.c_float]),
    "ssd_ctx_create_fanout": (C.c_int, [C.c_void_p, C.POINTER(ssd_round_config), C.POINTER(C.c_int32),
                                        C.POINTER(C.c_void_p)]),
    "ssd_ctx_fanout": (C.c_int, [C.c_void_p, C.POINTER(C.c_int32)]),
    "ssd_ctx_truncate_trunk": (C.c_int, [C.c_void_p, C.POINTER(C.c_int32), C.c_void_p]),
    "ssd_backup_random": (C.c_int, [C.c_uint64, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]),
    "ssd_geometric_fanout": (C.c_int, [C.c_int32, C.c_int32, C.c_double, C.c_double, C.c_int32, C.POINTER(C.c_int32)]),
    "ssd_cache_lookup": (C.c_int, [C.c_void_p] * 8),
    "ssd_ctx_commit": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "ssd_verify": (C.c_int, [C.c_void_p] * 4 + [C.c_int32] * 3 + [C.c_uint64] + [C.c_void_p] * 4),
    "ssd_verify_workspace_bytes": (C.c_size_t, [C.c_int32, C.c_int32]),
    "ssd_verify_static": (C.c_int, [C.c_void_p] * 4 + [C.c_int32] * 3 + [C.c_uint64] + [C.c_void_p] * 3),
    "ssd_verify_static_capacity": (C.c_size_t, []),
    "ssd_top_f": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                            C.c_void_p, C.c_void_p]),
    "ssd_top_f_workspace_bytes": (C.c_size_t, [C.c_int32]),
    "ssd_sample": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int32, C.c_int32, C.c_uint64, C.c_int32,
                             C.c_int32, C.c_void_p, C.c_void_p]),
    "ssd_sample_fp64_scan": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int32, C.c_int32, C.c_uint64, C.c_int32,
                                       C.c_int32, C.c_void_p, C.c_void_p]),
    "ssd_ctx_status": (C.c_int, [C.c_void_p]),
    "ssd_ctx_recover": (C.c_int, [C.c_void_p]),
    "ssd_ctx_debug_set": (C.c_int, [C.c_void_p, C.c_int32, C.c_uint32]),
    "ssd_ctx_extend": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]),
    "ssd_ctx_refresh_bounds": (C.c_int, [C.c_void_p, C.c_void_p]),
    "ssd_ctx_enable_timing": (C.c_int, [C.c_void_p, C.c_int32]),
    "ssd_ctx_read_timing": (C.c_int, [C.c_void_p, C.POINTER(C.c_float), C.c_int32]),
    "ssd_ctx_views": (C.c_int, [C.c_void_p, C.POINTER(ssd_views)]),
    "ssd_ctx_enable_phase_clocks": (C.c_int, [C.c_void_p, C.c_int32]),
    "ssd_ctx_read_phase_clocks": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.POINTER(C.c_int32),
                                            C.POINTER(C.c_int32)]),
}


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2603_03251_amd.build` "
                           "(there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    for name, (res, args) in EXPORTS.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    return lib


lib = _load()


def _check(status: int) -> None:
    if status != SSD_OK:
        raise SsdError(status, lib.ssd_last_error().decode())


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("device pointers must come from contiguous CUDA/HIP tensors")
    return t.data_ptr()


def _stream(stream: Optional[torch.cuda.Stream]) -> int:
    return (stream or torch.cuda.current_stream()).cuda_stream


def _hip():
    if not hasattr(_hip, "lib"):
        h = C.CDLL("libamdhip64.so.7")   # already loaded by torch: resolves to the same runtime
        h.hipMemcpyAsync.restype = C.c_int
        h.hipMemcpyAsync.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int, C.c_void_p]
        _hip.lib = h
    return _hip.lib


def device_copy(ptr: int, shape: Sequence[int], dtype: torch.dtype, stream=None) -> torch.Tensor:
    """A fresh tensor holding a copy of library-owned device memory (for tests and read-outs)."""
    out = torch.empty(tuple(shape), dtype=dtype, device="cuda")
    if out.numel():
        err = _hip().hipMemcpyAsync(out.data_ptr(), ptr, out.numel() * out.element_size(), 3, _stream(stream))
        if err != 0:
            raise RuntimeError(f"hipMemcpyAsync failed with {err}")
    return out


# --------------------------------------------------------------------------- same-name wrappers

def to_device_weight(a: np.ndarray, dtype: str) -> torch.Tensor:
    """float32 numpy (bf16-representable for bf16 models) -> device tensor of the model dtype."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.to(torch.bfloat16).cuda() if dtype == "bf16" else t.cuda()


def ssd_model_create(shape, weights: Dict[str, np.ndarray], stream=None) -> int:
    """shape: any object with the fields of ssd_model_config (dtype as "f32"/"bf16")."""
    cfg = ssd_model_config(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                           shape.d_ffn, shape.vocab, SSD_BF16 if shape.dtype == "bf16" else SSD_F32,
                           shape.rope_theta, shape.rms_eps, 1 if shape.tie_embeddings else 0)
    keep = {}

    def dev(name):
        # one upload per distinct array: a caller may give several layers the same weights (a deep model for timing
        # whose host copy stays small)
        a = weights[name]
        if id(a) not in keep:
            keep[id(a)] = to_device_weight(a, shape.dtype)
        return keep[id(a)].data_ptr()

    w = ssd_model_weights()
    w.d_embed = dev("embed")
    w.d_lm_head = None if shape.tie_embeddings else dev("lm_head")
    w.d_final_norm = dev("final_norm")
    tables = {}
    for field, leaf in (("h_attn_norm", "attn_norm"), ("h_wq", "wq"), ("h_wk", "wk"), ("h_wv", "wv"), ("h_wo", "wo"),
                        ("h_mlp_norm", "mlp_norm"), ("h_w_gate", "w_gate"), ("h_w_up", "w_up"), ("h_w_down", "w_down")):
        arr = (C.c_void_p * shape.n_layers)(*[dev(f"l{l}.{leaf}") for l in range(shape.n_layers)])
        tables[field] = arr
        setattr(w, field, arr)
    out = C.c_void_p()
    _check(lib.ssd_model_create(C.byref(cfg), C.byref(w), _stream(stream), C.byref(out)))
    torch.cuda.synchronize()     # the caller's copies (keep) may go once the re-tiling has run
    return out.value


def _model_config(shape) -> ssd_model_config:
    return ssd_model_config(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                            shape.d_ffn, shape.vocab, SSD_BF16 if shape.dtype == "bf16" else SSD_F32,
                            shape.rope_theta, shape.rms_eps, 1 if shape.tie_embeddings else 0)


def ssd_model_create_random(shape, seed: int, stream=None) -> int:
    cfg = _model_config(shape)
    out = C.c_void_p()
    _check(lib.ssd_model_create_random(C.byref(cfg), seed, _stream(stream), C.byref(out)))
    return out.value


def ssd_model_destroy(model: int) -> None:
    _check(lib.ssd_model_destroy(model))


def ssd_model_release_operator_weights(model: int) -> None:
    _check(lib.ssd_model_release_operator_weights(model))


def ssd_ctx_create(model: int, batch: int, K: int, F: int, max_trunk: int, flags: int = 0, kv_pages: int = 0) -> int:
    cfg = ssd_round_config(batch, K, F, max_trunk, flags, kv_pages)
    out = C.c_void_p()
    _check(lib.ssd_ctx_create(model, C.byref(cfg), C.byref(out)))
    return out.value


def ssd_ctx_create_fanout(model: int, batch: int, K: int, fanout: Sequence[int], max_trunk: int, flags: int = 0,
                          kv_pages: int = 0) -> int:
    assert len(fanout) == K + 1
    cfg = ssd_round_config(batch, K, 0, max_trunk, flags, kv_pages)
    fan = (C.c_int32 * (K + 1))(*[int(f) for f in fanout])
    out = C.c_void_p()
    _check(lib.ssd_ctx_create_fanout(model, C.byref(cfg), fan, C.byref(out)))
    return out.value


def ssd_ctx_fanout(ctx: int) -> List[int]:
    K = ssd_ctx_views(ctx).K
    fan = (C.c_int32 * (K + 1))()
    _check(lib.ssd_ctx_fanout(ctx, fan))
    return list(fan)


def ssd_geometric_fanout(budget: int, K: int, a: float, r: float, f_max: int = SSD_MAX_F) -> List[int]:
    fan = (C.c_int32 * (K + 1))()
    _check(lib.ssd_geometric_fanout(budget, K, a, r, f_max, fan))
    return list(fan)


def ssd_ctx_destroy(ctx: int) -> None:
    _check(lib.ssd_ctx_destroy(ctx))


def ssd_ctx_prefill(ctx: int, tokens: torch.Tensor, lens: Sequence[int], stream=None) -> None:
    h = (C.c_int32 * len(lens))(*[int(x) for x in lens])
    _check(lib.ssd_ctx_prefill(ctx, _ptr(tokens), tokens.shape[1], h, _stream(stream)))


def ssd_ctx_load_trunk(ctx: int, k: torch.Tensor, v: torch.Tensor, length: int, stream=None) -> None:
    _check(lib.ssd_ctx_load_trunk(ctx, _ptr(k), _ptr(v), length, _stream(stream)))


def ssd_ctx_kv_pages(ctx: int) -> Tuple[int, int]:
    """(pages of the pool, pages free); (0, 0) for a contiguous trunk."""
    total, free = C.c_int32(), C.c_int32()
    _check(lib.ssd_ctx_kv_pages(ctx, C.byref(total), C.byref(free)))
    return total.value, free.value


def ssd_ctx_release_sequence(ctx: int, b: int, stream=None) -> None:
    _check(lib.ssd_ctx_release_sequence(ctx, b, _stream(stream)))


def ssd_ctx_prefill_sequence(ctx: int, b: int, tokens: torch.Tensor, stream=None) -> None:
    """tokens: device int32 [len]"""
    assert tokens.dtype == torch.int32 and tokens.is_cuda and tokens.dim() == 1 and tokens.is_contiguous()
    _check(lib.ssd_ctx_prefill_sequence(ctx, b, tokens.data_ptr(), tokens.numel(), _stream(stream)))


def ssd_ctx_fill_synthetic_kv(ctx: int, lens: Sequence[int], seed: int, stream=None) -> None:
    h = (C.c_int32 * len(lens))(*[int(x) for x in lens])
    _check(lib.ssd_ctx_fill_synthetic_kv(ctx, h, seed, _stream(stream)))


def ssd_ctx_truncate_trunk(ctx: int, lens: Sequence[int], stream=None) -> None:
    h = (C.c_int32 * len(lens))(*[int(x) for x in lens])
    _check(lib.ssd_ctx_truncate_trunk(ctx, h, _stream(stream)))


def ssd_prespeculate(ctx: int, pending: torch.Tensor, temperature: torch.Tensor, round_seed: int, stream=None) -> None:
    _check(lib.ssd_prespeculate(ctx, _ptr(pending), _ptr(temperature), round_seed, _stream(stream)))


def ssd_ctx_set_forced(ctx: int, keys: Optional[torch.Tensor], tokens: Optional[torch.Tensor]) -> None:
    _check(lib.ssd_ctx_set_forced(ctx, _ptr(keys), _ptr(tokens)))


def ssd_ctx_set_saguaro(ctx: int, C_: float) -> None:
    _check(lib.ssd_ctx_set_saguaro(ctx, float(C_)))


def ssd_cache_lookup(ctx: int, accept_len, bonus, hit, branch, spec_tokens, logits_ptr=None, stream=None) -> None:
    _check(lib.ssd_cache_lookup(ctx, _ptr(accept_len), _ptr(bonus), _ptr(hit), _ptr(branch), _ptr(spec_tokens),
                                _ptr(logits_ptr), _stream(stream)))


def ssd_ctx_commit(ctx: int, accept_len: torch.Tensor, stream=None) -> None:
    _check(lib.ssd_ctx_commit(ctx, _ptr(accept_len), _stream(stream)))


def ssd_verify_workspace_bytes(B: int, K: int) -> int:
    return lib.ssd_verify_workspace_bytes(B, K)


def ssd_verify(target_logits, draft_logits, spec_tokens, temperature, seed: int, accept_len, bonus, workspace,
               stream=None) -> None:
    B, K1, V = target_logits.shape
    _check(lib.ssd_verify(_ptr(target_logits), _ptr(draft_logits), _ptr(spec_tokens), _ptr(temperature), B, K1 - 1, V,
                          seed, _ptr(accept_len), _ptr(bonus), _ptr(workspace), _stream(stream)))


def ssd_verify_static(target_logits, draft_logits, spec_tokens, temperature, seed: int, accept_len, bonus,
                      stream=None) -> None:
    B, K1, V = target_logits.shape
    _check(lib.ssd_verify_static(_ptr(target_logits), _ptr(draft_logits), _ptr(spec_tokens), _ptr(temperature), B, K1 - 1,
                                 V, seed, _ptr(accept_len), _ptr(bonus), _stream(stream)))


def ssd_verify_static_capacity() -> int:
    return int(lib.ssd_verify_static_capacity())


def ssd_backup_random(seed: int, V: int, tokens: torch.Tensor, stream=None) -> None:
    nb, K = tokens.shape
    assert tokens.dtype == torch.int32 and tokens.is_contiguous()
    _check(lib.ssd_backup_random(seed, nb, K, V, _ptr(tokens), _stream(stream)))


def ssd_top_f_workspace_bytes(rows: int) -> int:
    return int(lib.ssd_top_f_workspace_bytes(rows))


def ssd_top_f(logits: torch.Tensor, exclude: Optional[torch.Tensor], F: int, ids: torch.Tensor,
              workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    rows, V = logits.shape
    assert workspace is None or workspace.numel() * workspace.element_size() >= ssd_top_f_workspace_bytes(rows)
    _check(lib.ssd_top_f(_ptr(logits), V, _ptr(exclude), rows, V, F, _ptr(ids), _ptr(workspace), _stream(stream)))


def ssd_sample(logits: torch.Tensor, temperature: torch.Tensor, seed: int, row_base: int, step: int,
               out: torch.Tensor, stream=None) -> None:
    rows, V = logits.shape
    _check(lib.ssd_sample(_ptr(logits), V, _ptr(temperature), rows, V, seed, row_base, step, _ptr(out), _stream(stream)))


def ssd_sample_fp64_scan(logits: torch.Tensor, temperature: torch.Tensor, seed: int, row_base: int, step: int,
                         out: torch.Tensor, stream=None) -> None:
    rows, V = logits.shape
    _check(lib.ssd_sample_fp64_scan(_ptr(logits), V, _ptr(temperature), rows, V, seed, row_base, step, _ptr(out),
                                    _stream(stream)))


def ssd_ctx_status(ctx: int) -> None:
    _check(lib.ssd_ctx_status(ctx))


def ssd_ctx_recover(ctx: int) -> None:
    _check(lib.ssd_ctx_recover(ctx))


def ssd_ctx_debug_set(ctx: int, what: int, value: int) -> None:
    _check(lib.ssd_ctx_debug_set(ctx, what, value))


def ssd_ctx_extend(ctx: int, tokens: torch.Tensor, offset: int, logits: Optional[torch.Tensor], stream=None) -> None:
    _check(lib.ssd_ctx_extend(ctx, _ptr(tokens), tokens.shape[1], offset, _ptr(logits), _stream(stream)))


def ssd_ctx_refresh_bounds(ctx: int, stream=None) -> None:
    _check(lib.ssd_ctx_refresh_bounds(ctx, _stream(stream)))


def ssd_ctx_enable_timing(ctx: int, on: bool) -> None:
    _check(lib.ssd_ctx_enable_timing(ctx, 1 if on else 0))


def ssd_ctx_read_timing(ctx: int, K: int, with_kernels: bool = False):
    """[glue, fan-out, step 0 .. step K-1] of the last timed round, in milliseconds; with_kernels (contexts served by
    the fused pass) appends the K durations of the fused kernel alone."""
    n = 2 * K + 2 if with_kernels else K + 2
    buf = (C.c_float * n)()
    _check(lib.ssd_ctx_read_timing(ctx, buf, n))
    return list(buf)


def ssd_ctx_enable_phase_clocks(ctx: int, on: bool) -> None:
    _check(lib.ssd_ctx_enable_phase_clocks(ctx, 1 if on else 0))


def ssd_ctx_read_phase_clocks(ctx: int) -> np.ndarray:
    """uint64 [phases][8][workgroups] ticks (100 MHz) of the most recent fused pass; synchronises the device."""
    cap = 1 << 20
    buf = np.zeros(cap, dtype=np.uint64)
    n_ph, n_wg = C.c_int32(), C.c_int32()
    _check(lib.ssd_ctx_read_phase_clocks(ctx, buf.ctypes.data_as(C.c_void_p), cap, C.byref(n_ph), C.byref(n_wg)))
    return buf[: n_ph.value * 8 * n_wg.value].reshape(n_ph.value, 8, n_wg.value)


def ssd_ctx_views(ctx: int) -> ssd_views:
    v = ssd_views()
    _check(lib.ssd_ctx_views(ctx, C.byref(v)))
    return v


def _read_ragged_cache(v: ssd_views, fan: List[int], with_logits: bool) -> Dict[str, torch.Tensor]:
    """Cache of a context whose fan-out differs per accept length, spread out to [B][K+1][max F_k] (unused
    entries: key -1, everything else zero)."""
    B, K, F, V, d = v.batch, v.K, v.F, v.vocab, v.d_model
    R = sum(fan)
    flat = {
        "keys": device_copy(v.d_keys, (B, R), torch.int32),
        "tokens": device_copy(v.d_tokens, (B, R, K), torch.int32),
        "hidden": device_copy(v.d_hidden, (B, R, K, d), torch.float32),
    }
    if with_logits:
        flat["logits"] = device_copy(v.d_logits, (B, R, K, V), torch.float32)
    out = {
        "trunk_len": device_copy(v.d_trunk_len, (B,), torch.int32),
        "glue_hidden": device_copy(v.d_glue_hidden, (B, K + 1, d), torch.float32),
        "glue_logits": device_copy(v.d_glue_logits, (B, K + 1, V), torch.float32),
    }
    for name, t in flat.items():
        wide = torch.zeros((B, K + 1, F) + tuple(t.shape[2:]), dtype=t.dtype, device=t.device)
        if name == "keys":
            wide.fill_(-1)
        off = 0
        for k, f in enumerate(fan):
            wide[:, k, :f] = t[:, off:off + f]
            off += f
        out[name] = wide
    torch.cuda.synchronize()
    return out


def read_cache(ctx: int, with_logits: bool = True) -> Dict[str, torch.Tensor]:
    """Copies of the speculation cache and glue outputs as tensors (test/read-out helper)."""
    v = ssd_ctx_views(ctx)
    B, K, F, V, d = v.batch, v.K, v.F, v.vocab, v.d_model
    fan = ssd_ctx_fanout(ctx)
    if len(set(fan)) > 1:
        return _read_ragged_cache(v, fan, with_logits)
    out = {
        "trunk_len": device_copy(v.d_trunk_len, (B,), torch.int32),
        "keys": device_copy(v.d_keys, (B, K + 1, F), torch.int32),
        "tokens": device_copy(v.d_tokens, (B, K + 1, F, K), torch.int32),
        "hidden": device_copy(v.d_hidden, (B, K + 1, F, K, d), torch.float32),
        "glue_hidden": device_copy(v.d_glue_hidden, (B, K + 1, d), torch.float32),
        "glue_logits": device_copy(v.d_glue_logits, (B, K + 1, V), torch.float32),
    }
    if with_logits:
        out["logits"] = device_copy(v.d_logits, (B, K + 1, F, K, V), torch.float32)
    torch.cuda.synchronize()
    return out
