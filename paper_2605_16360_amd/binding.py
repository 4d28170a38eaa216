"""ctypes binding of libproxykv.so: same names as the C ABI (include/proxykv.h), argument
marshalling only.  Tensors are torch tensors used as device memory; every step of the path runs
in the library's HIP kernels.  There is no fallback: a missing library raises."""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libproxykv.so")

PROXYKV_OK, PROXYKV_EINVAL, PROXYKV_EUNSUPPORTED, PROXYKV_ENOMEM, PROXYKV_ESTATE, PROXYKV_EHIP, PROXYKV_ELIMIT = 0, -1, -2, -3, -4, -5, -6
PROXYKV_BF16, PROXYKV_FP32 = 0, 1
PROXYKV_REDUCE_MAX, PROXYKV_REDUCE_SUM = 0, 1

EXPORTS = [
    "proxykv_default_mapper", "proxykv_create", "proxykv_destroy", "proxykv_mapper_weight_count",
    "proxykv_set_mapper_weights", "proxykv_workspace_bytes", "proxykv_reserve", "proxykv_keep_count",
    "proxykv_layer_pairing", "proxykv_score", "proxykv_score_self", "proxykv_map", "proxykv_topk", "proxykv_topk_static",
    "proxykv_topk_static_limit", "proxykv_compact", "proxykv_compact_inplace",
    "proxykv_mask", "proxykv_topk_pooled", "proxykv_compact_pooled", "proxykv_prune", "proxykv_set_fused_select",
    "proxykv_profile_enable", "proxykv_profile_read", "proxykv_strerror", "proxykv_last_hip_error",
]
STAGES = ("score_lse", "score_colmax", "map", "topk", "compact")


class proxykv_config(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "L_s", "H_q", "H_kv", "d", "L_l", "H_l", "D",
        "d_time", "c_mid", "n_enc_layers", "n_enc_heads", "d_ffn", "d_head_x", "win", "stride", "reduce", "device")]


class ProxyKVError(RuntimeError):
    def __init__(self, status: int, where: str, hip_error: int = 0):
        self.status = status
        self.hip_error = hip_error
        msg = f"{where}: {strerror(status)} (status {status}"
        msg += f", hipError {hip_error})" if hip_error else ")"
        super().__init__(msg)


_lib = None


def load() -> ctypes.CDLL:
    """Loads the in-tree library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2605_16360_amd.build` "
                           "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, f64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_double, ctypes.c_size_t
    cfgp = ctypes.POINTER(proxykv_config)
    lib.proxykv_default_mapper.argtypes = [cfgp]; lib.proxykv_default_mapper.restype = None
    lib.proxykv_create.argtypes = [ctypes.POINTER(vp), cfgp]
    lib.proxykv_destroy.argtypes = [vp]
    lib.proxykv_mapper_weight_count.argtypes = [cfgp]; lib.proxykv_mapper_weight_count.restype = sz
    lib.proxykv_set_mapper_weights.argtypes = [vp, vp, sz]
    lib.proxykv_workspace_bytes.argtypes = [cfgp, i64, i64, ctypes.POINTER(sz)]
    lib.proxykv_reserve.argtypes = [vp, i64, i64]
    lib.proxykv_keep_count.argtypes = [i64, f64, ctypes.POINTER(i64)]
    lib.proxykv_layer_pairing.argtypes = [cfgp, ctypes.POINTER(i32)]
    lib.proxykv_score.argtypes = [vp, vp, vp, vp, i32, i64, i64, i32, vp, vp]
    lib.proxykv_score_self.argtypes = [vp, vp, vp, i32, i64, vp, vp]
    lib.proxykv_map.argtypes = [vp, vp, i64, vp, vp]
    lib.proxykv_topk.argtypes = [vp, vp, i64, i64, i64, vp, vp]
    lib.proxykv_topk_static.argtypes = [vp, vp, i64, i64, i64, vp, vp]
    lib.proxykv_topk_static_limit.argtypes = []; lib.proxykv_topk_static_limit.restype = sz
    lib.proxykv_compact.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, vp, vp, vp]
    lib.proxykv_compact_inplace.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, vp]
    lib.proxykv_mask.argtypes = [vp, vp, i64, i64, i64, vp, vp]
    lib.proxykv_topk_pooled.argtypes = [vp, vp, i64, i64, i64, i64, vp, vp, vp]
    lib.proxykv_compact_pooled.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, vp]
    lib.proxykv_prune.argtypes = [vp, vp, vp, vp, i32, i64, i64, i32, f64, vp, vp, vp, vp, vp, vp, vp,
                                  ctypes.POINTER(i64), vp]
    lib.proxykv_set_fused_select.argtypes = [vp, ctypes.c_int]
    lib.proxykv_profile_enable.argtypes = [vp, ctypes.c_int]
    lib.proxykv_profile_read.argtypes = [vp, ctypes.POINTER(ctypes.c_float)]
    lib.proxykv_strerror.argtypes = [ctypes.c_int]; lib.proxykv_strerror.restype = ctypes.c_char_p
    lib.proxykv_last_hip_error.argtypes = [vp]
    _lib = lib
    return lib


def strerror(status: int) -> str:
    return load().proxykv_strerror(int(status)).decode()


def _check(status: int, where: str, ctx=None) -> None:
    if status != PROXYKV_OK:
        hip = load().proxykv_last_hip_error(ctx) if ctx else 0
        raise ProxyKVError(status, where, hip)


def make_config(L_s: int, H_q: int, H_kv: int, d: int, L_l: int, H_l: int, D: int, device: int = 0,
                **mapper) -> proxykv_config:
    cfg = proxykv_config()
    cfg.L_s, cfg.H_q, cfg.H_kv, cfg.d, cfg.L_l, cfg.H_l, cfg.D = L_s, H_q, H_kv, d, L_l, H_l, D
    load().proxykv_default_mapper(ctypes.byref(cfg))
    cfg.device = device
    for k, v in mapper.items():
        setattr(cfg, k, v)
    return cfg


def config_for_case(case, device: int = 0) -> proxykv_config:
    return make_config(case.L_s, case.H_q, case.H_kv, case.d, case.L_l, case.H_l, case.D, device)


# ---- weight blob ------------------------------------------------------------------------------

def weight_names(cfg: proxykv_config) -> Sequence[str]:
    """Tensor names in blob order (the order documented in include/proxykv.h)."""
    names = ["stem.conv1.weight", "stem.conv1.bias", "stem.bn1.gamma", "stem.bn1.beta", "stem.bn1.mean", "stem.bn1.var",
             "stem.conv2.weight", "stem.conv2.bias", "stem.bn2.gamma", "stem.bn2.beta", "stem.bn2.mean", "stem.bn2.var"]
    for i in range(cfg.n_enc_layers):
        p = f"enc.{i}."
        names += [p + s for s in ("in_proj.weight", "in_proj.bias", "out_proj.weight", "out_proj.bias", "ln1.gamma",
                                  "ln1.beta", "ffn1.weight", "ffn1.bias", "ffn2.weight", "ffn2.bias", "ln2.gamma",
                                  "ln2.beta")]
    names += ["head.k_proj.weight", "head.k_proj.bias", "head.v_proj.weight", "head.v_proj.bias", "head.queries",
              "head.out.weight", "head.out.bias"]
    return names


def pack_mapper_weights(cfg: proxykv_config, weights: Dict[str, torch.Tensor]) -> np.ndarray:
    parts = [weights[n].detach().to(torch.float32).cpu().contiguous().numpy().ravel() for n in weight_names(cfg)]
    return np.ascontiguousarray(np.concatenate(parts), dtype=np.float32)


# ---- entry points -----------------------------------------------------------------------------

class Context:
    """Owns a proxykv_ctx*; destroyed with close() or garbage collection."""

    def __init__(self, cfg: proxykv_config):
        self.cfg = cfg
        self.handle = ctypes.c_void_p()
        _check(load().proxykv_create(ctypes.byref(self.handle), ctypes.byref(cfg)), "proxykv_create")

    def close(self):
        if getattr(self, "handle", None) and self.handle.value:
            load().proxykv_destroy(self.handle)
            self.handle = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def proxykv_create(cfg: proxykv_config) -> Context:
    return Context(cfg)


def proxykv_destroy(ctx: Context) -> None:
    ctx.close()


def proxykv_mapper_weight_count(cfg: proxykv_config) -> int:
    return int(load().proxykv_mapper_weight_count(ctypes.byref(cfg)))


def proxykv_set_mapper_weights(ctx: Context, weights) -> None:
    blob = weights if isinstance(weights, np.ndarray) else pack_mapper_weights(ctx.cfg, weights)
    blob = np.ascontiguousarray(blob, dtype=np.float32)
    _check(load().proxykv_set_mapper_weights(ctx.handle, blob.ctypes.data_as(ctypes.c_void_p), blob.size),
           "proxykv_set_mapper_weights", ctx.handle)


def proxykv_workspace_bytes(cfg: proxykv_config, N: int, N_q: int) -> int:
    out = ctypes.c_size_t()
    _check(load().proxykv_workspace_bytes(ctypes.byref(cfg), N, N_q, ctypes.byref(out)), "proxykv_workspace_bytes")
    return int(out.value)


def proxykv_reserve(ctx: Context, N: int, N_q: int) -> None:
    _check(load().proxykv_reserve(ctx.handle, N, N_q), "proxykv_reserve", ctx.handle)


def proxykv_keep_count(N: int, keep_ratio: float) -> int:
    out = ctypes.c_int64()
    _check(load().proxykv_keep_count(N, float(keep_ratio), ctypes.byref(out)), "proxykv_keep_count")
    return int(out.value)


def proxykv_layer_pairing(cfg: proxykv_config):
    arr = (ctypes.c_int32 * cfg.L_l)()
    _check(load().proxykv_layer_pairing(ctypes.byref(cfg), arr), "proxykv_layer_pairing")
    return list(arr)


def proxykv_set_fused_select(ctx: Context, on: bool) -> None:
    _check(load().proxykv_set_fused_select(ctx.handle, int(bool(on))), "proxykv_set_fused_select", ctx.handle)


def proxykv_profile_enable(ctx: Context, on: bool) -> None:
    _check(load().proxykv_profile_enable(ctx.handle, int(bool(on))), "proxykv_profile_enable", ctx.handle)


def proxykv_profile_read(ctx: Context) -> Dict[str, float]:
    """Stage durations (ms) of the most recent proxykv_prune; waits for it to finish."""
    ms = (ctypes.c_float * len(STAGES))()
    _check(load().proxykv_profile_read(ctx.handle, ms), "proxykv_profile_read", ctx.handle)
    return dict(zip(STAGES, (float(v) for v in ms)))


def _dev_ptr(t: Optional[torch.Tensor], name: str, dtype=None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must have dtype {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def _qk_dtype(q: torch.Tensor) -> int:
    if q.dtype == torch.bfloat16:
        return PROXYKV_BF16
    if q.dtype == torch.float32:
        return PROXYKV_FP32
    raise ValueError("proxy Q/K must be bf16 or fp32")


def proxykv_score(ctx: Context, q_rec, k_ctx, k_rec, chunk: int, x_out=None, stream=None) -> torch.Tensor:
    c = ctx.cfg
    N, N_q = k_ctx.shape[2], q_rec.shape[2]
    assert q_rec.shape == (c.L_s, c.H_q, N_q, c.d) and k_ctx.shape == (c.L_s, c.H_kv, N, c.d)
    assert k_rec.shape == (c.L_s, c.H_kv, N_q, c.d) and k_ctx.dtype == q_rec.dtype == k_rec.dtype
    if x_out is None:
        x_out = torch.empty(c.L_s, c.H_kv, N, dtype=torch.float32, device=q_rec.device)
    _check(load().proxykv_score(ctx.handle, _dev_ptr(q_rec, "q_rec"), _dev_ptr(k_ctx, "k_ctx"), _dev_ptr(k_rec, "k_rec"),
                                _qk_dtype(q_rec), N, N_q, chunk, _dev_ptr(x_out, "x_out", torch.float32),
                                _stream_ptr(stream)), "proxykv_score", ctx.handle)
    return x_out


def proxykv_score_self(ctx: Context, q, k, x_out=None, stream=None) -> torch.Tensor:
    """Causal self-attention probabilities summed over the query axis: q [L_s, H_q, N, d], k [L_s, H_kv, N, d]."""
    c = ctx.cfg
    N = q.shape[2]
    assert q.shape == (c.L_s, c.H_q, N, c.d) and k.shape == (c.L_s, c.H_kv, N, c.d) and q.dtype == k.dtype
    if x_out is None:
        x_out = torch.empty(c.L_s, c.H_kv, N, dtype=torch.float32, device=q.device)
    _check(load().proxykv_score_self(ctx.handle, _dev_ptr(q, "q"), _dev_ptr(k, "k"), _qk_dtype(q), N,
                                     _dev_ptr(x_out, "x_out", torch.float32), _stream_ptr(stream)), "proxykv_score_self", ctx.handle)
    return x_out


def proxykv_map(ctx: Context, x, yhat=None, stream=None) -> torch.Tensor:
    c = ctx.cfg
    N = x.shape[2]
    assert x.shape == (c.L_s, c.H_kv, N)
    if yhat is None:
        yhat = torch.empty(c.L_l, c.H_l, N, dtype=torch.float32, device=x.device)
    _check(load().proxykv_map(ctx.handle, _dev_ptr(x, "x", torch.float32), N, _dev_ptr(yhat, "yhat", torch.float32),
                              _stream_ptr(stream)), "proxykv_map", ctx.handle)
    return yhat


def proxykv_topk(ctx: Context, scores, K: int, idx_out=None, stream=None) -> torch.Tensor:
    N = scores.shape[-1]
    rows = scores.numel() // N
    if idx_out is None:
        idx_out = torch.empty(*scores.shape[:-1], K, dtype=torch.int32, device=scores.device)
    _check(load().proxykv_topk(ctx.handle, _dev_ptr(scores, "scores", torch.float32), rows, N, K,
                               _dev_ptr(idx_out, "idx_out", torch.int32), _stream_ptr(stream)), "proxykv_topk", ctx.handle)
    return idx_out


def proxykv_topk_static_limit() -> int:
    return int(load().proxykv_topk_static_limit())


def proxykv_topk_static(ctx: Context, scores, K: int, idx_out, stream=None) -> torch.Tensor:
    """proxykv_topk without any allocation: idx_out must be passed in; the library's scratch is a fixed device array."""
    N = scores.shape[-1]
    rows = scores.numel() // N
    _check(load().proxykv_topk_static(ctx.handle, _dev_ptr(scores, "scores", torch.float32), rows, N, K,
                                      _dev_ptr(idx_out, "idx_out", torch.int32), _stream_ptr(stream)), "proxykv_topk_static", ctx.handle)
    return idx_out


def proxykv_compact(ctx: Context, k_in, v_in, idx, k_out=None, v_out=None, stream=None):
    N, D = k_in.shape[-2], k_in.shape[-1]
    K = idx.shape[-1]
    rows = idx.numel() // K
    assert k_in.shape == v_in.shape and k_in.numel() == rows * N * D and k_in.element_size() == 2
    if k_out is None:
        k_out = torch.empty(*k_in.shape[:-2], K, D, dtype=k_in.dtype, device=k_in.device)
    if v_out is None:
        v_out = torch.empty_like(k_out)
    _check(load().proxykv_compact(ctx.handle, _dev_ptr(k_in, "k_in"), _dev_ptr(v_in, "v_in"),
                                  _dev_ptr(idx, "idx", torch.int32), rows, N, K, D, _dev_ptr(k_out, "k_out"),
                                  _dev_ptr(v_out, "v_out"), _stream_ptr(stream)), "proxykv_compact", ctx.handle)
    return k_out, v_out


def proxykv_compact_inplace(ctx: Context, k, v, idx, stream=None) -> None:
    """k, v [..., N, D] are compacted where they lie: tokens 0 .. K-1 of every row become the kept tokens."""
    N, D = k.shape[-2], k.shape[-1]
    K = idx.shape[-1]
    rows = idx.numel() // K
    assert k.shape == v.shape and k.numel() == rows * N * D and k.element_size() == 2
    _check(load().proxykv_compact_inplace(ctx.handle, _dev_ptr(k, "k"), _dev_ptr(v, "v"), _dev_ptr(idx, "idx", torch.int32),
                                          rows, N, K, D, _stream_ptr(stream)), "proxykv_compact_inplace", ctx.handle)


def proxykv_mask(ctx: Context, idx, N: int, mask_out=None, stream=None) -> torch.Tensor:
    K = idx.shape[-1]
    rows = idx.numel() // K
    if mask_out is None:
        mask_out = torch.empty(*idx.shape[:-1], N, dtype=torch.uint8, device=idx.device)
    _check(load().proxykv_mask(ctx.handle, _dev_ptr(idx, "idx", torch.int32), rows, N, K, _dev_ptr(mask_out, "mask_out", torch.uint8),
                               _stream_ptr(stream)), "proxykv_mask", ctx.handle)
    return mask_out


def proxykv_topk_pooled(ctx: Context, scores, K: int, flat_out=None, counts_out=None, stream=None):
    """scores [layers, heads, N]; one budget of heads*K per layer.  Returns (flat [layers, heads*K], counts [layers, heads])."""
    layers, heads, N = scores.shape
    if flat_out is None:
        flat_out = torch.empty(layers, heads * K, dtype=torch.int32, device=scores.device)
    if counts_out is None:
        counts_out = torch.empty(layers, heads, dtype=torch.int32, device=scores.device)
    _check(load().proxykv_topk_pooled(ctx.handle, _dev_ptr(scores, "scores", torch.float32), layers, heads, N, K,
                                      _dev_ptr(flat_out, "flat_out", torch.int32), _dev_ptr(counts_out, "counts_out", torch.int32),
                                      _stream_ptr(stream)), "proxykv_topk_pooled", ctx.handle)
    return flat_out, counts_out


def proxykv_compact_pooled(ctx: Context, k, v, flat, counts, stream=None) -> None:
    """k, v [layers, heads, N, D] compacted where they lie with the ragged lists of proxykv_topk_pooled."""
    layers, heads, N, D = k.shape
    K = flat.shape[-1] // heads
    assert k.shape == v.shape and k.element_size() == 2 and flat.shape == (layers, heads * K) and counts.shape == (layers, heads)
    _check(load().proxykv_compact_pooled(ctx.handle, _dev_ptr(k, "k"), _dev_ptr(v, "v"), _dev_ptr(flat, "flat", torch.int32),
                                         _dev_ptr(counts, "counts", torch.int32), layers, heads, N, K, D, _stream_ptr(stream)),
           "proxykv_compact_pooled", ctx.handle)


def proxykv_prune(ctx: Context, q_rec, k_ctx, k_rec, chunk: int, keep_ratio: float, k_in, v_in, k_out=None, v_out=None,
                  idx_out=None, x_out=None, yhat_out=None, stream=None):
    """Returns (k_out, v_out, idx_out, K)."""
    c = ctx.cfg
    N, N_q = k_ctx.shape[2], q_rec.shape[2]
    K = proxykv_keep_count(N, keep_ratio)
    dev = k_in.device
    if k_out is None:
        k_out = torch.empty(c.L_l, c.H_l, K, c.D, dtype=k_in.dtype, device=dev)
    if v_out is None:
        v_out = torch.empty_like(k_out)
    if idx_out is None:
        idx_out = torch.empty(c.L_l, c.H_l, K, dtype=torch.int32, device=dev)
    K_host = ctypes.c_int64()
    _check(load().proxykv_prune(ctx.handle, _dev_ptr(q_rec, "q_rec"), _dev_ptr(k_ctx, "k_ctx"), _dev_ptr(k_rec, "k_rec"),
                                _qk_dtype(q_rec), N, N_q, chunk, float(keep_ratio), _dev_ptr(k_in, "k_in"),
                                _dev_ptr(v_in, "v_in"), _dev_ptr(k_out, "k_out"), _dev_ptr(v_out, "v_out"),
                                _dev_ptr(idx_out, "idx_out", torch.int32), _dev_ptr(x_out, "x_out", torch.float32),
                                _dev_ptr(yhat_out, "yhat_out", torch.float32), ctypes.byref(K_host),
                                _stream_ptr(stream)), "proxykv_prune", ctx.handle)
    assert K_host.value == K
    return k_out, v_out, idx_out, K
