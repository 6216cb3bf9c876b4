"""Thin ctypes binding of libvismoe.so: same entry points, same names, argument marshalling only.

Every step of the layer runs in the HIP kernels behind the C-ABI (include/moe.h); this module converts torch
tensors to device pointers, passes the current HIP stream and turns a non-zero status into an exception.
There is no fallback: importing this module without the built library raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libvismoe.so")
if not os.path.exists(_LIB_PATH):
    raise ImportError(f"{_LIB_PATH} is missing: build it first (python -m paper_2605_05899_amd.build); "
                      "there is no CPU or PyTorch fallback for the MoE layer")
# torch first: it ships its own HIP runtime, and the library must bind to that same runtime (the one that owns
# the tensors' memory and streams) instead of pulling a second copy into the process.
import torch  # noqa: E402,F401

_lib = ctypes.CDLL(_LIB_PATH)

(MOE_OK, MOE_ERR_NULL, MOE_ERR_SHAPE, MOE_ERR_ALIGN, MOE_ERR_WORKSPACE, MOE_ERR_UNSUPPORTED, MOE_ERR_HIP,
 MOE_ERR_INDEX, MOE_ERR_CACHE_FULL) = range(9)

EXPORTS = ("moe_workspace_bytes", "moe_status_string", "moe_route", "moe_dispatch", "moe_expert_ffn",
           "moe_shared_ffn", "moe_combine", "moe_layer_forward", "moe_stage_timing_enable", "moe_stage_timing_read",
           "moe_compress_workspace_bytes", "moe_token_compress", "moe_expert_ffn_slabs", "moe_mean_pool_workspace_bytes",
           "moe_mean_pool", "moe_routing_histogram", "moe_lookahead_target", "moe_cache_create", "moe_cache_destroy",
           "moe_cache_predict", "moe_cache_acquire", "moe_cache_layer_done", "moe_cache_query", "moe_cache_stats",
           "moe_predictor_workspace_bytes", "moe_predictor_forward", "moe_index_checks_enable",
           "moe_static_scratch_bytes", "moe_layer_forward_static", "moe_compress_wide_min_tokens")
N_STAGES = 5
STAGE_NAMES = ("route", "dispatch", "gate_up_swiglu", "down", "combine")


class _CConfig(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("H", "I", "E", "k", "S", "norm_topk", "max_tokens")]


@dataclass(frozen=True)
class MoEConfig:
    """Mirror of the C struct moe_config."""
    H: int
    I: int
    E: int
    k: int
    S: int = 0
    norm_topk: int = 1
    max_tokens: int = 0

    def c(self) -> _CConfig:
        return _CConfig(self.H, self.I, self.E, self.k, self.S, self.norm_topk, self.max_tokens)


class MoEError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({moe_status_string(status)})")


_P, _I32 = ctypes.c_void_p, ctypes.c_int32
_CFG = ctypes.POINTER(_CConfig)
_lib.moe_workspace_bytes.restype = ctypes.c_size_t
_lib.moe_workspace_bytes.argtypes = [_CFG]
_lib.moe_status_string.restype = ctypes.c_char_p
_lib.moe_status_string.argtypes = [ctypes.c_int]
_lib.moe_route.restype = ctypes.c_int
_lib.moe_route.argtypes = [_CFG, _P, _I32, _P, _I32, _P, _P, _P, _P, _P]
_lib.moe_dispatch.restype = ctypes.c_int
_lib.moe_dispatch.argtypes = [_CFG, _P, _I32, _P, _P, _P, _P, _P]
_lib.moe_expert_ffn.restype = ctypes.c_int
_lib.moe_expert_ffn.argtypes = [_CFG, _P, _I32, _P, _I32, _P, _P, _P, _P, _P, _P, _P, _P]
_lib.moe_expert_ffn_slabs.restype = ctypes.c_int
_lib.moe_expert_ffn_slabs.argtypes = [_CFG, _P, _I32, _P, _I32, _P, _P, _P, _P, _P, _P, _P]
_lib.moe_shared_ffn.restype = ctypes.c_int
_lib.moe_shared_ffn.argtypes = [_CFG, _P, _I32, _P, _I32, _P, _P, _P, _P, _P, _P]
_lib.moe_combine.restype = ctypes.c_int
_lib.moe_combine.argtypes = [_CFG, _P, _P, _P, _I32, _P, _P, _P]
_lib.moe_layer_forward.restype = ctypes.c_int
_lib.moe_layer_forward.argtypes = [_CFG, _P, _I32, _P, _I32] + [_P] * 12
_lib.moe_layer_forward_static.restype = ctypes.c_int
_lib.moe_layer_forward_static.argtypes = [_CFG, _P, _I32, _P, _I32] + [_P] * 11
_lib.moe_static_scratch_bytes.restype = ctypes.c_size_t
_lib.moe_static_scratch_bytes.argtypes = []
_lib.moe_compress_wide_min_tokens.restype = ctypes.c_int32
_lib.moe_compress_wide_min_tokens.argtypes = [_I32]
_lib.moe_compress_workspace_bytes.restype = ctypes.c_size_t
_lib.moe_compress_workspace_bytes.argtypes = [_I32, _I32]
_lib.moe_token_compress.restype = ctypes.c_int
_lib.moe_token_compress.argtypes = [_P, _I32, _I32, _P, _I32, _I32, _I32, ctypes.c_double, ctypes.c_double, ctypes.c_float,
                                    _P, _P, _P, _P, _P]
_lib.moe_mean_pool_workspace_bytes.restype = ctypes.c_size_t
_lib.moe_mean_pool_workspace_bytes.argtypes = [_I32]
_lib.moe_mean_pool.restype = ctypes.c_int
_lib.moe_mean_pool.argtypes = [_P, _I32, _I32, _P, _I32, _P, _P, _P]
_lib.moe_routing_histogram.restype = ctypes.c_int
_lib.moe_routing_histogram.argtypes = [_P, ctypes.c_int64, _I32, _P, _P]
_lib.moe_lookahead_target.restype = ctypes.c_int
_lib.moe_lookahead_target.argtypes = [_P, _I32, ctypes.c_int64, _I32, ctypes.c_float, _P, _P]
_lib.moe_predictor_workspace_bytes.restype = ctypes.c_size_t
_lib.moe_predictor_workspace_bytes.argtypes = [_I32, _I32]
_lib.moe_predictor_forward.restype = ctypes.c_int
_lib.moe_predictor_forward.argtypes = [_P, _I32, _P, _P, _P, _I32, _P, _P, _P, _I32, _P, _I32, _I32, _P, _P, _P, _P]
_lib.moe_cache_create.restype = ctypes.c_int
_lib.moe_cache_create.argtypes = [_I32, _I32, ctypes.c_size_t, _I32, _P, ctypes.POINTER(ctypes.c_void_p)]
_lib.moe_cache_destroy.restype = None
_lib.moe_cache_destroy.argtypes = [_P]
_lib.moe_cache_predict.restype = ctypes.c_int
_lib.moe_cache_predict.argtypes = [_P, _P, _P, _P, _I32, _P, _P, _P, ctypes.POINTER(ctypes.c_int32)]
_lib.moe_cache_acquire.restype = ctypes.c_int
_lib.moe_cache_acquire.argtypes = [_P, _I32, _P, _I32, _P, _P, _P, _P, _P, ctypes.POINTER(ctypes.c_int32)]
_lib.moe_cache_layer_done.restype = ctypes.c_int
_lib.moe_cache_layer_done.argtypes = [_P, _I32, _P]
_lib.moe_cache_query.restype = ctypes.c_int
_lib.moe_cache_query.argtypes = [_P, _I32, _I32, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32),
                                 ctypes.POINTER(ctypes.c_float)]
_lib.moe_cache_stats.restype = ctypes.c_int
_lib.moe_cache_stats.argtypes = [_P, ctypes.POINTER(ctypes.c_int64)]
_lib.moe_stage_timing_enable.restype = ctypes.c_int
_lib.moe_stage_timing_enable.argtypes = [_I32]
_lib.moe_index_checks_enable.restype = ctypes.c_int
_lib.moe_index_checks_enable.argtypes = [_I32]
_lib.moe_stage_timing_read.restype = ctypes.c_int
_lib.moe_stage_timing_read.argtypes = [ctypes.POINTER(ctypes.c_float)]


def _ptr(t):
    """Device pointer of a torch tensor; None -> NULL; an int is passed through (tests of the error paths)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("tensors passed to the MoE library must be contiguous")
    return t.data_ptr()


def _stream(stream):
    if stream is not None:
        return stream if isinstance(stream, int) else stream.cuda_stream
    return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None


def _check(status: int, where: str, raise_on_error: bool):
    if status != MOE_OK and raise_on_error:
        raise MoEError(status, where)
    return status


def moe_workspace_bytes(cfg: MoEConfig) -> int:
    return int(_lib.moe_workspace_bytes(ctypes.byref(cfg.c())))


def moe_status_string(status: int) -> str:
    return _lib.moe_status_string(int(status)).decode()


def alloc_workspace(cfg: MoEConfig, device="cuda"):
    """Device buffer for `ws` (torch is used for device memory only)."""
    n = moe_workspace_bytes(cfg)
    if n == 0:
        raise MoEError(MOE_ERR_SHAPE, "moe_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def moe_route(cfg, x, T_in, keep_idx, T, w_router, topk_ids, topk_w, ws, stream=None, check=True):
    st = _lib.moe_route(ctypes.byref(cfg.c()), _ptr(x), T_in, _ptr(keep_idx), T, _ptr(w_router), _ptr(topk_ids),
                        _ptr(topk_w), _ptr(ws), _stream(stream))
    return _check(st, "moe_route", check)


def moe_dispatch(cfg, topk_ids, T, expert_offsets, sorted_token, inv_perm, ws, stream=None, check=True):
    st = _lib.moe_dispatch(ctypes.byref(cfg.c()), _ptr(topk_ids), T, _ptr(expert_offsets), _ptr(sorted_token),
                           _ptr(inv_perm), _ptr(ws), _stream(stream))
    return _check(st, "moe_dispatch", check)


def moe_expert_ffn(cfg, x, T_in, keep_idx, T, expert_offsets, sorted_token, w_gate, w_up, w_down, y_sorted, ws,
                   stream=None, check=True):
    st = _lib.moe_expert_ffn(ctypes.byref(cfg.c()), _ptr(x), T_in, _ptr(keep_idx), T, _ptr(expert_offsets),
                             _ptr(sorted_token), _ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(y_sorted), _ptr(ws),
                             _stream(stream))
    return _check(st, "moe_expert_ffn", check)


def moe_expert_ffn_slabs(cfg, x, T_in, keep_idx, T, expert_offsets, sorted_token, slab_table, y_sorted, missing, ws,
                         stream=None, check=True):
    """slab_table: int64 device tensor [E] of device addresses (0 = not resident)."""
    st = _lib.moe_expert_ffn_slabs(ctypes.byref(cfg.c()), _ptr(x), T_in, _ptr(keep_idx), T, _ptr(expert_offsets),
                                   _ptr(sorted_token), _ptr(slab_table), _ptr(y_sorted), _ptr(missing), _ptr(ws),
                                   _stream(stream))
    return _check(st, "moe_expert_ffn_slabs", check)


def moe_shared_ffn(cfg, x, T_in, keep_idx, T, ws_gate, ws_up, ws_down, shared_out, ws, stream=None, check=True):
    st = _lib.moe_shared_ffn(ctypes.byref(cfg.c()), _ptr(x), T_in, _ptr(keep_idx), T, _ptr(ws_gate), _ptr(ws_up),
                             _ptr(ws_down), _ptr(shared_out), _ptr(ws), _stream(stream))
    return _check(st, "moe_shared_ffn", check)


def moe_combine(cfg, y_sorted, inv_perm, topk_w, T, shared_out, out, stream=None, check=True):
    st = _lib.moe_combine(ctypes.byref(cfg.c()), _ptr(y_sorted), _ptr(inv_perm), _ptr(topk_w), T, _ptr(shared_out),
                          _ptr(out), _stream(stream))
    return _check(st, "moe_combine", check)


def moe_layer_forward(cfg, x, T_in, keep_idx, T, w_router, w_gate, w_up, w_down, ws_gate, ws_up, ws_down, out,
                      topk_ids_opt, topk_w_opt, ws, stream=None, check=True):
    st = _lib.moe_layer_forward(ctypes.byref(cfg.c()), _ptr(x), T_in, _ptr(keep_idx), T, _ptr(w_router), _ptr(w_gate),
                                _ptr(w_up), _ptr(w_down), _ptr(ws_gate), _ptr(ws_up), _ptr(ws_down), _ptr(out),
                                _ptr(topk_ids_opt), _ptr(topk_w_opt), _ptr(ws), _stream(stream))
    return _check(st, "moe_layer_forward", check)


def moe_static_scratch_bytes() -> int:
    return int(_lib.moe_static_scratch_bytes())


def moe_layer_forward_static(cfg, x, T_in, keep_idx, T, w_router, w_gate, w_up, w_down, ws_gate, ws_up, ws_down, out,
                             topk_ids_opt, topk_w_opt, stream=None, check=True):
    st = _lib.moe_layer_forward_static(ctypes.byref(cfg.c()), _ptr(x), T_in, _ptr(keep_idx), T, _ptr(w_router),
                                       _ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(ws_gate), _ptr(ws_up),
                                       _ptr(ws_down), _ptr(out), _ptr(topk_ids_opt), _ptr(topk_w_opt), _stream(stream))
    return _check(st, "moe_layer_forward_static", check)


def moe_compress_workspace_bytes(N: int, E: int) -> int:
    return int(_lib.moe_compress_workspace_bytes(int(N), int(E)))


def alloc_compress_workspace(N: int, E: int, device="cuda"):
    n = moe_compress_workspace_bytes(N, E)
    if n == 0:
        raise MoEError(MOE_ERR_SHAPE, "moe_compress_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def moe_token_compress(attn, n_heads, N, prefix_topk_ids, L, k, E, alpha, beta, lam, keep_idx, s_norm, delta, ws,
                       stream=None, check=True):
    st = _lib.moe_token_compress(_ptr(attn), n_heads, N, _ptr(prefix_topk_ids), L, k, E, float(alpha), float(beta),
                                 float(lam), _ptr(keep_idx), _ptr(s_norm), _ptr(delta), _ptr(ws), _stream(stream))
    return _check(st, "moe_token_compress", check)


def moe_compress_wide_min_tokens(n: int) -> int:
    return int(_lib.moe_compress_wide_min_tokens(int(n)))


def moe_mean_pool_workspace_bytes(D: int) -> int:
    return int(_lib.moe_mean_pool_workspace_bytes(int(D)))


def moe_mean_pool(rows, n_rows, D, idx, K, out, ws, stream=None, check=True):
    st = _lib.moe_mean_pool(_ptr(rows), n_rows, D, _ptr(idx), K, _ptr(out), _ptr(ws), _stream(stream))
    return _check(st, "moe_mean_pool", check)


def moe_routing_histogram(ids, n, E, out, stream=None, check=True):
    return _check(_lib.moe_routing_histogram(_ptr(ids), int(n), E, _ptr(out), _stream(stream)), "moe_routing_histogram",
                  check)


def moe_lookahead_target(future_ids, W, n, E, gamma, g, stream=None, check=True):
    return _check(_lib.moe_lookahead_target(_ptr(future_ids), W, int(n), E, float(gamma), _ptr(g), _stream(stream)),
                  "moe_lookahead_target", check)


def moe_predictor_workspace_bytes(D1: int, D2: int) -> int:
    return int(_lib.moe_predictor_workspace_bytes(int(D1), int(D2)))


def moe_predictor_forward(x, D, W1, s1, t1, D1, W2, s2, t2, D2, Wo, E, B, y, top, ws, stream=None, check=True):
    st = _lib.moe_predictor_forward(_ptr(x), D, _ptr(W1), _ptr(s1), _ptr(t1), D1, _ptr(W2), _ptr(s2), _ptr(t2), D2,
                                    _ptr(Wo), E, B, _ptr(y), _ptr(top), _ptr(ws), _stream(stream))
    return _check(st, "moe_predictor_forward", check)


class ExpertCache:
    """Argument marshalling for the moe_cache_* calls (the policy and the stream work are in the library).

    pool: uint8 device tensor of n_slabs * slab_bytes bytes. Host images are passed as integer addresses of pinned
    host memory (for a pinned torch tensor t: t.data_ptr())."""
    STAT_NAMES = ("hits", "misses", "prefetches", "evictions", "refused", "bytes_copied")

    def __init__(self, n_layers, E, slab_bytes, n_slabs, pool, check=True):
        self.E, self.pool = E, pool
        h = ctypes.c_void_p()
        st = _lib.moe_cache_create(n_layers, E, slab_bytes, n_slabs, _ptr(pool), ctypes.byref(h))
        self.status = _check(st, "moe_cache_create", check)
        self._h = h if st == MOE_OK else None

    def close(self):
        if self._h is not None:
            _lib.moe_cache_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()

    def predict(self, items, host_addr, trans_stream, check=True):
        """items: [(layer, expert, priority)]; host_addr(layer, expert) -> address of the pinned image.
        Returns the (layer, expert) pairs whose copy was started."""
        n = len(items)
        L = (ctypes.c_int32 * max(n, 1))(*[i[0] for i in items])
        Ex = (ctypes.c_int32 * max(n, 1))(*[i[1] for i in items])
        P = (ctypes.c_float * max(n, 1))(*[i[2] for i in items])
        src = (ctypes.c_void_p * max(n, 1))(*[host_addr(i[0], i[1]) for i in items])
        started = (ctypes.c_int32 * max(2 * n, 1))()
        ns = ctypes.c_int32(0)
        st = _lib.moe_cache_predict(self._h, L, Ex, P, n, src, _stream(trans_stream), started, ctypes.byref(ns))
        _check(st, "moe_cache_predict", check)
        return [(started[2 * i], started[2 * i + 1]) for i in range(ns.value)] if st == MOE_OK else st

    def acquire(self, layer, needed, host_addr, trans_stream, comp_stream, check=True):
        """Returns (table, missed): table = list of E device addresses (0 = not needed), missed = experts fetched on
        demand."""
        n = len(needed)
        N = (ctypes.c_int32 * max(n, 1))(*needed)
        src = (ctypes.c_void_p * max(n, 1))(*[host_addr(layer, e) for e in needed])
        table = (ctypes.c_void_p * self.E)()
        missed = (ctypes.c_int32 * max(n, 1))()
        nm = ctypes.c_int32(0)
        st = _lib.moe_cache_acquire(self._h, layer, N, n, src, _stream(trans_stream), _stream(comp_stream), table, missed,
                                    ctypes.byref(nm))
        _check(st, "moe_cache_acquire", check)
        if st != MOE_OK:
            return st
        return [int(a or 0) for a in table], [missed[i] for i in range(nm.value)]

    def layer_done(self, layer, comp_stream, check=True):
        return _check(_lib.moe_cache_layer_done(self._h, layer, _stream(comp_stream)), "moe_cache_layer_done", check)

    def query(self, layer, expert):
        s, c, p = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_float()
        _check(_lib.moe_cache_query(self._h, layer, expert, ctypes.byref(s), ctypes.byref(c), ctypes.byref(p)),
               "moe_cache_query", True)
        return s.value, c.value, p.value

    def stats(self):
        out = (ctypes.c_int64 * 6)()
        _check(_lib.moe_cache_stats(self._h, out), "moe_cache_stats", True)
        return dict(zip(self.STAT_NAMES, [int(v) for v in out]))


def moe_stage_timing_enable(enable: bool, check=True):
    return _check(_lib.moe_stage_timing_enable(1 if enable else 0), "moe_stage_timing_enable", check)


def moe_index_checks_enable(enable: bool, check=True):
    return _check(_lib.moe_index_checks_enable(1 if enable else 0), "moe_index_checks_enable", check)


def moe_stage_timing_read(check=True):
    """Milliseconds per stage of the last call (waits for that call's events)."""
    buf = (ctypes.c_float * N_STAGES)()
    st = _lib.moe_stage_timing_read(buf)
    _check(st, "moe_stage_timing_read", check)
    return [float(v) for v in buf]
