"""Thin ctypes binding over libdkv.so (argument marshalling only; every step runs in the HIP kernels).

The functions carry the names of the C ABI (include/dkv.h).  torch is used for device memory and streams
only: tensors are passed as raw device pointers, the current torch stream as the hipStream_t.
There is no CPU fallback: a missing library or a failing call raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdkv.so")

DKV_F32, DKV_BF16 = 0, 1
DKV_MAX_SELECT_LAYERS = 32
DKV_MAX_UPDATES = 8
DKV_OK, DKV_ERR_INVALID_ARG, DKV_ERR_UNSUPPORTED, DKV_ERR_WORKSPACE, DKV_ERR_LAUNCH = 0, -1, -2, -3, -4

EXPORTS = ("dkv_version", "dkv_status_string", "dkv_workspace_bytes", "dkv_profile_begin", "dkv_profile_end", "dkv_score_window",
           "dkv_score_window_layers", "dkv_score_window_stats", "dkv_score_window_emit", "dkv_score_window_lse", "dkv_score_window_lse_layers", "dkv_row_lse", "dkv_select_topk", "dkv_select_topk_layers", "dkv_rebalance", "dkv_rebalance_batch",
           "dkv_gather_kv", "dkv_gather_kv_layers", "dkv_pack_cache", "dkv_decode_attention", "dkv_layer_budgets",
           "dkv_apply_budgets", "dkv_select_recent", "dkv_score_window_static", "dkv_static_scratch_limit", "dkv_score_path",
           "dkv_decode_attention_layers")
DKV_SCHEDULE_FIXED, DKV_SCHEDULE_PYRAMID = 0, 1


class dkv_desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "n_q_heads", "n_kv_heads", "head_dim", "window", "pool_kernel",
                                         "layer_max", "mean_budget", "interval", "dtype", "n_seqs", "total_tokens",
                                         "max_seq_len")] + [("softmax_scale", C.c_float), ("row_scale", C.c_float)]


class DkvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _lib.dkv_status_string(status).decode() if _lib is not None else "?"
        super().__init__("%s: %s (%d)" % (where, msg, status))


_lib = None


def load() -> C.CDLL:
    """Load libdkv.so (built by paper_2412_14838_amd.build). Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    import torch  # noqa: F401  (loads the HIP runtime the library is linked against, before the library)
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError("libdkv.so not built: run `python -m paper_2412_14838_amd.build` (%s)" % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    P, I32, I64, SZ = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    D = C.POINTER(dkv_desc)
    lib.dkv_version.restype = C.c_int
    lib.dkv_version.argtypes = []
    lib.dkv_status_string.restype = C.c_char_p
    lib.dkv_status_string.argtypes = [C.c_int]
    lib.dkv_workspace_bytes.restype = SZ
    lib.dkv_workspace_bytes.argtypes = [D]
    lib.dkv_profile_begin.restype = C.c_int
    lib.dkv_profile_begin.argtypes = [I32]
    lib.dkv_profile_end.restype = C.c_int
    lib.dkv_profile_end.argtypes = [P, P, I32]
    for name in ("dkv_score_window", "dkv_score_window_stats", "dkv_score_window_emit"):
        getattr(lib, name).restype = C.c_int
        getattr(lib, name).argtypes = [D, P, P, I64, I64, P, P, I64, P, SZ, P]
    lib.dkv_score_window_layers.restype = C.c_int
    lib.dkv_score_window_layers.argtypes = [D, I32, I32, P, P, I64, I64, P, P, P, SZ, P]
    lib.dkv_score_window_lse.restype = C.c_int
    lib.dkv_score_window_lse.argtypes = [D, P, P, I64, I64, P, P, P, I64, P]
    lib.dkv_score_window_lse_layers.restype = C.c_int
    lib.dkv_score_window_lse_layers.argtypes = [D, I32, I32, P, P, I64, I64, P, P, P, P, SZ, P]
    lib.dkv_row_lse.restype = C.c_int
    lib.dkv_row_lse.argtypes = [D, I64, P, P, P, SZ, P]
    lib.dkv_select_topk.restype = C.c_int
    lib.dkv_select_topk.argtypes = [D, I32, P, I64, P, P, P, P, SZ, P]
    lib.dkv_select_topk_layers.restype = C.c_int
    lib.dkv_select_topk_layers.argtypes = [D, I32, I32, P, P, P, P, P, SZ, P]
    lib.dkv_gather_kv_layers.restype = C.c_int
    lib.dkv_gather_kv_layers.argtypes = [D, I32, I32, P, P, I64, I64, P, P, P, P, P, I64, I64, I64, P]
    lib.dkv_pack_cache.restype = C.c_int
    lib.dkv_pack_cache.argtypes = [D, P, P, P, P, I64, I64, I64, P, P, I64, P, P]
    lib.dkv_decode_attention.restype = C.c_int
    lib.dkv_decode_attention.argtypes = [D, I32, P, P, P, I64, I64, P, P, P, P, P, SZ, P]
    lib.dkv_decode_attention_layers.restype = C.c_int
    lib.dkv_decode_attention_layers.argtypes = [D, I32, I32, P, P, P, I64, I64, I64, P, P, P, P, P, SZ, P]
    lib.dkv_rebalance.restype = C.c_int
    lib.dkv_rebalance.argtypes = [D, I32, C.c_uint32, P, P, P, P, P, P, SZ, P]
    lib.dkv_rebalance_batch.restype = C.c_int
    lib.dkv_rebalance_batch.argtypes = [D, I32, I32, C.c_uint32, P, P, P, P, P, I64, P, SZ, P]
    lib.dkv_gather_kv.restype = C.c_int
    lib.dkv_gather_kv.argtypes = [D, I32, P, P, I64, I64, P, P, P, P, P, I64, I64, P]
    lib.dkv_layer_budgets.restype = C.c_int
    lib.dkv_layer_budgets.argtypes = [D, I32, I32, P]
    lib.dkv_apply_budgets.restype = C.c_int
    lib.dkv_apply_budgets.argtypes = [D, I32, P, P, P]
    lib.dkv_select_recent.restype = C.c_int
    lib.dkv_select_recent.argtypes = [D, I32, I32, P, P, P, P]
    lib.dkv_score_window_static.restype = C.c_int
    lib.dkv_score_window_static.argtypes = [D, P, P, I64, I64, P, P, I64, P]
    lib.dkv_score_path.restype = C.c_int
    lib.dkv_score_path.argtypes = [D, I64]
    lib.dkv_static_scratch_limit.restype = SZ
    lib.dkv_static_scratch_limit.argtypes = []
    _lib = lib
    return lib


def make_desc(*, n_layers, n_q_heads, n_kv_heads, head_dim, window, pool_kernel, layer_max, mean_budget, interval,
              dtype, n_seqs, total_tokens, max_seq_len, softmax_scale=0.0, row_scale=0.0) -> dkv_desc:
    return dkv_desc(n_layers, n_q_heads, n_kv_heads, head_dim, window, pool_kernel, layer_max, mean_budget, interval,
                    dtype, n_seqs, total_tokens, max_seq_len, softmax_scale, row_scale)


def desc_from_workload(cfg, **override) -> dkv_desc:
    kw = dict(n_layers=cfg.L, n_q_heads=cfg.Hq, n_kv_heads=cfg.Hkv, head_dim=cfg.d, window=cfg.w, pool_kernel=cfg.P,
              layer_max=cfg.layer_max, mean_budget=cfg.mean_budget, interval=cfg.interval,
              dtype=DKV_BF16 if cfg.dtype == "bf16" else DKV_F32, n_seqs=cfg.n_seqs, total_tokens=cfg.total_tokens,
              max_seq_len=max(cfg.seqlens))
    kw.update(override)
    return make_desc(**kw)


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _check(status: int, where: str) -> None:
    if status != DKV_OK:
        raise DkvError(status, where)


def dkv_version() -> int:
    return load().dkv_version()


def dkv_status_string(status: int) -> str:
    return load().dkv_status_string(status).decode()


def dkv_workspace_bytes(desc: dkv_desc) -> int:
    return int(load().dkv_workspace_bytes(C.byref(desc)))


KERNEL_NAMES = ("score_stats", "score_emit", "select", "gather", "rebalance_hist", "rebalance_scan",
                "rebalance_final", "fill", "score_borders", "score_lse", "pack", "decode", "score_merge", "rebalance_pick",
                "schedule")


def dkv_profile_begin(capacity: int) -> None:
    _check(load().dkv_profile_begin(capacity), "dkv_profile_begin")


def dkv_profile_end(capacity: int):
    """Returns [(kernel name, microseconds)] of the launches recorded since dkv_profile_begin, in launch order."""
    ids = (C.c_int32 * capacity)()
    us = (C.c_float * capacity)()
    n = load().dkv_profile_end(ids, us, capacity)
    if n < 0:
        raise DkvError(n, "dkv_profile_end")
    return [(KERNEL_NAMES[ids[i]], float(us[i])) for i in range(min(n, capacity))]


def dkv_score_window(desc, q_win, k, k_stride_token, k_stride_head, cu_seqlens, scores_out, scores_stride_head,
                     workspace, stream=None) -> None:
    _check(load().dkv_score_window(C.byref(desc), _ptr(q_win), _ptr(k), k_stride_token, k_stride_head, _ptr(cu_seqlens),
                                   _ptr(scores_out), scores_stride_head, _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), _stream(stream)), "dkv_score_window")


def dkv_score_window_static(desc, q_win, k, k_stride_token, k_stride_head, cu_seqlens, scores_out, scores_stride_head,
                            stream=None) -> None:
    _check(load().dkv_score_window_static(C.byref(desc), _ptr(q_win), _ptr(k), k_stride_token, k_stride_head,
                                          _ptr(cu_seqlens), _ptr(scores_out), scores_stride_head, _stream(stream)),
           "dkv_score_window_static")


def dkv_static_scratch_limit() -> int:
    return int(load().dkv_static_scratch_limit())


def dkv_layer_budgets(desc, schedule, beta=4):
    """The L budgets of a fixed-pattern schedule as a list of ints (host only)."""
    out = (C.c_int32 * desc.n_layers)()
    _check(load().dkv_layer_budgets(C.byref(desc), schedule, beta, out), "dkv_layer_budgets")
    return list(out)


def dkv_apply_budgets(desc, n_layers, budgets, counts, stream=None) -> None:
    _check(load().dkv_apply_budgets(C.byref(desc), n_layers, _ptr(budgets), _ptr(counts), _stream(stream)),
           "dkv_apply_budgets")


def dkv_select_recent(desc, layer, n_sink, cu_seqlens, idx_out, counts, stream=None) -> None:
    _check(load().dkv_select_recent(C.byref(desc), layer, n_sink, _ptr(cu_seqlens), _ptr(idx_out), _ptr(counts),
                                    _stream(stream)), "dkv_select_recent")


def dkv_score_window_layers(desc, layer_begin, q_layers, k_layers, k_stride_token, k_stride_head, cu_seqlens, scores_all,
                            workspace, stream=None) -> None:
    """q_layers, k_layers: sequences of device tensors, one per layer of the call."""
    n = len(k_layers)
    qs = (C.c_void_p * n)(*[t.data_ptr() for t in q_layers])
    ks = (C.c_void_p * n)(*[t.data_ptr() for t in k_layers])
    _check(load().dkv_score_window_layers(C.byref(desc), layer_begin, n, qs, ks, k_stride_token, k_stride_head,
                                          _ptr(cu_seqlens), _ptr(scores_all), _ptr(workspace),
                                          workspace.numel() * workspace.element_size(), _stream(stream)),
           "dkv_score_window_layers")


def dkv_score_window_lse_layers(desc, layer_begin, q_layers, k_layers, k_stride_token, k_stride_head, cu_seqlens,
                                lse_layers, scores_all, workspace, stream=None) -> None:
    """q_layers, k_layers, lse_layers: sequences of device tensors, one per layer of the call."""
    n = len(k_layers)
    qs = (C.c_void_p * n)(*[t.data_ptr() for t in q_layers])
    ks = (C.c_void_p * n)(*[t.data_ptr() for t in k_layers])
    ls = (C.c_void_p * n)(*[t.data_ptr() for t in lse_layers])
    _check(load().dkv_score_window_lse_layers(C.byref(desc), layer_begin, n, qs, ks, k_stride_token, k_stride_head,
                                              _ptr(cu_seqlens), ls, _ptr(scores_all), _ptr(workspace),
                                              workspace.numel() * workspace.element_size(), _stream(stream)),
           "dkv_score_window_lse_layers")


def dkv_score_window_stats(desc, q_win, k, k_stride_token, k_stride_head, cu_seqlens, scores_out, scores_stride_head,
                           workspace, stream=None) -> None:
    _check(load().dkv_score_window_stats(C.byref(desc), _ptr(q_win), _ptr(k), k_stride_token, k_stride_head,
                                         _ptr(cu_seqlens), _ptr(scores_out), scores_stride_head, _ptr(workspace),
                                         workspace.numel() * workspace.element_size(), _stream(stream)),
           "dkv_score_window_stats")


def dkv_score_window_emit(desc, q_win, k, k_stride_token, k_stride_head, cu_seqlens, scores_out, scores_stride_head,
                          workspace, stream=None) -> None:
    _check(load().dkv_score_window_emit(C.byref(desc), _ptr(q_win), _ptr(k), k_stride_token, k_stride_head,
                                        _ptr(cu_seqlens), _ptr(scores_out), scores_stride_head, _ptr(workspace),
                                        workspace.numel() * workspace.element_size(), _stream(stream)),
           "dkv_score_window_emit")


def dkv_score_window_lse(desc, q_win, k, k_stride_token, k_stride_head, cu_seqlens, lse, scores_out, scores_stride_head,
                         stream=None) -> None:
    _check(load().dkv_score_window_lse(C.byref(desc), _ptr(q_win), _ptr(k), k_stride_token, k_stride_head,
                                       _ptr(cu_seqlens), _ptr(lse), _ptr(scores_out), scores_stride_head,
                                       _stream(stream)), "dkv_score_window_lse")


def dkv_row_lse(desc, k_stride_token, cu_seqlens, lse_out, workspace, stream=None) -> None:
    _check(load().dkv_row_lse(C.byref(desc), k_stride_token, _ptr(cu_seqlens), _ptr(lse_out), _ptr(workspace),
                              workspace.numel() * workspace.element_size(), _stream(stream)), "dkv_row_lse")


def dkv_select_topk(desc, layer, scores, scores_stride_head, cu_seqlens, idx_out, counts, workspace,
                    stream=None) -> None:
    _check(load().dkv_select_topk(C.byref(desc), layer, _ptr(scores), scores_stride_head, _ptr(cu_seqlens),
                                  _ptr(idx_out), _ptr(counts), _ptr(workspace),
                                  workspace.numel() * workspace.element_size(), _stream(stream)), "dkv_select_topk")


def dkv_select_topk_layers(desc, layer_begin, n_layers, scores_all, cu_seqlens, idx_all, counts, workspace,
                           stream=None) -> None:
    _check(load().dkv_select_topk_layers(C.byref(desc), layer_begin, n_layers, _ptr(scores_all), _ptr(cu_seqlens),
                                         _ptr(idx_all), _ptr(counts), _ptr(workspace),
                                         workspace.numel() * workspace.element_size(), _stream(stream)),
           "dkv_select_topk_layers")


def dkv_gather_kv_layers(desc, layer_begin, k_layers, v_layers, stride_token, stride_head, cu_seqlens, idx_all, counts,
                         k_out_all, v_out_all, out_stride_layer, out_stride_seq, out_stride_head, stream=None) -> None:
    """k_layers, v_layers: sequences of device tensors, one per layer of the call."""
    n = len(k_layers)
    ks = (C.c_void_p * n)(*[t.data_ptr() for t in k_layers])
    vs = (C.c_void_p * n)(*[t.data_ptr() for t in v_layers])
    _check(load().dkv_gather_kv_layers(C.byref(desc), layer_begin, n, ks, vs, stride_token, stride_head,
                                       _ptr(cu_seqlens), _ptr(idx_all), _ptr(counts), _ptr(k_out_all), _ptr(v_out_all),
                                       out_stride_layer, out_stride_seq, out_stride_head, _stream(stream)),
           "dkv_gather_kv_layers")


def dkv_rebalance(desc, layers_done, epoch, scores_all, cu_seqlens, counts, budgets_out, hits_out, workspace,
                  stream=None) -> None:
    _check(load().dkv_rebalance(C.byref(desc), layers_done, epoch, _ptr(scores_all), _ptr(cu_seqlens), _ptr(counts),
                                _ptr(budgets_out), _ptr(hits_out), _ptr(workspace),
                                workspace.numel() * workspace.element_size(), _stream(stream)), "dkv_rebalance")


def dkv_rebalance_batch(desc, layers_done, n_updates, epoch, scores_all, cu_seqlens, counts, budgets_out, hits_out,
                        out_stride_update, workspace, stream=None) -> None:
    _check(load().dkv_rebalance_batch(C.byref(desc), layers_done, n_updates, epoch, _ptr(scores_all), _ptr(cu_seqlens),
                                      _ptr(counts), _ptr(budgets_out), _ptr(hits_out), out_stride_update,
                                      _ptr(workspace), workspace.numel() * workspace.element_size(),
                                      _stream(stream)), "dkv_rebalance_batch")


def dkv_gather_kv(desc, layer, k, v, stride_token, stride_head, cu_seqlens, idx, counts, k_out, v_out, out_stride_seq,
                  out_stride_head, stream=None) -> None:
    _check(load().dkv_gather_kv(C.byref(desc), layer, _ptr(k), _ptr(v), stride_token, stride_head, _ptr(cu_seqlens),
                                _ptr(idx), _ptr(counts), _ptr(k_out), _ptr(v_out), out_stride_seq, out_stride_head,
                                _stream(stream)), "dkv_gather_kv")


def dkv_pack_cache(desc, cu_seqlens, counts, kb_all, vb_all, stride_layer, stride_seq, stride_head, k_packed, v_packed,
                   capacity_rows, row_offsets, stream=None) -> None:
    _check(load().dkv_pack_cache(C.byref(desc), _ptr(cu_seqlens), _ptr(counts), _ptr(kb_all), _ptr(vb_all),
                                 stride_layer, stride_seq, stride_head, _ptr(k_packed), _ptr(v_packed), capacity_rows,
                                 _ptr(row_offsets), _stream(stream)), "dkv_pack_cache")


def dkv_decode_attention(desc, layer, q_new, kb, vb, stride_seq, stride_head, cu_seqlens, counts, out, lse_out, workspace,
                         stream=None) -> None:
    _check(load().dkv_decode_attention(C.byref(desc), layer, _ptr(q_new), _ptr(kb), _ptr(vb), stride_seq, stride_head,
                                       _ptr(cu_seqlens), _ptr(counts), _ptr(out), _ptr(lse_out), _ptr(workspace),
                                       workspace.numel() * workspace.element_size(), _stream(stream)),
           "dkv_decode_attention")


def dkv_decode_attention_layers(desc, layer_begin, n_layers, q_new_all, kb_all, vb_all, stride_layer, stride_seq,
                                stride_head, cu_seqlens, counts, out_all, lse_all, workspace, stream=None) -> None:
    _check(load().dkv_decode_attention_layers(C.byref(desc), layer_begin, n_layers, _ptr(q_new_all), _ptr(kb_all),
                                              _ptr(vb_all), stride_layer, stride_seq, stride_head, _ptr(cu_seqlens),
                                              _ptr(counts), _ptr(out_all), _ptr(lse_all), _ptr(workspace),
                                              workspace.numel() * workspace.element_size(), _stream(stream)),
           "dkv_decode_attention_layers")


def alloc_workspace(desc, device="cuda"):
    """Allocate (torch) the workspace the stage calls need."""
    import torch
    n = dkv_workspace_bytes(desc)
    if n == 0:
        raise DkvError(DKV_ERR_INVALID_ARG, "dkv_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)
