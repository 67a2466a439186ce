"""Thin ctypes binding over libtokenlake.so: same names as the C ABI (include/tokenlake.h),
argument marshalling only.  Every step of the path runs in the library's kernels; there is
no Python or CPU fallback -- if the library is missing, loading raises.

Device arguments are torch tensors (their data_ptr is passed) or raw integer addresses;
host arrays are numpy arrays.  `stream=None` uses torch's current HIP stream.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtokenlake.so")

TL_OK, TL_EINVAL, TL_ENOMEM, TL_EFULL, TL_ENOTFOUND, TL_EHIP = 0, -1, -2, -3, -4, -5
TL_PLAN_SELF_BLOCK, TL_PLAN_NO_SHARING, TL_PLAN_FUSE_ROWS, TL_PLAN_WALK_REPEATS, TL_PLAN_FUSE_TAILS = 1, 2, 4, 8, 16


class TokenLakeError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("tokenlake status %d: %s" % (status, message))
        self.status = status


class tl_plan_info(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_req", "n_tokens", "q_heads", "kv_heads", "n_items", "n_partial_rows", "self_row_base",
        "n_tiles", "n_units", "n_causal_tiles", "n_list_entries", "n_merge_entries")] + [
        (n, C.c_int64) for n in ("prefix_pairs", "self_pairs", "unique_kv_tokens")] + [
        (n, C.c_int32) for n in ("n_fused_tiles", "n_fused_tokens", "n_single_tokens")] + [
        ("tile_pairs", C.c_int64), ("item_pairs", C.c_int64), ("n_prior_rows", C.c_int32)]


_lib = None

_P, _I32, _U64, _F32, _F64 = C.c_void_p, C.c_int32, C.c_uint64, C.c_float, C.c_double
_PF64 = C.POINTER(C.c_double)
_SIGNATURES = {
    "tl_status_str": (C.c_char_p, [_I32]),
    "tl_last_error": (C.c_char_p, []),
    "tl_set_option": (_I32, [C.c_char_p, _I32]),
    "tl_pool_create": (_I32, [C.POINTER(_P), _I32, _I32, _I32, _I32, _P, _P]),
    "tl_pool_destroy": (_I32, [_P]),
    "tl_pool_put": (_I32, [_P, _U64, _P, _P, _I32, _I32, C.POINTER(_I32), _P]),
    "tl_pool_append": (_I32, [_P, _I32, _U64, _P, _I32, _P, _P, _I32, _P, _P]),
    "tl_pool_append_batch": (_I32, [_P, _I32, _P, _P, _P, _P, _P, _P, _P, _P, _P]),
    "tl_pool_adopt": (_I32, [_P, _P, _P, _P, _I32, _P]),
    "tl_pool_release": (_I32, [_P, _U64]),
    "tl_pool_evict_lru": (_I32, [_P, C.POINTER(_U64)]),
    "tl_pool_lookup": (_I32, [_P, _P, _I32, _P]),
    "tl_pool_hot_segments": (_I32, [_P, _I32, _P, _P, _P, C.POINTER(_I32)]),
    "tl_pool_prefix_tree": (_I32, [_P, _I32, _P, _P, _P, C.POINTER(_I32), C.POINTER(_I32)]),
    "tl_pool_fills": (_I32, [_P, _P, _I32, _P]),
    "tl_pool_used": (_I32, [_P, C.POINTER(_I32)]),
    "tl_pool_gather": (_I32, [_P, _P, _I32, _P, _P, _P]),
    "tl_plan_create": (_I32, [C.POINTER(_P), _P, _I32, _I32, _P, _P, _P, _I32, _I32, _I32]),
    "tl_plan_destroy": (_I32, [_P]),
    "tl_plan_get_info": (_I32, [_P, C.POINTER(tl_plan_info)]),
    "tl_plan_export_sizes": (_I32, [_P, C.POINTER(_I32), C.POINTER(_I32)]),
    "tl_plan_hot_slots": (_I32, [_P, _I32, _P, _P, C.POINTER(_I32)]),
    "tl_plan_export": (_I32, [_P, _P, _P, _P, _P, _P, _P, _P]),
    "tl_segment_attn": (_I32, [_P, _P, _P, _F32, _P, _P, _P]),
    "tl_causal_block": (_I32, [_P, _P, _P, _P, _F32, _P, _P, _P]),
    "tl_merge": (_I32, [_P, _P, _P, _P, _I32, _P, _P]),
    "tl_fused_attn": (_I32, [_P, _P, _P, _P, _P, _F32, _P, _P, _P, _I32, _P, _P]),
    "tl_fused_attn_static": (_I32, [_P, _P, _P, _P, _P, _F32, _P, _P, _P, _I32, _P, _P]),
    "tl_model_segment_time": (_I32, [_F64, _F64, _F64, _F64, _F64, _PF64]),
    "tl_model_comm_time": (_I32, [_F64, _F64, _F64, _PF64]),
    "tl_model_segment_threshold": (_I32, [_F64, _F64, _F64, _F64, _F64, _F64, _PF64]),
    "tl_model_cache_load": (_I32, [_F64, _P, _P, _I32, _I32, _F64, _F64, _F64, _PF64, _PF64, _PF64]),
    "tl_segment_ids": (_I32, [_P, C.c_int64, _I32, C.c_uint64, _P]),
}
EXPORTED = tuple(_SIGNATURES)


def load_library(path: Optional[str] = None):
    """Load libtokenlake.so (built by paper_2508_17219_amd.build).  Raises if it is absent."""
    global _lib
    if _lib is None:
        p = path or os.environ.get("TOKENLAKE_LIB") or LIB_PATH
        if not os.path.exists(p):
            raise FileNotFoundError(
                "%s not found: build it with `python -m paper_2508_17219_amd.build` "
                "(there is no fallback path)" % p)
        lib = C.CDLL(p)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def _check(status: int):
    if status != TL_OK:
        raise TokenLakeError(status, load_library().tl_last_error().decode())


def _dev(x) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if not x.is_contiguous():
        raise ValueError("device tensor must be contiguous")
    return x.data_ptr()


def _host(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=dtype)


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        if torch.cuda.is_available():
            return torch.cuda.current_stream().cuda_stream or None
        return None
    return int(stream) or None


# ---- pool -------------------------------------------------------------------------------
def tl_pool_create(n_slots: int, seg_len: int, kv_heads: int, head_dim: int, k_dev=None, v_dev=None) -> int:
    h = _P()
    _check(load_library().tl_pool_create(C.byref(h), n_slots, seg_len, kv_heads, head_dim, _dev(k_dev), _dev(v_dev)))
    return h.value


def tl_pool_destroy(pool: int):
    _check(load_library().tl_pool_destroy(pool))


def tl_pool_put(pool: int, segment_id: int, k_src, v_src, fill: int, want_slot: int = -1, stream=None) -> int:
    slot = _I32(-1)
    _check(load_library().tl_pool_put(pool, segment_id, _dev(k_src), _dev(v_src), fill, want_slot, C.byref(slot),
                                      _stream(stream)))
    return slot.value


def tl_pool_append(pool: int, tail_id, new_ids, k_rows, v_rows, n_rows: int, stream=None) -> np.ndarray:
    """tail_id None = no partly filled tail.  Returns the slots given to new_ids."""
    ids = _host(new_ids, np.uint64)
    slots = np.full(len(ids), -1, np.int32)
    _check(load_library().tl_pool_append(pool, 0 if tail_id is None else 1, 0 if tail_id is None else int(tail_id),
                                         ids.ctypes.data if len(ids) else None, len(ids), _dev(k_rows), _dev(v_rows),
                                         n_rows, slots.ctypes.data if len(ids) else None, _stream(stream)))
    return slots


def tl_pool_append_batch(pool: int, tail_ids, new_ids, row_counts, k_rows, v_rows, stream=None) -> np.ndarray:
    """One call for many chains.  tail_ids: per chain an id or None; new_ids: per chain a list of
    ids; row_counts: per chain the number of rows it takes from k_rows/v_rows (in chain order).
    Returns the slots given to the new ids, flattened in chain order."""
    n = len(tail_ids)
    has_tail = np.array([0 if t is None else 1 for t in tail_ids], np.int32)
    tails = np.array([0 if t is None else int(t) for t in tail_ids], np.uint64)
    new_ptr = np.zeros(n + 1, np.int32)
    new_ptr[1:] = np.cumsum([len(x) for x in new_ids])
    ids = np.array([i for x in new_ids for i in x], np.uint64)
    row_ptr = np.zeros(n + 1, np.int32)
    row_ptr[1:] = np.cumsum(row_counts)
    slots = np.full(len(ids), -1, np.int32)
    _check(load_library().tl_pool_append_batch(pool, n, has_tail.ctypes.data, tails.ctypes.data, new_ptr.ctypes.data,
                                               ids.ctypes.data if len(ids) else None, row_ptr.ctypes.data,
                                               _dev(k_rows), _dev(v_rows), slots.ctypes.data if len(ids) else None,
                                               _stream(stream)))
    return slots


def tl_pool_adopt(pool: int, ids, slots, fills, stream=None):
    ids, slots, fills = _host(ids, np.uint64), _host(slots, np.int32), _host(fills, np.int32)
    if not (len(ids) == len(slots) == len(fills)):
        raise ValueError("ids/slots/fills length mismatch")
    _check(load_library().tl_pool_adopt(pool, ids.ctypes.data, slots.ctypes.data, fills.ctypes.data, len(ids),
                                        _stream(stream)))


def tl_pool_release(pool: int, segment_id: int):
    _check(load_library().tl_pool_release(pool, segment_id))


def tl_pool_evict_lru(pool: int) -> int:
    out = _U64(0)
    _check(load_library().tl_pool_evict_lru(pool, C.byref(out)))
    return out.value


def tl_pool_hot_segments(pool: int, max_n: int):
    """(ids, loads, depths) of the prefix tree's most loaded nodes, at most max_n, parents first."""
    m = max(max_n, 1)
    ids, loads, depths, n = np.zeros(m, np.uint64), np.zeros(m, np.int64), np.zeros(m, np.int32), _I32(0)
    _check(load_library().tl_pool_hot_segments(pool, max_n, ids.ctypes.data, loads.ctypes.data, depths.ctypes.data, C.byref(n)))
    return ids[:n.value], loads[:n.value], depths[:n.value]


def tl_pool_prefix_tree(pool: int, max_nodes: int):
    """(ids, parents, loads, n_total): the pool's prefix tree in level order, at most max_nodes nodes."""
    m = max(max_nodes, 1)
    ids, parents, loads = np.zeros(m, np.uint64), np.zeros(m, np.int32), np.zeros(m, np.int64)
    n, total = _I32(0), _I32(0)
    _check(load_library().tl_pool_prefix_tree(pool, max_nodes, ids.ctypes.data, parents.ctypes.data, loads.ctypes.data,
                                              C.byref(n), C.byref(total)))
    return ids[:n.value], parents[:n.value], loads[:n.value], total.value


def tl_pool_lookup(pool: int, ids) -> np.ndarray:
    ids = _host(ids, np.uint64)
    out = np.empty(len(ids), np.int32)
    _check(load_library().tl_pool_lookup(pool, ids.ctypes.data, len(ids), out.ctypes.data))
    return out


def tl_pool_fills(pool: int, slots) -> np.ndarray:
    slots = _host(slots, np.int32)
    out = np.empty(len(slots), np.int32)
    _check(load_library().tl_pool_fills(pool, slots.ctypes.data, len(slots), out.ctypes.data))
    return out


def tl_pool_used(pool: int) -> int:
    n = _I32(0)
    _check(load_library().tl_pool_used(pool, C.byref(n)))
    return n.value


def tl_pool_gather(pool: int, slots, k_out, v_out, stream=None):
    slots = _host(slots, np.int32)
    _check(load_library().tl_pool_gather(pool, slots.ctypes.data, len(slots), _dev(k_out), _dev(v_out), _stream(stream)))


# ---- plan -------------------------------------------------------------------------------
def tl_plan_create(pool: int, q_heads: int, req_row_ptr, req_seg_ptr, seg_ids, flags: int = TL_PLAN_SELF_BLOCK,
                   split_segments: int = 0, compute_units: int = -1) -> int:
    rp, sp, ids = _host(req_row_ptr, np.int32), _host(req_seg_ptr, np.int32), _host(seg_ids, np.uint64)
    if len(rp) != len(sp) or len(rp) < 1:
        raise ValueError("req_row_ptr/req_seg_ptr must both have n_req+1 entries")
    if len(ids) < int(sp[-1]):
        raise ValueError("seg_ids shorter than req_seg_ptr[-1]")
    h = _P()
    _check(load_library().tl_plan_create(C.byref(h), pool, q_heads, len(rp) - 1, rp.ctypes.data, sp.ctypes.data,
                                         ids.ctypes.data if len(ids) else None, flags, split_segments, compute_units))
    return h.value


def tl_plan_destroy(plan: int):
    _plan_shapes.pop(plan, None)
    _check(load_library().tl_plan_destroy(plan))


# (n_tokens, n_partial_rows, q_heads, kv_heads) of every live plan: the compute wrappers check the
# tensors they are handed against it -- the C ABI sees only pointers and cannot
_plan_shapes = {}


def _shape_of(plan: int):
    sh = _plan_shapes.get(plan)
    if sh is None:
        i = tl_plan_get_info(plan)
        sh = _plan_shapes[plan] = (i.n_tokens, i.n_partial_rows, i.q_heads, i.kv_heads)
    return sh


def _need(t, name: str, rows: int, heads: int, dim, kind: str):
    """t must be a device tensor of the given element kind with at least rows x heads (x dim) elements."""
    if t is None or rows == 0 or isinstance(t, int):
        return
    if not _kinds:
        import torch
        _kinds.update(bf16=torch.bfloat16, f32=torch.float32)
    if t.dtype != _kinds[kind]:
        raise TypeError("%s must be %s, is %s" % (name, kind, t.dtype))
    n = rows * heads * (dim or 1)
    if t.numel() < n:
        raise ValueError("%s has %d elements, the plan needs %d" % (name, t.numel(), n))


_kinds = {}


def tl_plan_get_info(plan: int) -> tl_plan_info:
    info = tl_plan_info()
    _check(load_library().tl_plan_get_info(plan, C.byref(info)))
    return info


def tl_plan_hot_slots(plan: int, max_n: int):
    """(slots, loads) of the batch's most loaded slots, at most max_n."""
    slots, loads, n = np.zeros(max(max_n, 1), np.int32), np.zeros(max(max_n, 1), np.int64), _I32(0)
    _check(load_library().tl_plan_hot_slots(plan, max_n, slots.ctypes.data, loads.ctypes.data, C.byref(n)))
    return slots[:n.value], loads[:n.value]


def tl_plan_export(plan: int) -> dict:
    lib = load_library()
    info = tl_plan_get_info(plan)
    nt, ns = _I32(0), _I32(0)
    _check(lib.tl_plan_export_sizes(plan, C.byref(nt), C.byref(ns)))
    out = {
        "item_row_base": np.zeros(info.n_items, np.int32),
        "item_tok_ptr": np.zeros(info.n_items + 1, np.int32),
        "item_tokens": np.zeros(nt.value, np.int32),
        "item_slot_ptr": np.zeros(info.n_items + 1, np.int32),
        "item_slots": np.zeros(ns.value, np.int32),
        "merge_ptr": np.zeros(info.n_tokens + 1, np.int32),
        "merge_rows": np.zeros(info.n_merge_entries, np.int32),
    }
    _check(lib.tl_plan_export(plan, *[out[k].ctypes.data for k in (
        "item_row_base", "item_tok_ptr", "item_tokens", "item_slot_ptr", "item_slots", "merge_ptr", "merge_rows")]))
    return out


# ---- compute ----------------------------------------------------------------------------
def tl_segment_attn(pool: int, plan: int, q, scale: float, out_partial, lse, stream=None):
    T, R, hq, _ = _shape_of(plan)
    _need(q, "q", T, hq, 128, "bf16"); _need(out_partial, "out_partial", R, hq, 128, "f32"); _need(lse, "lse", R, hq, None, "f32")
    _check(load_library().tl_segment_attn(pool, plan, _dev(q), scale, _dev(out_partial), _dev(lse), _stream(stream)))


def tl_causal_block(plan: int, q, k_new, v_new, scale: float, out_partial, lse, stream=None):
    T, R, hq, hkv = _shape_of(plan)
    _need(q, "q", T, hq, 128, "bf16"); _need(k_new, "k_new", T, hkv, 128, "bf16"); _need(v_new, "v_new", T, hkv, 128, "bf16")
    _need(out_partial, "out_partial", R, hq, 128, "f32"); _need(lse, "lse", R, hq, None, "f32")
    _check(load_library().tl_causal_block(plan, _dev(q), _dev(k_new), _dev(v_new), scale, _dev(out_partial), _dev(lse),
                                          _stream(stream)))


def tl_fused_attn(pool: int, plan: int, q, k_new, v_new, scale: float, out, out_is_bf16: bool, lse_out=None, stream=None,
                  prior_partial=None, prior_lse=None):
    """prior_partial / prior_lse: the partial buffers tl_segment_attn wrote (needed by TL_PLAN_FUSE_TAILS plans)."""
    T, R, hq, hkv = _shape_of(plan)
    _need(q, "q", T, hq, 128, "bf16"); _need(k_new, "k_new", T, hkv, 128, "bf16"); _need(v_new, "v_new", T, hkv, 128, "bf16")
    _need(out, "out", T, hq, 128, "bf16" if out_is_bf16 else "f32"); _need(lse_out, "lse_out", T, hq, None, "f32")
    _need(prior_partial, "prior_partial", R, hq, 128, "f32"); _need(prior_lse, "prior_lse", R, hq, None, "f32")
    _check(load_library().tl_fused_attn(pool, plan, _dev(q), _dev(k_new), _dev(v_new), scale, _dev(prior_partial),
                                        _dev(prior_lse), _dev(out), int(bool(out_is_bf16)), _dev(lse_out), _stream(stream)))


def tl_fused_attn_static(pool: int, plan: int, q, k_new, v_new, scale: float, out, out_is_bf16: bool, lse_out=None,
                         stream=None, prior_partial=None, prior_lse=None):
    """tl_fused_attn without any device allocation (the plan's work lists go to a static device buffer)."""
    T, R, hq, hkv = _shape_of(plan)
    _need(q, "q", T, hq, 128, "bf16"); _need(k_new, "k_new", T, hkv, 128, "bf16"); _need(v_new, "v_new", T, hkv, 128, "bf16")
    _need(out, "out", T, hq, 128, "bf16" if out_is_bf16 else "f32"); _need(lse_out, "lse_out", T, hq, None, "f32")
    _need(prior_partial, "prior_partial", R, hq, 128, "f32"); _need(prior_lse, "prior_lse", R, hq, None, "f32")
    _check(load_library().tl_fused_attn_static(pool, plan, _dev(q), _dev(k_new), _dev(v_new), scale, _dev(prior_partial),
                                               _dev(prior_lse), _dev(out), int(bool(out_is_bf16)), _dev(lse_out),
                                               _stream(stream)))


def tl_merge(plan: int, out_partial, lse, out, out_is_bf16: bool, lse_out=None, stream=None):
    T, R, hq, _ = _shape_of(plan)
    _need(out_partial, "out_partial", R, hq, 128, "f32"); _need(lse, "lse", R, hq, None, "f32")
    _need(out, "out", T, hq, 128, "bf16" if out_is_bf16 else "f32"); _need(lse_out, "lse_out", T, hq, None, "f32")
    _check(load_library().tl_merge(plan, _dev(out_partial), _dev(lse), _dev(out), int(bool(out_is_bf16)), _dev(lse_out),
                                   _stream(stream)))


def tl_set_option(knob: str, value: int):
    _check(load_library().tl_set_option(knob.encode(), value))


# ---- analytic models ----------------------------------------------------------------------
def tl_model_segment_time(n_tokens: float, d_q: float, d_kv: float, flops: float, mem_bw: float) -> float:
    out = _F64(0.0)
    _check(load_library().tl_model_segment_time(n_tokens, d_q, d_kv, flops, mem_bw, C.byref(out)))
    return out.value


def tl_model_comm_time(d_q: float, net_latency: float, net_bw: float) -> float:
    out = _F64(0.0)
    _check(load_library().tl_model_comm_time(d_q, net_latency, net_bw, C.byref(out)))
    return out.value


def tl_model_segment_threshold(d_q: float, d_kv: float, flops: float, mem_bw: float, net_latency: float,
                               net_bw: float) -> float:
    out = _F64(0.0)
    _check(load_library().tl_model_segment_threshold(d_q, d_kv, flops, mem_bw, net_latency, net_bw, C.byref(out)))
    return out.value


def tl_model_cache_load(d: float, prefix_len, input_len, n_gpus: int, mem_bw: float, flops: float, t_ideal: float):
    """Returns (M_r bytes, F_r flop, L)."""
    pl, il = _host(prefix_len, np.int64), _host(input_len, np.int64)
    if len(pl) != len(il):
        raise ValueError("prefix_len/input_len length mismatch")
    m, f, load = _F64(0.0), _F64(0.0), _F64(0.0)
    _check(load_library().tl_model_cache_load(d, pl.ctypes.data if len(pl) else None, il.ctypes.data if len(il) else None,
                                              len(pl), n_gpus, mem_bw, flops, t_ideal, C.byref(m), C.byref(f), C.byref(load)))
    return m.value, f.value, load.value


def tl_segment_ids(tokens, seg_len: int, salt: int = 0) -> np.ndarray:
    """Content-derived ids of the segments of a token sequence (uint64, one per started segment)."""
    t = _host(tokens, np.int32)
    n_ids = (len(t) + seg_len - 1) // seg_len if seg_len > 0 else 0
    ids = np.zeros(n_ids, np.uint64)
    _check(load_library().tl_segment_ids(t.ctypes.data if len(t) else None, len(t), seg_len, salt & 0xFFFFFFFFFFFFFFFF,
                                         ids.ctypes.data if n_ids else None))
    return ids
