"""Test-side glue: run a workload batch through the C-ABI on the GPU, and evaluate the fp64
oracle on chosen rows of the same batch.  The two sides meet only here, in the tests."""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np
import torch

from oracle import tokenlake_oracle as orc
from paper_2508_17219_amd import binding as B
from paper_2508_17219_amd import workloads as wl

TOL_O = 2e-2      # max abs error on O      (bf16 inputs, fp32 accumulate)
TOL_LSE = 1e-3    # max abs error on LSE


@dataclass
class DeviceRun:
    batch: wl.Batch
    pool: int
    plan: int
    info: object
    q: torch.Tensor
    k_new: torch.Tensor
    v_new: torch.Tensor
    pool_k: torch.Tensor
    pool_v: torch.Tensor
    out_partial: torch.Tensor
    lse_partial: torch.Tensor
    out: torch.Tensor
    lse: torch.Tensor

    def close(self):
        B.tl_plan_destroy(self.plan)
        B.tl_pool_destroy(self.pool)


def device_pool(batch: wl.Batch, device="cuda", poison: bool = True):
    """Pool tensors with every resident segment written by the generator.  Unwritten memory
    (free slots, tails beyond fill) holds NaN bit patterns when `poison` is set, so any read
    of a token that does not exist shows up in the output."""
    shape = (batch.n_slots, batch.seg_len, batch.kv_heads, batch.head_dim)
    if poison:
        pk = torch.full(shape, float("nan"), dtype=torch.bfloat16, device=device)
        pv = torch.full(shape, float("nan"), dtype=torch.bfloat16, device=device)
    else:
        pk = torch.zeros(shape, dtype=torch.bfloat16, device=device)
        pv = torch.zeros(shape, dtype=torch.bfloat16, device=device)
    batch.fill_pool(pk, pv)
    return pk, pv


def run_gpu(batch: wl.Batch, flags=None, split_segments: int = 0, out_bf16: bool = False, poison: bool = True,
            pool_tensors=None, fuse: bool = False, fill_cus: int = 0, compute_units=None) -> DeviceRun:
    dev = "cuda"
    pk, pv = pool_tensors if pool_tensors is not None else device_pool(batch, dev, poison)
    pool = B.tl_pool_create(batch.n_slots, batch.seg_len, batch.kv_heads, batch.head_dim, pk, pv)
    B.tl_pool_adopt(pool, batch.pool_ids, batch.pool_slots, batch.pool_fills)
    if flags is None:
        flags = B.TL_PLAN_SELF_BLOCK if batch.self_block else 0
    if fuse:
        flags |= B.TL_PLAN_FUSE_ROWS
    # compute_units 0: one-pass rows, and uncut row-tile items, even when the batch is small (the
    # default for one-pass plans here: the tests' batches are small)
    if compute_units is None:
        compute_units = fill_cus if fuse else -1
    plan = B.tl_plan_create(pool, batch.q_heads, batch.req_row_ptr, batch.req_seg_ptr, batch.seg_ids, flags,
                            split_segments, compute_units)
    info = B.tl_plan_get_info(plan)
    q = batch.q(dev)
    kn = batch.k_new(dev)
    vn = batch.v_new(dev)
    R, T, H = info.n_partial_rows, info.n_tokens, batch.q_heads
    # poison outputs so that an unwritten row is noticed
    outp = torch.full((max(R, 1), H, batch.head_dim), float("nan"), dtype=torch.float32, device=dev)
    lsep = torch.full((max(R, 1), H), float("nan"), dtype=torch.float32, device=dev)
    out = torch.full((max(T, 1), H, batch.head_dim), float("nan"),
                     dtype=torch.bfloat16 if out_bf16 else torch.float32, device=dev)
    lse = torch.full((max(T, 1), H), float("nan"), dtype=torch.float32, device=dev)
    B.tl_segment_attn(pool, plan, q, batch.scale, outp, lsep)
    if flags & B.TL_PLAN_SELF_BLOCK:
        B.tl_causal_block(plan, q, kn, vn, batch.scale, outp, lsep)
    B.tl_merge(plan, outp, lsep, out, out_bf16, lse)
    if flags & (B.TL_PLAN_FUSE_ROWS | B.TL_PLAN_FUSE_TAILS):
        B.tl_fused_attn(pool, plan, q, kn, vn, batch.scale, out, out_bf16, lse, prior_partial=outp, prior_lse=lsep)
    torch.cuda.synchronize()
    return DeviceRun(batch, pool, plan, info, q, kn, vn, pk, pv, outp, lsep, out, lse)


# ---- oracle side -------------------------------------------------------------------------
def host_request_inputs(batch: wl.Batch, r: int):
    """Everything the oracle needs for request r, generated on the CPU: a compact pool that
    holds only this request's segments (slot = position among its distinct ids)."""
    ids = batch.seg_ids[batch.req_seg_ptr[r]:batch.req_seg_ptr[r + 1]]
    uniq = list(dict.fromkeys(int(s) for s in ids))
    pos = {s: i for i, s in enumerate(uniq)}
    fill_of = dict(zip(batch.pool_ids.tolist(), batch.pool_fills.tolist()))
    if uniq:
        k, v = batch.segment_kv(np.array(uniq, dtype=np.uint64), "cpu")
        pk, pv = wl.bits_u16(k), wl.bits_u16(v)
    else:
        shp = (0, batch.seg_len, batch.kv_heads, batch.head_dim)
        pk, pv = np.zeros(shp, np.uint16), np.zeros(shp, np.uint16)
    slots = np.array([pos[int(s)] for s in ids], dtype=np.int64)
    fills = np.array([fill_of[int(s)] for s in ids], dtype=np.int64)
    t0, t1 = int(batch.req_row_ptr[r]), int(batch.req_row_ptr[r + 1])
    qb = wl.bits_u16(batch.q("cpu", t0, t1))
    kn = wl.bits_u16(batch.k_new("cpu", t0, t1))
    vn = wl.bits_u16(batch.v_new("cpu", t0, t1))
    return qb, pk, pv, slots, fills, kn, vn


def oracle_request_rows(batch: wl.Batch, r: int, rows=None):
    """Oracle O [n, Hq, d], LSE [n, Hq] for the given new-token indices (local to request r;
    default all) -- full attention over the prefix plus the causal self block."""
    qb, pk, pv, slots, fills, kn, vn = host_request_inputs(batch, r)
    lq = qb.shape[0]
    rows = np.arange(lq) if rows is None else np.asarray(rows, np.int64)
    if not batch.self_block:
        return orc.request_attention(qb[rows], pk, pv, slots, fills, None, None, batch.scale)
    gk, gv = orc.gather_segments(pk, pv, slots, fills)
    k_all = np.concatenate([gk, kn], axis=0)
    v_all = np.concatenate([gv, vn], axis=0)
    n_vis = gk.shape[0] + rows + 1
    return orc.partial_attention(qb[rows], k_all, v_all, batch.scale, n_visible=n_vis)


def compare_rows(run: DeviceRun, r: int, rows=None, tol_o=TOL_O, tol_lse=TOL_LSE):
    """Max abs errors of the merged output of request r against the oracle on `rows`."""
    b = run.batch
    t0 = int(b.req_row_ptr[r])
    lq = int(b.req_row_ptr[r + 1]) - t0
    rows = np.arange(lq) if rows is None else np.asarray(rows, np.int64)
    want_o, want_l = oracle_request_rows(b, r, rows)
    idx = torch.as_tensor(t0 + rows, device=run.out.device)
    got_o = run.out[idx].double().cpu().numpy()
    got_l = run.lse[idx].double().cpu().numpy()
    assert not np.isnan(got_o).any(), "NaN in output of request %d" % r
    assert not np.isnan(got_l).any(), "NaN in LSE of request %d" % r
    err_o = float(np.abs(got_o - want_o).max()) if got_o.size else 0.0
    both_inf = np.isneginf(got_l) & np.isneginf(want_l)
    err_l = float(np.abs(np.where(both_inf, 0.0, got_l - want_l)).max()) if got_l.size else 0.0
    ref = float(np.abs(want_o).max()) if want_o.size else 0.0
    return {"err_o": err_o, "err_lse": err_l, "ref_o": ref, "rel_o": err_o / ref if ref > 0 else 0.0,
            "ok": err_o <= tol_o and err_l <= tol_lse}


def device_request_inputs(run: DeviceRun, r: int, kv_sel=None):
    """The oracle's inputs for request r, copied back from the tensors the seeded generator wrote
    on the device (pool slots, Q, new K/V; the generator's output is bit-identical on either
    device) instead of generated a second time on the host: what makes every request of the
    full-size configurations affordable.  A compact pool of the request's distinct slots.
    kv_sel: optional list of kv heads; only they and their q heads are taken."""
    b = run.batch
    cache = run.__dict__.setdefault("_maps", {})
    if not cache:
        cache["slot"] = dict(zip(b.pool_ids.tolist(), b.pool_slots.tolist()))
        cache["fill"] = dict(zip(b.pool_ids.tolist(), b.pool_fills.tolist()))
    g = b.q_heads // b.kv_heads
    kv_sel = list(range(b.kv_heads)) if kv_sel is None else [int(x) for x in kv_sel]
    q_sel = [kv * g + j for kv in kv_sel for j in range(g)]
    ids = b.seg_ids[b.req_seg_ptr[r]:b.req_seg_ptr[r + 1]]
    uniq = list(dict.fromkeys(int(s) for s in ids))
    pos = {s: i for i, s in enumerate(uniq)}
    dev = run.pool_k.device
    kv_idx = torch.as_tensor(kv_sel, device=dev)
    if uniq:
        dslots = torch.as_tensor([cache["slot"][s] for s in uniq], device=dev, dtype=torch.int64)
        pk = wl.bits_u16(run.pool_k[dslots].index_select(2, kv_idx))
        pv = wl.bits_u16(run.pool_v[dslots].index_select(2, kv_idx))
    else:
        shp = (0, b.seg_len, len(kv_sel), b.head_dim)
        pk, pv = np.zeros(shp, np.uint16), np.zeros(shp, np.uint16)
    slots = np.array([pos[int(s)] for s in ids], dtype=np.int64)
    fills = np.array([cache["fill"][int(s)] for s in ids], dtype=np.int64)
    t0, t1 = int(b.req_row_ptr[r]), int(b.req_row_ptr[r + 1])
    qb = wl.bits_u16(run.q[t0:t1].index_select(1, torch.as_tensor(q_sel, device=dev)))
    kn = wl.bits_u16(run.k_new[t0:t1].index_select(1, kv_idx))
    vn = wl.bits_u16(run.v_new[t0:t1].index_select(1, kv_idx))
    return qb, pk, pv, slots, fills, kn, vn, q_sel


def compare_rows_device(run: DeviceRun, r: int, rows=None, kv_sel=None):
    """compare_rows with the oracle's inputs taken from the device tensors (device_request_inputs),
    optionally on a subset of kv heads."""
    b = run.batch
    qb, pk, pv, slots, fills, kn, vn, q_sel = device_request_inputs(run, r, kv_sel)
    t0 = int(b.req_row_ptr[r])
    lq = qb.shape[0]
    rows = np.arange(lq) if rows is None else np.asarray(rows, np.int64)
    if b.self_block:
        gk, gv = orc.gather_segments(pk, pv, slots, fills)
        k_all = np.concatenate([gk, kn], axis=0)
        v_all = np.concatenate([gv, vn], axis=0)
        want_o, want_l = orc.partial_attention(qb[rows], k_all, v_all, b.scale, n_visible=gk.shape[0] + rows + 1)
    else:
        want_o, want_l = orc.request_attention(qb[rows], pk, pv, slots, fills, None, None, b.scale)
    idx = torch.as_tensor(t0 + rows, device=run.out.device)
    hsel = torch.as_tensor(q_sel, device=run.out.device)
    got_o = run.out[idx].index_select(1, hsel).double().cpu().numpy()
    got_l = run.lse[idx].index_select(1, hsel).double().cpu().numpy()
    assert not np.isnan(got_o).any(), "NaN in output of request %d" % r
    assert not np.isnan(got_l).any(), "NaN in LSE of request %d" % r
    err_o = float(np.abs(got_o - want_o).max()) if got_o.size else 0.0
    both_inf = np.isneginf(got_l) & np.isneginf(want_l)
    err_l = float(np.abs(np.where(both_inf, 0.0, got_l - want_l)).max()) if got_l.size else 0.0
    ref = float(np.abs(want_o).max()) if want_o.size else 0.0
    return {"err_o": err_o, "err_lse": err_l, "ref_o": ref, "rel_o": err_o / ref if ref > 0 else 0.0,
            "ok": err_o <= TOL_O and err_l <= TOL_LSE}


def sample_rows(lq: int, n: int, rng: np.random.Generator):
    """First, last and tile-boundary rows plus random ones."""
    fixed = [0, lq - 1, 31, 32, 63, 64, 65, 127, 128, 255, 256]
    rows = sorted(set(x for x in fixed if 0 <= x < lq) | set(rng.integers(0, lq, size=n).tolist()))
    return np.array(rows, np.int64)
