"""Seeded synthetic inputs for the segment-attention hot path.

This module only *draws inputs*: request shapes, segment lists, slot placement and bf16 tensor
values.  It contains none of the method's arithmetic (no attention, no softmax, no merge) and
is the one module that both the CPU oracle's tests and the GPU path consume.

Tensor values come from a counter-based generator so that any slice can be produced on any
device with identical bits: element i of stream s under seed z is
    table[ top16( mix64(i + GOLDEN * (z * 16 + s + 1)) ) ]
where mix64 is the splitmix64 finaliser (integer-only) and `table` holds the 65536 mid-point
quantiles of N(0,1) rounded to bf16.  Only integer ops and one gather run on the device, so
CPU and GPU agree bit for bit.  The request *structure* (lengths, placements) is small and is
drawn on the host with numpy's PCG64.

The five workloads are the build's named configurations (they stand in for the paper's
LooGLE shared-prefix / SCBench multi-turn / ShareGPT traces, which are not available):
  tiny, prefill (Llama-3-8B layer shape), decode (70B layer shape), longctx, multiturn.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np
import torch

HEAD_DIM = 128

STREAM_Q, STREAM_KNEW, STREAM_VNEW, STREAM_POOL_K, STREAM_POOL_V = 0, 1, 2, 3, 4

_GOLDEN = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB


def _s64(x: int) -> int:
    """Python int -> the int64 with the same low 64 bits."""
    x &= (1 << 64) - 1
    return x - (1 << 64) if x >= (1 << 63) else x


_TABLE_CACHE = {}


def quantile_table(device="cpu") -> torch.Tensor:
    """65536 mid-point quantiles of N(0,1), rounded to bf16 (built once on the host)."""
    key = str(device)
    if key not in _TABLE_CACHE:
        if "cpu" not in _TABLE_CACHE:
            from scipy.special import ndtri
            u = (np.arange(65536, dtype=np.float64) + 0.5) / 65536.0
            t = torch.from_numpy(ndtri(u).astype(np.float32)).to(torch.bfloat16)
            _TABLE_CACHE["cpu"] = t
        _TABLE_CACHE[key] = _TABLE_CACHE["cpu"].to(device)
    return _TABLE_CACHE[key]


def _lsr(z: torch.Tensor, k: int) -> torch.Tensor:
    """Logical shift right of an int64 tensor."""
    return (z >> k) & ((1 << (64 - k)) - 1)


def _mix64(z: torch.Tensor) -> torch.Tensor:
    z = (z ^ _lsr(z, 30)) * _s64(_M1)
    z = (z ^ _lsr(z, 27)) * _s64(_M2)
    return z ^ _lsr(z, 31)


def normal_bf16(seed: int, stream: int, index: torch.Tensor) -> torch.Tensor:
    """bf16 N(0,1) draws at the given int64 element indices (any shape, any device)."""
    key = _s64(_GOLDEN * (int(seed) * 16 + int(stream) + 1))
    h = _mix64(index + key)
    return quantile_table(index.device)[_lsr(h, 48)]


def normal_bf16_range(seed: int, stream: int, start: int, count: int, device="cpu",
                      chunk: int = 1 << 24) -> torch.Tensor:
    out = torch.empty(count, dtype=torch.bfloat16, device=device)
    for c0 in range(0, count, chunk):
        c1 = min(count, c0 + chunk)
        idx = torch.arange(start + c0, start + c1, dtype=torch.int64, device=device)
        out[c0:c1] = normal_bf16(seed, stream, idx)
    return out


def bits_u16(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor -> numpy uint16 bit patterns (host copy)."""
    return t.detach().contiguous().cpu().view(torch.int16).numpy().view(np.uint16)


# --------------------------------------------------------------------------------------
@dataclass
class Batch:
    """One batch of requests against a segment pool (one layer, one iteration)."""
    name: str
    seed: int
    q_heads: int
    kv_heads: int
    seg_len: int
    n_slots: int
    req_row_ptr: np.ndarray            # int32 [n_req+1]   offsets of each request's new tokens
    req_seg_ptr: np.ndarray            # int32 [n_req+1]   offsets into seg_ids
    seg_ids: np.ndarray                # uint64 [n_entries] each request's prefix, in order
    pool_ids: np.ndarray               # uint64 [n_resident] ids resident in the pool
    pool_slots: np.ndarray             # int32  [n_resident] their slots
    pool_fills: np.ndarray             # int32  [n_resident] valid tokens in each
    head_dim: int = HEAD_DIM
    k_gain: float = 1.0                # power of two; >1 makes the softmax peaked
    v_offset_mod: int = 0              # >0: V of segment id s gets the integer offset (s % mod) - mod//2
    k_boost: tuple = ()                # (lo, hi, gain): K of segments at list positions lo <= p < hi (the low
                                       # 32 bits of the id) is multiplied by the power of two `gain`
    self_block: bool = True
    row_base: int = 0                  # first element index of this batch in the Q/Knew/Vnew streams
    notes: str = ""

    @property
    def n_req(self) -> int:
        return len(self.req_row_ptr) - 1

    @property
    def n_tokens(self) -> int:
        return int(self.req_row_ptr[-1])

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.head_dim)

    @property
    def seg_elems(self) -> int:
        return self.seg_len * self.kv_heads * self.head_dim

    def prefix_tokens(self) -> np.ndarray:
        """Valid prefix tokens of each request."""
        fill_of = dict(zip(self.pool_ids.tolist(), self.pool_fills.tolist()))
        out = np.zeros(self.n_req, np.int64)
        for r in range(self.n_req):
            ids = self.seg_ids[self.req_seg_ptr[r]:self.req_seg_ptr[r + 1]]
            out[r] = sum(fill_of[int(s)] for s in ids)
        return out

    # ---- tensor values -------------------------------------------------------------
    def _rows(self, stream: int, heads: int, t0: int, t1: int, device, gain: float = 1.0):
        per = heads * self.head_dim
        x = normal_bf16_range(self.seed, stream, (self.row_base + t0) * per, (t1 - t0) * per, device)
        x = x.view(t1 - t0, heads, self.head_dim)
        return x * gain if gain != 1.0 else x

    def q(self, device="cpu", t0: int = 0, t1: Optional[int] = None):
        return self._rows(STREAM_Q, self.q_heads, t0, self.n_tokens if t1 is None else t1, device)

    def k_new(self, device="cpu", t0: int = 0, t1: Optional[int] = None):
        return self._rows(STREAM_KNEW, self.kv_heads, t0, self.n_tokens if t1 is None else t1, device,
                          self.k_gain)

    def v_new(self, device="cpu", t0: int = 0, t1: Optional[int] = None):
        return self._rows(STREAM_VNEW, self.kv_heads, t0, self.n_tokens if t1 is None else t1, device)

    def segment_kv(self, ids, device="cpu"):
        """K, V contents of the given segment ids: bf16 [n, seg_len, kv_heads, head_dim] each.
        Contents depend on the id only (never on the slot), so placement and deduplication
        cannot change them.  All seg_len tokens are generated; tokens beyond a segment's
        fill are simply never stored."""
        ids_t = torch.as_tensor(np.asarray(ids, dtype=np.uint64).view(np.int64), device=device)
        e = self.seg_elems
        idx = ids_t[:, None] * e + torch.arange(e, dtype=torch.int64, device=device)[None, :]
        shape = (len(ids_t), self.seg_len, self.kv_heads, self.head_dim)
        k = normal_bf16(self.seed, STREAM_POOL_K, idx).view(shape)
        v = normal_bf16(self.seed, STREAM_POOL_V, idx).view(shape)
        if self.k_gain != 1.0:
            k = k * self.k_gain
        if self.k_boost:
            lo, hi, gain = self.k_boost
            pos = ids_t & 0xFFFFFFFF
            boosted = ((pos >= lo) & (pos < hi))[:, None, None, None]
            k = torch.where(boosted, k * gain, k)
        if self.v_offset_mod > 0:
            off = (ids_t % self.v_offset_mod - self.v_offset_mod // 2).to(torch.float32)
            v = (v.to(torch.float32) + off[:, None, None, None]).to(torch.bfloat16)
        return k, v

    def fill_pool(self, pool_k: torch.Tensor, pool_v: torch.Tensor, slots_per_chunk: int = 32):
        """Write every resident segment into its slot of pool_k/pool_v
        ([n_slots, seg_len, kv_heads, head_dim] bf16, any device).  Tokens at or beyond a
        segment's fill are left as they are (callers poison or zero them as they wish)."""
        dev = pool_k.device
        n = len(self.pool_ids)
        for c0 in range(0, n, slots_per_chunk):
            c1 = min(n, c0 + slots_per_chunk)
            k, v = self.segment_kv(self.pool_ids[c0:c1], dev)
            fills = torch.as_tensor(self.pool_fills[c0:c1], device=dev)
            slots = torch.as_tensor(self.pool_slots[c0:c1].astype(np.int64), device=dev)
            if bool((fills == self.seg_len).all()):
                pool_k[slots] = k
                pool_v[slots] = v
            else:
                keep = (torch.arange(self.seg_len, device=dev)[None, :] < fills[:, None])[:, :, None, None]
                pool_k[slots] = torch.where(keep, k, pool_k[slots])
                pool_v[slots] = torch.where(keep, v, pool_v[slots])


# --------------------------------------------------------------------------------------
def _place(rng: np.random.Generator, n_slots: int, n: int) -> np.ndarray:
    """n distinct slots in seeded random order."""
    if n > n_slots:
        raise ValueError("pool too small: %d segments, %d slots" % (n, n_slots))
    return rng.permutation(n_slots)[:n].astype(np.int32)


def _private_id(req: int, pos: int) -> int:
    return ((req + 1) << 32) | pos


def _finish(name, seed, hq, hkv, seg_len, n_slots, new_tokens, lists, fills_by_id, rng, **kw) -> Batch:
    row_ptr = np.zeros(len(new_tokens) + 1, np.int32)
    row_ptr[1:] = np.cumsum(new_tokens)
    seg_ptr = np.zeros(len(lists) + 1, np.int32)
    seg_ptr[1:] = np.cumsum([len(l) for l in lists])
    seg_ids = np.array([s for l in lists for s in l], dtype=np.uint64)
    uniq = list(dict.fromkeys(int(s) for s in seg_ids))          # first-seen order
    pool_ids = np.array(uniq, dtype=np.uint64)
    pool_slots = _place(rng, n_slots, len(uniq))
    pool_fills = np.array([fills_by_id.get(s, seg_len) for s in uniq], dtype=np.int32)
    return Batch(name=name, seed=seed, q_heads=hq, kv_heads=hkv, seg_len=seg_len, n_slots=n_slots,
                 req_row_ptr=row_ptr, req_seg_ptr=seg_ptr, seg_ids=seg_ids, pool_ids=pool_ids,
                 pool_slots=pool_slots, pool_fills=pool_fills, **kw)


def _lists_from_lengths(lengths, seg_len, n_shared=0):
    """Per-request id lists for prefix lengths in tokens.  The first n_shared list positions
    are ids common to all requests; the last segment of a request may be partly filled."""
    lists, fills = [], {}
    for r, L in enumerate(lengths):
        n = -(-int(L) // seg_len)
        ids = []
        for p in range(n):
            sid = p if p < n_shared else _private_id(r, p)
            ids.append(sid)
        tail = int(L) - (n - 1) * seg_len
        if n and tail < seg_len:
            if n - 1 < n_shared:                  # never shorten a shared segment
                ids[-1] = _private_id(r, n - 1)
            fills[ids[-1]] = tail
        lists.append(ids)
    return lists, fills


def tiny(seed: int = 0, **kw) -> Batch:
    """1 request, 8 q-heads / 2 kv-heads, 512-token prefix = 4 segments of 128 in an 8-slot pool
    (random slots), 32 new tokens with a causal self block."""
    rng = np.random.Generator(np.random.PCG64(seed))
    lists, fills = _lists_from_lengths([512], 128)
    return _finish("tiny", seed, 8, 2, 128, 8, [32], lists, fills, rng, **kw)


def prefill(seed: int = 1, n_req: int = 16, new_tokens: int = 512, lo: int = 8192, hi: int = 32768,
            seg_len: int = 256, n_slots: int = 4096, n_shared: int = 8, hq: int = 32, hkv: int = 8,
            **kw) -> Batch:
    """Chunked-prefill batch, Llama-3-8B layer shape: prefix lengths uniform in [lo, hi] tokens
    (not rounded to segments), the first n_shared segments common to all requests."""
    rng = np.random.Generator(np.random.PCG64(seed))
    lengths = rng.integers(lo, hi + 1, size=n_req)
    lists, fills = _lists_from_lengths(lengths, seg_len, n_shared)
    return _finish("prefill", seed, hq, hkv, seg_len, n_slots, [new_tokens] * n_req, lists, fills, rng, **kw)


def decode(seed: int = 2, n_req: int = 256, median: int = 16384, sigma: float = 1.0, cap: int = 131072,
           seg_len: int = 256, hq: int = 64, hkv: int = 8, n_slots: Optional[int] = None, **kw) -> Batch:
    """Decode batch, 70B layer shape: one query token per request, prefix lengths lognormal
    (median `median`, shape `sigma`), clamped to [1, cap]; every segment private."""
    rng = np.random.Generator(np.random.PCG64(seed))
    lengths = np.clip(np.rint(rng.lognormal(math.log(median), sigma, size=n_req)), 1, cap).astype(np.int64)
    lists, fills = _lists_from_lengths(lengths, seg_len)
    n_seg = sum(len(l) for l in lists)
    if n_slots is None:
        n_slots = max(8, 1 << int(math.ceil(math.log2(n_seg))))
    return _finish("decode", seed, hq, hkv, seg_len, n_slots, [1] * n_req, lists, fills, rng, **kw)


def longctx(seed: int = 3, n_req: int = 4, entries: int = 256, new_tokens: int = 2048, seg_len: int = 512,
            n_ids: int = 1000, zipf_s: float = 1.1, hq: int = 32, hkv: int = 8,
            n_slots: Optional[int] = None, **kw) -> Batch:
    """Long-context batch: each request's 128k-token prefix is `entries` segments drawn with
    replacement from n_ids distinct segments with finite-Zipf(s) popularity; duplicates share
    one pool slot."""
    rng = np.random.Generator(np.random.PCG64(seed))
    p = 1.0 / np.arange(1, n_ids + 1, dtype=np.float64) ** zipf_s
    p /= p.sum()
    lists = [[int(x) for x in rng.choice(n_ids, size=entries, p=p)] for _ in range(n_req)]
    if n_slots is None:
        n_slots = n_ids
    return _finish("longctx", seed, hq, hkv, seg_len, n_slots, [new_tokens] * n_req, lists, {}, rng, **kw)


def multiturn(seed: int = 4, turn: int = 0, n_sessions: int = 64, shared_segments: int = 16,
              growth_segments: int = 4, new_tokens: int = 256, seg_len: int = 256, hq: int = 32, hkv: int = 8,
              n_slots: int = 4096, n_turns: int = 8, **kw) -> Batch:
    """Turn `turn` (0-based) of the multi-turn heavy-hitter workload: every session's prefix is
    the shared system prompt (shared_segments) followed by growth_segments*turn private
    history segments; the new tokens of all sessions form one batch.  Slot placement is drawn
    once for the final turn's pool, so a segment keeps its slot from turn to turn."""
    rng = np.random.Generator(np.random.PCG64(seed))
    all_ids = list(range(shared_segments))
    for s in range(n_sessions):
        all_ids += [_private_id(s, shared_segments + p) for p in range(growth_segments * (n_turns - 1))]
    slot_of = dict(zip(all_ids, _place(rng, n_slots, len(all_ids)).tolist()))
    lists = [list(range(shared_segments)) +
             [_private_id(s, shared_segments + p) for p in range(growth_segments * turn)]
             for s in range(n_sessions)]
    b = _finish("multiturn[t=%d]" % turn, seed, hq, hkv, seg_len, n_slots, [new_tokens] * n_sessions,
                lists, {}, rng, **kw)
    b.pool_slots = np.array([slot_of[int(s)] for s in b.pool_ids], dtype=np.int32)
    b.row_base = turn * n_sessions * new_tokens
    return b


WORKLOADS = {"tiny": tiny, "prefill": prefill, "decode": decode, "longctx": longctx, "multiturn": multiturn}
