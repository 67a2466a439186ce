"""fp64 CPU oracle for TokenLake's cache-aware operation (segment-level prefix attention).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition that the GPU library is
checked against.  Nothing on the product path may import it; it shares no code with the HIP
kernels or their host library and uses numpy only.

What it defines (paper: Background / "LLM serving systems", and Section 4 opening paragraph on
segment independence):

* a request's new query tokens attend (i) to the whole prefix cache, which is stored as
  fixed-size segments in pool slots, and (ii) causally to the new tokens' own K/V;
* each segment (or any subset of keys) yields a partial output plus a normalizer; partials are
  combined into exactly the output of one softmax over all keys.

The exact result has a plain definition -- softmax attention over the concatenation of the
prefix keys and the visible new keys -- so `request_attention` is that definition written
out.  `partial_attention` is the same definition restricted to a subset of keys and
`merge_partials` is the recombination rule; the identity "merge of partials == full softmax"
is therefore a test *of this file*, not an assumption.

Readings the paper leaves open (all fixed by the build's problem statement):
  - normalizer = natural-log log-sum-exp of the scaled scores;
  - q-head h reads kv-head h // (q_heads // kv_heads);
  - a slot holds `fill` valid tokens (1..seg_len); tokens at or beyond `fill` do not exist;
  - a new token i sees new tokens 0..i (inclusive) and every prefix token;
  - a slot listed twice contributes twice (multiset concatenation);
  - no keys at all -> O = 0, LSE = -inf (never NaN).

All floating-point work is fp64 on values converted exactly from bf16 bit patterns.
Parity pins: tests/test_oracle_pins.py (hand-expanded tiny cases, closed forms, invariants,
brute-force loops, scipy cross-checks).  No function here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "bf16_bits_to_f64",
    "SlotTable",
    "gather_segments",
    "append_rows",
    "segment_loads",
    "PrefixTree",
    "attention_rows",
    "partial_attention",
    "merge_partials",
    "request_attention",
    "request_partials_by_segment",
]


# --------------------------------------------------------------------------------------
# bf16 bit patterns -> exact fp64
# --------------------------------------------------------------------------------------
def bf16_bits_to_f64(bits) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns (uint16) to float64.

    bfloat16 is the upper half of an IEEE binary32, so the value is obtained by placing the
    16 bits in the high half of a 32-bit word; binary32 -> binary64 is exact.
    """
    b = np.ascontiguousarray(bits)
    if b.dtype != np.uint16:
        raise TypeError("expected uint16 bf16 bit patterns, got %s" % b.dtype)
    as32 = b.astype(np.uint32) << np.uint32(16)
    return as32.view(np.float32).astype(np.float64)


# --------------------------------------------------------------------------------------
# segment table and gather (integer work; must be reproduced bit-exactly by the library)
# --------------------------------------------------------------------------------------
class SlotTable:
    """segment_id -> (slot, fill).  One copy per id (deduplication, paper Section 1 / 3.1).

    Putting an id that is already present returns the existing slot and stores nothing.
    A new id takes `want_slot` if given (must be free), else the lowest-numbered free slot.

    Life cycle (paper Section 4.3, "Replicated segment selection and eviction": eviction is
    global LRU on the recorded last access time).  Every resident segment has a count of holders
    and a last-access time on a logical clock that ticks once per access event:
      put of a new id        count = 1, accessed
      put of a resident id   count + 1, accessed
      touch(ids)             one event for a whole batch of ids (a plan naming them): all get the same time
      append into a tail     the tail is accessed
      release(id)            count - 1 (the segment stays resident and usable)
      evict_lru()            among segments with count 0, the one accessed longest ago leaves and
                             its slot becomes free; equal times (same touch) -> the lowest slot
    Where the paper is silent (who holds a segment, ties), this is the build's reading.
    """

    def __init__(self, n_slots: int, seg_len: int):
        self.n_slots = int(n_slots)
        self.seg_len = int(seg_len)
        self._slot_of = {}
        self._fill = np.zeros(self.n_slots, dtype=np.int32)
        self._used = np.zeros(self.n_slots, dtype=bool)
        self._id_of = {}
        self._holders = np.zeros(self.n_slots, dtype=np.int64)
        self._accessed = np.zeros(self.n_slots, dtype=np.int64)
        self._clock = 0

    def _tick(self) -> int:
        self._clock += 1
        return self._clock

    def touch(self, seg_ids):
        """One access event for all the listed (resident) ids."""
        slots = [self._slot_of[int(s)] for s in seg_ids]       # KeyError for an id that is not resident
        now = self._tick()
        for s in slots:
            self._accessed[s] = now

    def holders(self, seg_id: int) -> int:
        return int(self._holders[self._slot_of[int(seg_id)]])

    def n_used(self) -> int:
        return int(self._used.sum())

    def release(self, seg_id: int):
        seg_id = int(seg_id)
        if seg_id not in self._slot_of:
            raise KeyError("segment not in the pool")
        slot = self._slot_of[seg_id]
        if self._holders[slot] <= 0:
            raise ValueError("segment has no holder")
        self._holders[slot] -= 1

    def evict_lru(self) -> int:
        """Removes the least recently accessed segment among those nobody holds; returns its id."""
        best = -1
        for slot in range(self.n_slots):
            if self._used[slot] and self._holders[slot] == 0:
                if best < 0 or self._accessed[slot] < self._accessed[best]:
                    best = slot
        if best < 0:
            raise LookupError("no segment without holders")
        seg_id = self._id_of.pop(best)
        del self._slot_of[seg_id]
        self._used[best] = False
        self._fill[best] = 0
        return seg_id

    def put(self, seg_id: int, fill: int, want_slot: int = -1) -> int:
        seg_id = int(seg_id)
        if seg_id in self._slot_of:
            slot = self._slot_of[seg_id]
            self._holders[slot] += 1
            self._accessed[slot] = self._tick()
            return slot
        if not (1 <= fill <= self.seg_len):
            raise ValueError("fill out of range")
        if want_slot >= 0:
            if want_slot >= self.n_slots or self._used[want_slot]:
                raise ValueError("slot not free")
            slot = int(want_slot)
        else:
            free = np.flatnonzero(~self._used)
            if free.size == 0:
                raise MemoryError("pool full")
            slot = int(free[0])
        self._used[slot] = True
        self._fill[slot] = fill
        self._slot_of[seg_id] = slot
        self._id_of[slot] = seg_id
        self._holders[slot] = 1
        self._accessed[slot] = self._tick()
        return slot

    def lookup(self, seg_ids) -> np.ndarray:
        """Slot of each id, -1 for an id that is not in the pool."""
        return np.array([self._slot_of.get(int(s), -1) for s in seg_ids], dtype=np.int32)

    def fill(self, slots) -> np.ndarray:
        return self._fill[np.asarray(slots, dtype=np.int64)]

    def append(self, tail_id, new_ids, n_rows: int):
        """Placement of n_rows new token rows at the end of a chain of segments (paper Section
        3.2: the KV of new tokens is `put` into the pool, so that later turns find it as prefix).

        The rows go, in order, first to the slot of `tail_id` from its current fill up to
        seg_len (tail_id None: there is no partly filled tail), then to new segments
        `new_ids` in order, seg_len rows each, the last one possibly partly filled.  Each new
        id takes the lowest-numbered free slot at the moment it is created.  `new_ids` must
        be exactly as many ids as the rows need.  Returns [(slot, first_token, n_tokens,
        first_row), ...]; nothing changes if an argument is invalid.
        """
        n_rows = int(n_rows)
        if n_rows < 0:
            raise ValueError("negative row count")
        new_ids = [int(x) for x in new_ids]
        room = 0
        if tail_id is not None:
            tail_id = int(tail_id)
            if tail_id not in self._slot_of:
                raise KeyError("tail segment not in the pool")
            if self._holders[self._slot_of[tail_id]] != 1:
                raise ValueError("a tail with other holders (or none) does not grow")
            room = self.seg_len - int(self._fill[self._slot_of[tail_id]])
        rest = max(0, n_rows - room)
        need = -(-rest // self.seg_len)
        if len(new_ids) != need:
            raise ValueError("need exactly %d new ids, got %d" % (need, len(new_ids)))
        if len(set(new_ids)) != len(new_ids) or any(i in self._slot_of for i in new_ids):
            raise ValueError("new id repeated or already in the pool")
        if int((~self._used).sum()) < need:
            raise MemoryError("pool full")
        out, row = [], 0
        if tail_id is not None and n_rows > 0 and room > 0:
            slot = self._slot_of[tail_id]
            n = min(room, n_rows)
            out.append((slot, int(self._fill[slot]), n, 0))
            self._fill[slot] += n
            self._accessed[slot] = self._tick()
            row = n
        for sid in new_ids:
            n = min(self.seg_len, n_rows - row)
            slot = self.put(sid, n)
            out.append((slot, 0, n, row))
            row += n
        return out


def gather_segments(pool_k_bits, pool_v_bits, slots, fills):
    """Concatenate, in list order, the valid tokens of the listed slots.

    pool_*_bits: uint16 [n_slots, seg_len, kv_heads, head_dim] (bf16 bit patterns).
    Returns (K_bits, V_bits), each uint16 [sum(fills), kv_heads, head_dim].
    """
    slots = np.asarray(slots, dtype=np.int64)
    fills = np.asarray(fills, dtype=np.int64)
    if slots.shape != fills.shape:
        raise ValueError("slots/fills mismatch")
    n_slots, seg_len = pool_k_bits.shape[0], pool_k_bits.shape[1]
    ks, vs = [], []
    for s, f in zip(slots, fills):
        if not (0 <= s < n_slots) or not (0 <= f <= seg_len):
            raise IndexError("bad slot or fill")
        ks.append(pool_k_bits[s, :f])
        vs.append(pool_v_bits[s, :f])
    if not ks:
        shp = (0,) + tuple(pool_k_bits.shape[2:])
        return np.zeros(shp, np.uint16), np.zeros(shp, np.uint16)
    return np.concatenate(ks, axis=0), np.concatenate(vs, axis=0)


def segment_loads(req_lists, req_new_tokens):
    """Load of every listed segment (paper Section 4.3: accesses concentrate on segments near the
    root of the prefix tree): the number of new tokens whose request lists it, an id listed
    twice by a request counting twice.  Returns [(id, load), ...] by decreasing load; equal
    loads keep the order of first appearance (requests in order, each list front to back)."""
    load = {}
    for ids, n in zip(req_lists, req_new_tokens):
        for s in ids:
            load[int(s)] = load.get(int(s), 0) + int(n)      # dicts keep insertion order
    return sorted(load.items(), key=lambda kv: -kv[1])          # sorted() is stable


class PrefixTree:
    """The prefix tree over the requests' segment lists, by brute force (paper Section 3.1: a global
    prefix tree indexes the cache segments; Section 4.3: a segment is accessed only when its prefix
    is, so accesses concentrate near the root, and heavy hitters are found from the root).

    A node is the tuple of segment ids from the root down to it; the same id under two different
    prefixes is two nodes.  Every request that walks its list from the root adds its number of new
    tokens to the load of each node on the way, so a node's load never exceeds its parent's.
    Nodes are kept in a dict in order of creation.  `walk` returns the batch's own loads, nodes in
    order of first visit (requests in order, each list front to back).  `hot` sorts by decreasing
    load, equal loads in order of creation (batch: of first visit): a parent, which is at least as
    loaded and older than its children, always comes before them.  `evict(id)` removes every node
    of that id together with everything below it (a prefix with a hole cannot be used).
    """

    def __init__(self):
        self.load = {}

    def walk(self, req_lists, req_new_tokens):
        batch = {}
        for ids, n in zip(req_lists, req_new_tokens):
            path = ()
            for s in ids:
                path = path + (int(s),)
                self.load[path] = self.load.get(path, 0) + int(n)
                batch[path] = batch.get(path, 0) + int(n)
        return batch

    @staticmethod
    def ranked(loads, k=None):
        """[(path, load), ...] by decreasing load; equal loads keep the dict's order."""
        out = sorted(loads.items(), key=lambda kv: -kv[1])          # sorted() is stable
        return out if k is None else out[:k]

    def hot(self, k=None):
        return self.ranked(self.load, k)

    def evict(self, seg_id: int):
        seg_id = int(seg_id)
        for path in [p for p in self.load if seg_id in p]:
            del self.load[path]

    def n_nodes(self) -> int:
        return len(self.load)


FNV64_OFFSET = 0xCBF29CE484222325
FNV64_PRIME = 0x100000001B3


def fnv1a64(data: bytes, start: int = FNV64_OFFSET) -> int:
    """64-bit FNV-1a of a byte string (the published algorithm: xor the byte in, multiply by the prime,
    modulo 2^64), from the given starting value."""
    h = start
    for b in data:
        h = ((h ^ b) * FNV64_PRIME) & 0xFFFFFFFFFFFFFFFF
    return h


def content_segment_ids(tokens, seg_len: int, salt: int = 0):
    """Segment ids derived from what the segments hold (paper Section 3.1: the global prefix tree is keyed
    by the token sequence, so that requests name the same cached segment exactly as far as their prompts
    agree).  Segment k of a sequence covers tokens [k seg_len, min(n, (k+1) seg_len)); its id is the FNV-1a
    hash of ALL tokens up to its end (each token as four little-endian bytes), started from the offset basis
    xor `salt` (one salt per model / layer group).  Written as that definition: every id from scratch."""
    toks = [int(t) for t in tokens]
    n = len(toks)
    ids = []
    for k in range((n + seg_len - 1) // seg_len):
        end = min(n, (k + 1) * seg_len)
        data = b"".join((t & 0xFFFFFFFF).to_bytes(4, "little") for t in toks[:end])
        ids.append(fnv1a64(data, FNV64_OFFSET ^ (salt & 0xFFFFFFFFFFFFFFFF)))
    return ids


def append_rows(pool_k_bits, pool_v_bits, table: SlotTable, tail_id, new_ids, k_rows_bits, v_rows_bits):
    """Store new token rows [n, kv_heads, head_dim] (bf16 bit patterns) at the end of a chain
    of segments: `table.append` decides where each row goes, the rows are copied there.
    Returns the placement list of `table.append`."""
    if k_rows_bits.shape != v_rows_bits.shape or k_rows_bits.shape[1:] != pool_k_bits.shape[2:]:
        raise ValueError("row shape mismatch")
    placement = table.append(tail_id, new_ids, k_rows_bits.shape[0])
    for slot, tok, n, row in placement:
        pool_k_bits[slot, tok:tok + n] = k_rows_bits[row:row + n]
        pool_v_bits[slot, tok:tok + n] = v_rows_bits[row:row + n]
    return placement


# --------------------------------------------------------------------------------------
# softmax attention, one head
# --------------------------------------------------------------------------------------
def attention_rows(q, k, v, scale, n_visible=None):
    """Exact softmax attention of query rows over keys, one head, fp64.

    q [nq, d], k [nk, d], v [nk, dv] float64.  `n_visible[i]` (optional) = number of
    leading keys row i may see (used for the causal block); default: all nk.

    s_ij = scale * <q_i, k_j>;  M_i = max_j s_ij;  Z_i = sum_j exp(s_ij - M_i)
    LSE_i = M_i + ln Z_i;       O_i = sum_j exp(s_ij - LSE_i) v_j
    Rows with no visible key give O = 0, LSE = -inf.
    """
    q = np.asarray(q, np.float64)
    k = np.asarray(k, np.float64)
    v = np.asarray(v, np.float64)
    nq, nk = q.shape[0], k.shape[0]
    out = np.zeros((nq, v.shape[1] if v.ndim == 2 else 0), np.float64)
    lse = np.full(nq, -np.inf, np.float64)
    if nq == 0 or nk == 0:
        return out, lse
    s = (q @ k.T) * float(scale)
    if n_visible is not None:
        nvis = np.asarray(n_visible, np.int64)
        hidden = np.arange(nk)[None, :] >= nvis[:, None]
        s = np.where(hidden, -np.inf, s)
    m = s.max(axis=1)
    live = np.isfinite(m)
    m_safe = np.where(live, m, 0.0)
    p = np.exp(s - m_safe[:, None])          # exp(-inf) = 0 for hidden keys
    z = p.sum(axis=1)
    with np.errstate(divide="ignore"):
        lse = np.where(live, m_safe + np.log(np.where(live, z, 1.0)), -np.inf)
    o = (p @ v) / np.where(live, z, 1.0)[:, None]
    out = np.where(live[:, None], o, 0.0)
    return out, lse


def _group(q_heads: int, kv_heads: int) -> int:
    if kv_heads <= 0 or q_heads % kv_heads:
        raise ValueError("q_heads must be a multiple of kv_heads")
    return q_heads // kv_heads


def partial_attention(q_bits, k_bits, v_bits, scale, n_visible=None):
    """Partial attention of every (token, q-head) row over one set of keys.

    q_bits [n_tok, q_heads, d], k_bits/v_bits [n_keys, kv_heads, d] (uint16 bf16 bits).
    Returns O [n_tok, q_heads, d] and LSE [n_tok, q_heads] in fp64.
    """
    q = bf16_bits_to_f64(q_bits)
    k = bf16_bits_to_f64(k_bits)
    v = bf16_bits_to_f64(v_bits)
    n_tok, hq, d = q.shape
    hkv = k.shape[1]
    g = _group(hq, hkv)
    out = np.zeros((n_tok, hq, d), np.float64)
    lse = np.full((n_tok, hq), -np.inf, np.float64)
    for h in range(hq):
        o_h, l_h = attention_rows(q[:, h, :], k[:, h // g, :], v[:, h // g, :], scale, n_visible)
        out[:, h, :] = o_h
        lse[:, h] = l_h
    return out, lse


# --------------------------------------------------------------------------------------
# recombination of partials
# --------------------------------------------------------------------------------------
def merge_partials(outs, lses):
    """Combine partial (O_j, LSE_j) pairs into the result of one softmax over all their keys.

    outs [n, ..., d], lses [n, ...].  With M = max_j LSE_j and w_j = exp(LSE_j - M):
        O = sum_j w_j O_j / sum_j w_j,      LSE = M + ln sum_j w_j.
    A partial with LSE = -inf has weight 0; if all are -inf the result is O = 0, LSE = -inf.
    """
    outs = np.asarray(outs, np.float64)
    lses = np.asarray(lses, np.float64)
    if outs.shape[0] == 0:
        return np.zeros(outs.shape[1:], np.float64), np.full(lses.shape[1:], -np.inf)
    m = lses.max(axis=0)
    live = np.isfinite(m)
    m_safe = np.where(live, m, 0.0)
    w = np.exp(lses - m_safe)                 # [n, ...]
    w = np.where(np.isfinite(lses), w, 0.0)
    wsum = w.sum(axis=0)
    wsum_safe = np.where(live, wsum, 1.0)
    o = (w[..., None] * outs).sum(axis=0) / wsum_safe[..., None]
    o = np.where(live[..., None], o, 0.0)
    with np.errstate(divide="ignore"):
        lse = np.where(live, m_safe + np.log(wsum_safe), -np.inf)
    return o, lse


# --------------------------------------------------------------------------------------
# one request: prefix segments + causal new tokens
# --------------------------------------------------------------------------------------
def request_attention(q_bits, pool_k_bits, pool_v_bits, slots, fills, knew_bits, vnew_bits, scale):
    """Full attention output of one request's new tokens (the definition).

    Keys of new token i = [valid tokens of the listed slots, in order] ++ new tokens 0..i.
    q_bits [Lq, q_heads, d]; knew/vnew_bits [Lq, kv_heads, d]; pool as in gather_segments.
    Pass knew_bits=None to leave the self block out (prefix-only attention).
    Returns O [Lq, q_heads, d], LSE [Lq, q_heads] (fp64).
    """
    pk, pv = gather_segments(pool_k_bits, pool_v_bits, slots, fills)
    n_prefix = pk.shape[0]
    lq = q_bits.shape[0]
    if knew_bits is None:
        return partial_attention(q_bits, pk, pv, scale)
    k_all = np.concatenate([pk, knew_bits], axis=0)
    v_all = np.concatenate([pv, vnew_bits], axis=0)
    n_vis = n_prefix + np.arange(1, lq + 1)
    return partial_attention(q_bits, k_all, v_all, scale, n_visible=n_vis)


def request_partials_by_segment(q_bits, pool_k_bits, pool_v_bits, slots, fills, knew_bits, vnew_bits,
                                scale, groups=None):
    """Partials of one request, piece by piece, for the merge identity and for checking the
    library's per-item partials.

    `groups` is a list of index lists into `slots` (default: one group per list entry).  The
    causal self block, if knew_bits is given, is appended as the last partial.
    Returns (outs [n_parts, Lq, q_heads, d], lses [n_parts, Lq, q_heads]).
    """
    slots = np.asarray(slots, np.int64)
    fills = np.asarray(fills, np.int64)
    if groups is None:
        groups = [[i] for i in range(len(slots))]
    outs, lses = [], []
    for grp in groups:
        grp = np.asarray(grp, np.int64)
        pk, pv = gather_segments(pool_k_bits, pool_v_bits, slots[grp], fills[grp])
        o, l = partial_attention(q_bits, pk, pv, scale)
        outs.append(o)
        lses.append(l)
    if knew_bits is not None:
        lq = q_bits.shape[0]
        o, l = partial_attention(q_bits, knew_bits, vnew_bits, scale, n_visible=np.arange(1, lq + 1))
        outs.append(o)
        lses.append(l)
    return np.stack(outs), np.stack(lses)
