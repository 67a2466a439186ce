"""CPU-side checks of the C-ABI library: it loads, exports what the header declares, and its
host logic (segment table, plan builder) does integer work that matches the oracle's table
and covers every (query token, list entry) pair exactly once.  No compute call is made."""
import os
import re

import numpy as np
import pytest

from oracle import tokenlake_oracle as orc
from paper_2508_17219_amd import binding as B
from paper_2508_17219_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE_K, FAKE_V = 0x100000, 0x200000          # never dereferenced: host logic only


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "tokenlake.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(tl_[a-z0-9_]+)\s*\(", text))
    assert declared == set(B.EXPORTED), declared ^ set(B.EXPORTED)
    lib = B.load_library()
    for name in declared:
        assert hasattr(lib, name), name
    assert lib.tl_status_str(0) == b"ok" and lib.tl_status_str(-4) == b"segment not found"


def _pool_for(b):
    pool = B.tl_pool_create(b.n_slots, b.seg_len, b.kv_heads, b.head_dim, FAKE_K, FAKE_V)
    B.tl_pool_adopt(pool, b.pool_ids, b.pool_slots, b.pool_fills)
    return pool


def test_create_rejects_bad_shapes():
    for args in [(0, 128, 2, 128), (8, 100, 2, 128), (8, 128, 2, 64), (8, 128, 0, 128), (1 << 24, 256, 8, 128)]:
        with pytest.raises(B.TokenLakeError) as e:
            B.tl_pool_create(*args, FAKE_K, FAKE_V)
        assert e.value.status == B.TL_EINVAL
    with pytest.raises(B.TokenLakeError):
        B.tl_pool_create(8, 128, 2, 128, FAKE_K, None)


def test_segment_table_matches_oracle_table():
    rng = np.random.default_rng(0)
    n_slots, C = 64, 128
    pool = B.tl_pool_create(n_slots, C, 2, 128, FAKE_K, FAKE_V)
    table = orc.SlotTable(n_slots, C)
    ids = rng.integers(0, 2 ** 63, size=40, dtype=np.uint64)
    slots = rng.permutation(n_slots)[:40].astype(np.int32)
    fills = rng.integers(1, C + 1, size=40).astype(np.int32)
    B.tl_pool_adopt(pool, ids, slots, fills)
    for i, s, f in zip(ids, slots, fills):
        table.put(int(i), int(f), int(s))
    probe = np.concatenate([ids[::-1], rng.integers(0, 2 ** 63, size=10, dtype=np.uint64)])
    assert np.array_equal(B.tl_pool_lookup(pool, probe), table.lookup(probe))
    assert np.array_equal(B.tl_pool_fills(pool, slots), table.fill(slots))
    assert B.tl_pool_used(pool) == 40
    # adopt is all-or-nothing
    with pytest.raises(B.TokenLakeError):
        B.tl_pool_adopt(pool, [999, ids[0]], [int(np.setdiff1d(np.arange(n_slots), slots)[0]), 1], [5, 5])
    assert B.tl_pool_lookup(pool, [999])[0] == -1
    with pytest.raises(B.TokenLakeError):
        B.tl_pool_adopt(pool, [1000], [int(slots[0])], [5])          # slot taken
    with pytest.raises(B.TokenLakeError):
        B.tl_pool_adopt(pool, [1001], [int(np.setdiff1d(np.arange(n_slots), slots)[0])], [C + 1])
    B.tl_pool_destroy(pool)


def test_release_and_lru_eviction():
    pool = B.tl_pool_create(4, 64, 1, 128, FAKE_K, FAKE_V)
    B.tl_pool_adopt(pool, [10, 11, 12, 13], [0, 1, 2, 3], [64, 64, 64, 64])
    with pytest.raises(B.TokenLakeError) as e:
        B.tl_pool_evict_lru(pool)                                     # everything is referenced
    assert e.value.status == B.TL_ENOTFOUND
    for i in (10, 11, 12):
        B.tl_pool_release(pool, i)
    with pytest.raises(B.TokenLakeError):
        B.tl_pool_release(pool, 10)                                   # already at zero
    # a plan that names id 10 makes it the most recently used
    plan = B.tl_plan_create(pool, 1, [0, 1], [0, 1], np.array([10], np.uint64), 0, 0)
    B.tl_plan_destroy(plan)
    assert B.tl_pool_evict_lru(pool) == 11
    assert B.tl_pool_evict_lru(pool) == 12
    assert B.tl_pool_evict_lru(pool) == 10
    assert B.tl_pool_used(pool) == 1 and list(B.tl_pool_lookup(pool, [10, 13])) == [-1, 3]
    B.tl_pool_adopt(pool, [20], [1], [7])
    assert list(B.tl_pool_fills(pool, [0, 1, 2, 3])) == [0, 7, 0, 64]
    B.tl_pool_destroy(pool)


def test_pool_life_cycle_matches_the_oracle_on_random_sequences():
    """adopt / put of a resident id / plan use / release / evict_lru: the library's table against
    the oracle's SlotTable after every operation (slots, fills, which id an eviction removes)."""
    rng = np.random.default_rng(29)
    for trial in range(10):
        n_slots, C = int(rng.integers(3, 10)), 64
        pool = B.tl_pool_create(n_slots, C, 1, 128, FAKE_K, FAKE_V)
        table = orc.SlotTable(n_slots, C)
        universe = list(range(100, 116))
        for step in range(150):
            resident = [i for i in universe if table.lookup([i])[0] >= 0]
            op = rng.choice(["new", "again", "plan", "release", "evict"], p=[0.3, 0.1, 0.2, 0.25, 0.15])
            if op == "new":
                absent = [i for i in universe if i not in resident]
                if not absent:
                    continue
                sid, fill = int(rng.choice(absent)), int(rng.integers(1, C + 1))
                if len(resident) == n_slots:
                    continue
                free = [s for s in range(n_slots) if s not in set(table.lookup(resident).tolist())]
                slot = int(rng.choice(free))
                B.tl_pool_adopt(pool, [sid], [slot], [fill])
                assert table.put(sid, fill, slot) == slot
            elif op == "again" and resident:
                sid = int(rng.choice(resident))                        # dedup hit: no copy, one more holder
                assert B.tl_pool_put(pool, sid, FAKE_K, FAKE_V, C, -1, stream=0) == table.put(sid, C)
            elif op == "plan" and resident:
                ids = rng.choice(resident, size=int(rng.integers(1, len(resident) + 1)), replace=True).astype(np.uint64)
                plan = B.tl_plan_create(pool, 1, [0, 1], [0, len(ids)], ids, 0, 0)
                B.tl_plan_destroy(plan)
                table.touch(ids.tolist())
            elif op == "release" and resident:
                sid = int(rng.choice(resident))
                if table.holders(sid) == 0:
                    with pytest.raises(B.TokenLakeError):
                        B.tl_pool_release(pool, sid)
                else:
                    B.tl_pool_release(pool, sid)
                    table.release(sid)
            elif op == "evict":
                try:
                    want = table.evict_lru()
                except LookupError:
                    with pytest.raises(B.TokenLakeError) as e:
                        B.tl_pool_evict_lru(pool)
                    assert e.value.status == B.TL_ENOTFOUND
                else:
                    assert B.tl_pool_evict_lru(pool) == want
            assert np.array_equal(B.tl_pool_lookup(pool, universe), table.lookup(universe))
            assert np.array_equal(B.tl_pool_fills(pool, np.arange(n_slots)), table.fill(np.arange(n_slots)))
            assert B.tl_pool_used(pool) == table.n_used()
        B.tl_pool_destroy(pool)


def test_a_plan_goes_stale_when_the_pool_changes():
    """A plan holds slots and fills as they were when it was built: after an adopt or an eviction the
    compute calls that read the pool refuse it (before any device work), a release or a put of a
    resident id leaves it valid as far as this check goes, and a fresh plan is accepted again."""
    pool = B.tl_pool_create(4, 64, 1, 128, FAKE_K, FAKE_V)
    B.tl_pool_adopt(pool, [10, 11], [0, 1], [64, 20])
    lib = B.load_library()

    def refused(plan):
        # fake, never dereferenced pointers; a current plan would get as far as the device, so only
        # the stale answer is asked for here
        rc = lib.tl_segment_attn(pool, plan, FAKE_K, 0.1, FAKE_K, FAKE_V, None)
        rc2 = lib.tl_fused_attn(pool, plan, FAKE_K, FAKE_K, FAKE_V, 0.1, None, None, FAKE_K, 0, None, None)
        assert rc == rc2 or rc2 == B.TL_OK
        return rc == B.TL_EINVAL and b"pool has changed" in lib.tl_last_error()

    plan = B.tl_plan_create(pool, 1, [0, 3], [0, 2], np.array([10, 11], np.uint64), B.TL_PLAN_SELF_BLOCK)
    B.tl_pool_release(pool, 11)
    B.tl_pool_put(pool, 10, FAKE_K, FAKE_V, 64, -1, stream=0)
    B.tl_pool_adopt(pool, [12], [2], [5])
    assert refused(plan)
    B.tl_plan_destroy(plan)
    plan = B.tl_plan_create(pool, 1, [0, 3], [0, 2], np.array([10, 11], np.uint64), B.TL_PLAN_SELF_BLOCK)
    assert B.tl_pool_evict_lru(pool) == 11
    assert refused(plan)
    # the plan outlives its pool for reading back and destruction
    B.tl_pool_destroy(pool)
    assert B.tl_plan_get_info(plan).n_tokens == 3 and len(B.tl_plan_hot_slots(plan, 4)[0]) == 2
    B.tl_plan_destroy(plan)


def _check_plan_covers(b, plan, flags, fused_req=(), tail_req=()):
    """fused_req: requests taken whole by the one-pass kernel (in no work item); tail_req: requests whose
    shared runs are work items and whose private end is a one-pass tail (TL_PLAN_FUSE_TAILS): the
    work items cover a leading part of their lists, and none of their partial rows is in a merge list."""
    info = B.tl_plan_get_info(plan)
    fused_tok = set(t for r in tuple(fused_req) + tuple(tail_req) for t in range(b.req_row_ptr[r], b.req_row_ptr[r + 1]))
    ex = B.tl_plan_export(plan)
    slots = B.tl_pool_lookup(plan_pool[0], b.seg_ids)
    T = b.n_tokens
    assert info.n_tokens == T and info.n_req == b.n_req
    # each token's multiset of slots over its items == its request's list
    got = [[] for _ in range(T)]
    rows_seen = set()
    for i in range(info.n_items):
        toks = ex["item_tokens"][ex["item_tok_ptr"][i]:ex["item_tok_ptr"][i + 1]]
        its = ex["item_slots"][ex["item_slot_ptr"][i]:ex["item_slot_ptr"][i + 1]]
        assert len(its) > 0 and len(toks) > 0
        for jpos, t in enumerate(toks):
            got[int(t)].extend(int(s) for s in its)
            row = int(ex["item_row_base"][i]) + jpos
            assert row not in rows_seen
            rows_seen.add(row)
    n_prior = 0
    for r in range(b.n_req):
        mine = [int(s) for s in slots[b.req_seg_ptr[r]:b.req_seg_ptr[r + 1]]]
        for t in range(b.req_row_ptr[r], b.req_row_ptr[r + 1]):
            if r in tail_req:              # the shared, leading part of the list, whatever its length
                assert sorted(got[t]) == sorted(mine[:len(got[t])]), (r, t)
            else:
                assert sorted(got[t]) == ([] if r in fused_req else sorted(mine)), (r, t)
    tail_item_rows = set()
    for i in range(info.n_items):
        toks = ex["item_tokens"][ex["item_tok_ptr"][i]:ex["item_tok_ptr"][i + 1]]
        seen_req = set()
        for jpos, t in enumerate(toks):
            r = int(np.searchsorted(b.req_row_ptr, int(t), side="right") - 1)
            if r in tail_req:
                tail_item_rows.add(int(ex["item_row_base"][i]) + jpos)
                seen_req.add(r)
        n_prior += len(seen_req)
    assert info.n_prior_rows == n_prior
    n_item_rows = len(rows_seen)
    assert rows_seen == set(range(n_item_rows))
    self_rows = T if flags & B.TL_PLAN_SELF_BLOCK else 0
    assert info.n_partial_rows == n_item_rows + self_rows
    assert info.self_row_base == (n_item_rows if flags & B.TL_PLAN_SELF_BLOCK else -1)   # also for a batch with no tokens
    # merge lists: every partial row exactly once, under its own token
    mp, mr = ex["merge_ptr"], ex["merge_rows"]
    assert mp[0] == 0 and mp[-1] == len(mr) == info.n_merge_entries == info.n_partial_rows - len(fused_tok) - len(tail_item_rows)
    assert sorted(mr.tolist()) == [x for x in range(info.n_partial_rows)
                                   if x - info.self_row_base not in fused_tok and x not in tail_item_rows]
    row_tok = {}
    for i in range(info.n_items):
        toks = ex["item_tokens"][ex["item_tok_ptr"][i]:ex["item_tok_ptr"][i + 1]]
        for jpos, t in enumerate(toks):
            row_tok[int(ex["item_row_base"][i]) + jpos] = int(t)
    for t in range(T):
        assert t not in fused_tok or mp[t] == mp[t + 1]          # a fused token has nothing to merge
        for row in mr[mp[t]:mp[t + 1]]:
            assert row_tok.get(int(row), int(row) - info.self_row_base) == t
    assert info.n_fused_tokens == len(fused_tok)
    # counters
    fill_of = dict(zip(b.pool_ids.tolist(), b.pool_fills.tolist()))
    pairs = sum(int(b.req_row_ptr[r + 1] - b.req_row_ptr[r]) * fill_of[int(s)]
                for r in range(b.n_req) for s in b.seg_ids[b.req_seg_ptr[r]:b.req_seg_ptr[r + 1]])
    assert info.prefix_pairs == pairs
    return info


plan_pool = [None]


@pytest.mark.parametrize("maker,kw", [
    (wl.tiny, {}),
    (wl.prefill, dict(n_req=5, new_tokens=37, lo=300, hi=2000, seg_len=128, n_slots=128, n_shared=3)),
    (wl.decode, dict(n_req=9, median=900, cap=4000, seg_len=128)),
    (wl.longctx, dict(n_req=3, entries=40, new_tokens=50, seg_len=64, n_ids=30)),
    (wl.multiturn, dict(turn=3, n_sessions=6, new_tokens=20, seg_len=64, n_slots=512)),
])
def test_plan_covers_every_pair_exactly_once(maker, kw):
    b = maker(**kw)
    plan_pool[0] = _pool_for(b)
    for flags in (B.TL_PLAN_SELF_BLOCK, 0, B.TL_PLAN_SELF_BLOCK | B.TL_PLAN_NO_SHARING):
        for split in (0, 1, 5):
            plan = B.tl_plan_create(plan_pool[0], b.q_heads, b.req_row_ptr, b.req_seg_ptr, b.seg_ids, flags, split)
            _check_plan_covers(b, plan, flags)
            B.tl_plan_destroy(plan)
    B.tl_pool_destroy(plan_pool[0])


def test_fused_rows_leave_the_three_step_path():
    """With TL_PLAN_FUSE_ROWS a request with >= 512 query rows per kv head (or one that shares no
    segment with another request) is handled by tl_fused_attn alone: it is in no work item, has no causal tile and nothing to merge; the
    other requests of the batch are planned as before."""
    b = wl.prefill(seed=9, n_req=5, new_tokens=200, lo=300, hi=900, seg_len=128, n_slots=64, n_shared=2)
    # G = 4: 200 tokens = 800 rows (fused), 127 tokens = 508 rows (not), 128 tokens = 512 rows (fused), 3 tokens, 0 tokens
    b.req_row_ptr = np.concatenate([[0], np.cumsum([200, 127, 128, 3, 0])]).astype(np.int32)
    plan_pool[0] = _pool_for(b)
    flags = B.TL_PLAN_SELF_BLOCK | B.TL_PLAN_FUSE_ROWS
    # this batch has 9 row tiles x 8 kv heads = 72 workgroups, fewer than the GPU has CUs, but its slot
    # lists (at most 900 tokens) are too short to be cut along the KV, so the same requests are fused
    # whatever the CU count; request 1 shares its first two segments with the others and stays unfused
    plan = B.tl_plan_create(plan_pool[0], b.q_heads, b.req_row_ptr, b.req_seg_ptr, b.seg_ids, flags)
    info = _check_plan_covers(b, plan, flags, fused_req=(0, 2))
    assert info.n_fused_tiles == 4 + 2
    B.tl_plan_destroy(plan)
    plan = B.tl_plan_create(plan_pool[0], b.q_heads, b.req_row_ptr, b.req_seg_ptr, b.seg_ids, flags, 0, 64)
    info = _check_plan_covers(b, plan, flags, fused_req=(0, 2))
    assert info.n_fused_tiles == 4 + 2 and info.n_fused_tokens == 328       # row tiles of 64 tokens
    assert info.n_causal_tiles == 2 + 1                                      # requests 1 and 3 only
    B.tl_plan_destroy(plan)
    with pytest.raises(B.TokenLakeError) as e:
        B.tl_plan_create(plan_pool[0], b.q_heads, b.req_row_ptr, b.req_seg_ptr, b.seg_ids, B.TL_PLAN_FUSE_ROWS)
    assert e.value.status == B.TL_EINVAL                                     # needs the self block
    # without the flag nothing is fused
    plan = B.tl_plan_create(plan_pool[0], b.q_heads, b.req_row_ptr, b.req_seg_ptr, b.seg_ids, B.TL_PLAN_SELF_BLOCK)
    info = _check_plan_covers(b, plan, B.TL_PLAN_SELF_BLOCK)
    assert info.n_fused_tiles == 0
    B.tl_plan_destroy(plan)
    B.tl_pool_destroy(plan_pool[0])


def test_small_batch_of_row_tiles_is_cut_along_its_kv():
    """One long prompt: 8 row tiles x 8 kv heads = 64 workgroups would leave three quarters of the
    GPU idle, so the plan cuts the slot list into chunks (more work items, each with partial rows
    of its own); every (token, list entry) pair is still covered exactly once."""
    b = wl.prefill(seed=10, n_req=1, new_tokens=512, lo=30000, hi=32768, seg_len=256, n_slots=160, n_shared=0)
    plan_pool[0] = _pool_for(b)
    for flags in (B.TL_PLAN_SELF_BLOCK, B.TL_PLAN_SELF_BLOCK | B.TL_PLAN_FUSE_ROWS):
        plan = B.tl_plan_create(plan_pool[0], b.q_heads, b.req_row_ptr, b.req_seg_ptr, b.seg_ids, flags)
        info = _check_plan_covers(b, plan, flags)
        assert info.n_fused_tiles == 0 and info.n_items == 8 and info.n_tiles == 64      # 2 * 256 / 64 = 8 chunks
        ex = B.tl_plan_export(plan)
        assert np.diff(ex["item_slot_ptr"]).min() >= 8                                 # >= 2048 tokens per chunk
        B.tl_plan_destroy(plan)
    plan = B.tl_plan_create(plan_pool[0], b.q_heads, b.req_row_ptr, b.req_seg_ptr, b.seg_ids, B.TL_PLAN_SELF_BLOCK,
                            0, 0)                                                        # switched off: one item
    assert B.tl_plan_get_info(plan).n_items == 1
    B.tl_plan_destroy(plan)
    B.tl_pool_destroy(plan_pool[0])


def test_one_pass_tails_keep_shared_runs_as_work_items():
    """TL_PLAN_FUSE_TAILS: the shared system prompt stays one work item read once for every session's
    rows; each session's private history and its new tokens are one-pass rows that merge the session's
    partial rows of that item in; nothing is left for tl_causal_block or tl_merge."""
    b = wl.multiturn(turn=3)
    plan_pool[0] = _pool_for(b)
    flags = B.TL_PLAN_SELF_BLOCK | B.TL_PLAN_FUSE_TAILS
    plan = B.tl_plan_create(plan_pool[0], b.q_heads, b.req_row_ptr, b.req_seg_ptr, b.seg_ids, flags)
    info = _check_plan_covers(b, plan, flags, tail_req=tuple(range(64)))
    assert info.n_items == 1 and info.n_tiles == 64 * 256 // 64 and info.n_fused_tokens == b.n_tokens
    assert info.n_prior_rows == 64 and info.n_causal_tiles == 0 and info.n_merge_entries == 0
    assert info.item_pairs == 64 * 256 * 16 * 256 and info.prefix_pairs == 64 * 256 * (16 + 12) * 256
    B.tl_plan_destroy(plan)
    # with TL_PLAN_FUSE_ROWS as well, requests of 512 rows or more are taken whole and leave no work item
    plan = B.tl_plan_create(plan_pool[0], b.q_heads, b.req_row_ptr, b.req_seg_ptr, b.seg_ids, flags | B.TL_PLAN_FUSE_ROWS)
    info = _check_plan_covers(b, plan, flags | B.TL_PLAN_FUSE_ROWS, fused_req=tuple(range(64)))
    assert info.n_items == 0 and info.n_prior_rows == 0
    B.tl_plan_destroy(plan)
    B.tl_pool_destroy(plan_pool[0])
    # short chunks (40 tokens x 4 heads = 160 rows): FUSE_ROWS leaves them on the three steps, FUSE_TAILS takes the tails;
    # a decode token in the same batch keeps its split-K units and its merge list
    b = wl.multiturn(turn=2, n_sessions=6, new_tokens=40, seg_len=64, n_slots=512)
    lens = [40, 40, 1, 40, 0, 40]
    b.req_row_ptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    plan_pool[0] = _pool_for(b)
    both = B.TL_PLAN_SELF_BLOCK | B.TL_PLAN_FUSE_ROWS | B.TL_PLAN_FUSE_TAILS
    plan = B.tl_plan_create(plan_pool[0], b.q_heads, b.req_row_ptr, b.req_seg_ptr, b.seg_ids, both)
    info = _check_plan_covers(b, plan, both, tail_req=(0, 1, 3, 5))
    assert info.n_fused_tokens == 160 and info.n_single_tokens == 1 and info.n_units > 0 and info.n_causal_tiles == 0
    B.tl_plan_destroy(plan)
    with pytest.raises(B.TokenLakeError):
        B.tl_plan_create(plan_pool[0], b.q_heads, b.req_row_ptr, b.req_seg_ptr, b.seg_ids, B.TL_PLAN_FUSE_TAILS)     # needs the self block
    with pytest.raises(B.TokenLakeError):
        B.tl_plan_create(plan_pool[0], b.q_heads, b.req_row_ptr, b.req_seg_ptr, b.seg_ids,
                         B.TL_PLAN_SELF_BLOCK | B.TL_PLAN_FUSE_TAILS | B.TL_PLAN_NO_SHARING)
    B.tl_pool_destroy(plan_pool[0])


def test_shared_run_becomes_one_item_read_once():
    b = wl.multiturn(turn=2)
    pool = _pool_for(b)
    plan = B.tl_plan_create(pool, b.q_heads, b.req_row_ptr, b.req_seg_ptr, b.seg_ids)
    info, ex = B.tl_plan_get_info(plan), B.tl_plan_export(plan)
    n_tok = np.diff(ex["item_tok_ptr"])
    n_slot = np.diff(ex["item_slot_ptr"])
    assert info.n_items == 65
    hot = int(np.argmax(n_tok))
    assert n_tok[hot] == 64 * 256 and n_slot[hot] == 16          # system prompt: all rows, listed once
    assert sorted(n_slot.tolist()) == [8] * 64 + [16]
    B.tl_plan_destroy(plan)
    B.tl_pool_destroy(pool)


def test_run_shared_by_decode_tokens_becomes_units():
    """64 sessions decode one token each over a shared prompt and private histories: the shared run
    (64 tokens x 4 heads = 256 rows, one row tile's worth) is dealt to split-K units of 16 rows instead
    of a launch of row tiles of its own; with 200 tokens per session it stays a row-tile item."""
    b = wl.multiturn(turn=2, n_sessions=64, new_tokens=1, n_slots=2048)
    pool = _pool_for(b)
    plan = B.tl_plan_create(pool, b.q_heads, b.req_row_ptr, b.req_seg_ptr, b.seg_ids, B.TL_PLAN_SELF_BLOCK | B.TL_PLAN_FUSE_ROWS)
    info = B.tl_plan_get_info(plan)
    plan_pool[0] = pool
    _check_plan_covers(b, plan, B.TL_PLAN_SELF_BLOCK | B.TL_PLAN_FUSE_ROWS)
    assert info.n_tiles == 0 and info.n_fused_tiles == 0 and info.n_single_tokens == 64
    ex = B.tl_plan_export(plan)
    n_tok = np.diff(ex["item_tok_ptr"])
    shared_items = int((n_tok == 64).sum())                  # chunks of the shared run, all 64 tokens each
    assert shared_items >= 1 and info.n_units == (info.n_items - shared_items) + shared_items * 16   # 4 tokens per unit
    B.tl_plan_destroy(plan)
    B.tl_pool_destroy(pool)
    b = wl.multiturn(turn=2, n_sessions=64, new_tokens=200, n_slots=2048)
    pool = _pool_for(b)
    plan = B.tl_plan_create(pool, b.q_heads, b.req_row_ptr, b.req_seg_ptr, b.seg_ids, B.TL_PLAN_SELF_BLOCK)
    info = B.tl_plan_get_info(plan)
    assert info.n_tiles > 0 and info.n_units == 0
    B.tl_plan_destroy(plan)
    B.tl_pool_destroy(pool)


def test_single_new_tokens_get_no_causal_row_tile():
    """A request with one new token sees only itself in the self block: the plan lists it for
    the light kernel and makes row tiles only for requests with two or more tokens."""
    b = wl.decode(n_req=9, median=900, cap=4000, seg_len=128)
    b.req_row_ptr = np.concatenate([[0], np.cumsum([1, 1, 2, 1, 0, 1, 5, 1, 1])]).astype(np.int32)
    pool = _pool_for(b)
    plan = B.tl_plan_create(pool, b.q_heads, b.req_row_ptr, b.req_seg_ptr, b.seg_ids, B.TL_PLAN_SELF_BLOCK)
    info = B.tl_plan_get_info(plan)
    assert info.n_single_tokens == 6 and info.n_causal_tiles == 2
    assert info.self_pairs == 6 * 1 + 3 + 15
    B.tl_plan_destroy(plan)
    plan = B.tl_plan_create(pool, b.q_heads, b.req_row_ptr, b.req_seg_ptr, b.seg_ids, 0)
    info = B.tl_plan_get_info(plan)
    assert info.n_single_tokens == 0 and info.n_causal_tiles == 0
    B.tl_plan_destroy(plan)
    B.tl_pool_destroy(pool)


def test_tile_pairs_count_each_distinct_slot_of_a_work_item_once():
    """One work item per request (no sharing), and one-pass rows (150 tokens x 4 heads >= 512 rows):
    either way a request's whole list is one walk, so every distinct segment counts once."""
    for flags, ntok in ((B.TL_PLAN_SELF_BLOCK | B.TL_PLAN_NO_SHARING, 50), (B.TL_PLAN_SELF_BLOCK | B.TL_PLAN_FUSE_ROWS, 150)):
        b = wl.longctx(n_req=3, entries=40, new_tokens=ntok, seg_len=64, n_ids=10, n_slots=16)
        pool = _pool_for(b)
        fill_of = dict(zip(b.pool_ids.tolist(), b.pool_fills.tolist()))
        per_entry = sum(ntok * fill_of[int(i)] for i in b.seg_ids)
        distinct = sum(ntok * sum(fill_of[int(i)] for i in set(b.seg_ids[b.req_seg_ptr[r]:b.req_seg_ptr[r + 1]].tolist()))
                       for r in range(3))
        assert distinct < per_entry
        for dedupe in (1, 0):
            plan = B.tl_plan_create(pool, b.q_heads, b.req_row_ptr, b.req_seg_ptr, b.seg_ids,
                                    flags | (0 if dedupe else B.TL_PLAN_WALK_REPEATS), 0, 0)
            info = B.tl_plan_get_info(plan)
            assert info.prefix_pairs == per_entry
            assert info.tile_pairs == (distinct if dedupe else per_entry)
            assert (info.n_fused_tokens == 3 * ntok) == bool(flags & B.TL_PLAN_FUSE_ROWS)
            B.tl_plan_destroy(plan)
        B.tl_pool_destroy(pool)
    with pytest.raises(B.TokenLakeError):
        B.tl_plan_create(pool, b.q_heads, b.req_row_ptr, b.req_seg_ptr, b.seg_ids, flags, 0, 5000)   # compute_units above 4096


def test_plan_errors():
    b = wl.tiny()
    pool = _pool_for(b)
    with pytest.raises(B.TokenLakeError) as e:
        B.tl_plan_create(pool, b.q_heads, b.req_row_ptr, b.req_seg_ptr, b.seg_ids + np.uint64(1 << 40))
    assert e.value.status == B.TL_ENOTFOUND
    with pytest.raises(B.TokenLakeError):
        B.tl_plan_create(pool, 3, b.req_row_ptr, b.req_seg_ptr, b.seg_ids)          # 3 q heads on 2 kv heads
    with pytest.raises(B.TokenLakeError):
        B.tl_plan_create(pool, 66, b.req_row_ptr, b.req_seg_ptr, b.seg_ids)         # group of 33: above the limit of 32
    plan = B.tl_plan_create(pool, 12, b.req_row_ptr, b.req_seg_ptr, b.seg_ids)  # group of 6: any size up to 32 will do
    B.tl_plan_destroy(plan)
    with pytest.raises(B.TokenLakeError):
        B.tl_plan_create(pool, 8, [0, 5, 3], [0, 1, 2], b.seg_ids)                  # decreasing offsets
    with pytest.raises(B.TokenLakeError):
        B.tl_set_option("no-such-knob", 1)
    B.tl_pool_destroy(pool)


def test_append_refuses_bad_calls_without_changing_anything():
    """Validation of tl_pool_append happens before any device work, so it can be exercised with
    pointers that are never dereferenced."""
    pool = B.tl_pool_create(4, 64, 1, 128, FAKE_K, FAKE_V)
    B.tl_pool_adopt(pool, [10, 11], [0, 1], [64, 20])

    def state():
        return (B.tl_pool_used(pool), B.tl_pool_lookup(pool, [10, 11, 12, 13]).tolist(), B.tl_pool_fills(pool, [0, 1, 2, 3]).tolist())

    before = state()
    cases = [
        (dict(tail_id=99, new_ids=[], n_rows=5), B.TL_ENOTFOUND),          # unknown tail
        (dict(tail_id=11, new_ids=[12], n_rows=44), B.TL_EINVAL),          # 44 rows fit the tail's room exactly
        (dict(tail_id=11, new_ids=[], n_rows=45), B.TL_EINVAL),            # one row too many for no new id
        (dict(tail_id=None, new_ids=[], n_rows=1), B.TL_EINVAL),           # no tail: needs one new id
        (dict(tail_id=11, new_ids=[10], n_rows=50), B.TL_EINVAL),          # id already resident
        (dict(tail_id=None, new_ids=[12, 12], n_rows=100), B.TL_EINVAL),   # id listed twice
        (dict(tail_id=None, new_ids=[12, 13, 14], n_rows=130), B.TL_EFULL),  # 3 slots needed, 2 free
    ]
    for kw, status in cases:
        with pytest.raises(B.TokenLakeError) as e:
            B.tl_pool_append(pool, kw["tail_id"], kw["new_ids"], FAKE_K, FAKE_V, kw["n_rows"])
        assert e.value.status == status, (kw, e.value)
        assert state() == before
    # a tail that somebody else references too does not grow
    assert B.tl_pool_put(pool, 11, FAKE_K, FAKE_V, 20) == 1                 # second reference, no copy
    with pytest.raises(B.TokenLakeError) as e:
        B.tl_pool_append(pool, 11, [], FAKE_K, FAKE_V, 3)
    assert e.value.status == B.TL_EINVAL and state() == before
    # nothing to append is fine and does nothing
    B.tl_pool_append(pool, None, [], None, None, 0)
    assert state() == before
    B.tl_pool_destroy(pool)


def test_batched_append_validates_every_chain_before_anything_changes():
    pool = B.tl_pool_create(6, 64, 1, 128, FAKE_K, FAKE_V)
    B.tl_pool_adopt(pool, [10, 11, 12], [0, 1, 2], [64, 20, 30])

    def state():
        return (B.tl_pool_used(pool), B.tl_pool_lookup(pool, [10, 11, 12, 20, 21, 22, 23]).tolist(),
                B.tl_pool_fills(pool, list(range(6))).tolist())

    before = state()
    cases = [
        # (tails, new ids per chain, rows per chain), status: the fault sits in the LAST chain each time
        (([11, 12], [[], [20]], [10, 34]), B.TL_EINVAL),            # 34 rows fit chain 1's tail exactly
        (([11, 99], [[], []], [10, 3]), B.TL_ENOTFOUND),            # unknown tail
        (([11, 11], [[], []], [5, 5]), B.TL_EINVAL),                # two chains with one tail
        (([None, None], [[20], [20]], [10, 10]), B.TL_EINVAL),      # id given to two chains
        (([None, 12], [[20], [10]], [10, 40]), B.TL_EINVAL),        # id already resident
        (([None, None], [[20, 21], [22, 23]], [100, 100]), B.TL_EFULL),   # 4 slots needed, 3 free
    ]
    for (tails, ids, rows), status in cases:
        with pytest.raises(B.TokenLakeError) as e:
            B.tl_pool_append_batch(pool, tails, ids, rows, FAKE_K, FAKE_V)
        assert e.value.status == status, (tails, ids, rows, e.value)
        assert state() == before
    B.tl_pool_append_batch(pool, [], [], [], None, None)               # no chains
    B.tl_pool_append_batch(pool, [11, None], [[], []], [0, 0], None, None)   # chains with nothing to add
    assert state() == before
    B.tl_pool_destroy(pool)


def test_hot_slots_match_the_oracles_prefix_tree():
    """tl_plan_hot_slots against the oracle's brute-force prefix tree of the same batch (node = path of
    ids from the root; loads; parents first among equals).  Where every segment sits at one tree
    position (multi-turn, prefill) that is also the oracle's per-segment load table; the
    long-context lists name segments under many prefixes, one node each."""
    for b, tree_shaped in ((wl.multiturn(turn=3), True),
                           (wl.prefill(seed=9, n_req=5, new_tokens=40, lo=300, hi=900, seg_len=128, n_slots=64, n_shared=2), True),
                           (wl.longctx(n_req=2, entries=40, new_tokens=64, n_ids=25, n_slots=32), False)):
        pool = _pool_for(b)
        plan = B.tl_plan_create(pool, b.q_heads, b.req_row_ptr, b.req_seg_ptr, b.seg_ids)
        lists = [b.seg_ids[b.req_seg_ptr[r]:b.req_seg_ptr[r + 1]].tolist() for r in range(b.n_req)]
        ntok = np.diff(b.req_row_ptr).tolist()
        t = orc.PrefixTree()
        want = t.ranked(t.walk(lists, ntok))
        slots, loads = B.tl_plan_hot_slots(plan, 10 ** 6)
        assert slots.tolist() == B.tl_pool_lookup(pool, [path[-1] for path, _ in want]).tolist()
        assert loads.tolist() == [l for _, l in want]
        if tree_shaped:
            per_seg = orc.segment_loads(lists, ntok)
            assert slots.tolist() == B.tl_pool_lookup(pool, [i for i, _ in per_seg]).tolist() and loads.tolist() == [l for _, l in per_seg]
        top, _ = B.tl_plan_hot_slots(plan, 3)
        assert top.tolist() == slots[:3].tolist()
        B.tl_pool_destroy(pool)                                  # the plan keeps its own part of the tree
        again, _ = B.tl_plan_hot_slots(plan, 5)
        assert again.tolist() == slots[:5].tolist()
        B.tl_plan_destroy(plan)
    # the multi-turn batch: the 16 segments of the system prompt carry every new token
    b = wl.multiturn(turn=3)
    pool = _pool_for(b)
    plan = B.tl_plan_create(pool, b.q_heads, b.req_row_ptr, b.req_seg_ptr, b.seg_ids)
    slots, loads = B.tl_plan_hot_slots(plan, 17)
    assert loads[:16].tolist() == [64 * 256] * 16 and loads[16] == 256
    assert slots[:16].tolist() == B.tl_pool_lookup(pool, np.arange(16, dtype=np.uint64)).tolist()
    B.tl_plan_destroy(plan)
    B.tl_pool_destroy(pool)


def test_prefix_tree_lives_across_batches_and_loses_evicted_segments():
    """The pool's tree against the oracle's over a sequence of random batches with evictions in
    between: cumulative loads, ranking from the root, level-order export, and the removal of an
    evicted segment's nodes with everything below them; the plans of a batch built from the tree
    still cover every (token, list entry) pair."""
    rng = np.random.default_rng(77)
    n_ids, C = 14, 64
    pool = B.tl_pool_create(16, C, 1, 128, FAKE_K, FAKE_V)
    ids = np.arange(n_ids, dtype=np.uint64) + 50
    B.tl_pool_adopt(pool, ids, np.arange(n_ids), np.full(n_ids, C))
    resident = set(int(i) for i in ids)
    t = orc.PrefixTree()
    stems = [rng.choice(ids, size=3, replace=False).tolist() for _ in range(3)]
    for step in range(12):
        lists, ntok = [], []
        for r in range(int(rng.integers(1, 7))):
            l = stems[int(rng.integers(0, 3))][:int(rng.integers(0, 4))] + rng.choice(ids, size=int(rng.integers(0, 4))).tolist()
            lists.append([int(x) for x in l if int(x) in resident])
            ntok.append(int(rng.choice([0, 1, 5, 70])))
        row_ptr = np.concatenate([[0], np.cumsum(ntok)]).astype(np.int32)
        seg_ptr = np.concatenate([[0], np.cumsum([len(l) for l in lists])]).astype(np.int32)
        flat = np.array([x for l in lists for x in l], np.uint64)
        plan = B.tl_plan_create(pool, 4, row_ptr, seg_ptr, flat, B.TL_PLAN_SELF_BLOCK)
        batch = t.walk(lists, ntok)
        want = t.ranked(batch)
        slots, loads = B.tl_plan_hot_slots(plan, 1000)
        assert slots.tolist() == B.tl_pool_lookup(pool, [p[-1] for p, _ in want]).tolist() and loads.tolist() == [l for _, l in want]
        B.tl_plan_destroy(plan)
        # cumulative ranking and export
        hot = t.hot()
        got_ids, got_loads, got_depths = B.tl_pool_hot_segments(pool, 1000)
        assert got_ids.tolist() == [p[-1] for p, _ in hot] and got_loads.tolist() == [l for _, l in hot]
        assert got_depths.tolist() == [len(p) - 1 for p, _ in hot]
        k = int(rng.integers(0, 5))
        assert B.tl_pool_hot_segments(pool, k)[0].tolist() == [p[-1] for p, _ in hot[:k]]
        e_ids, e_par, e_loads, total = B.tl_pool_prefix_tree(pool, 1000)
        assert total == t.n_nodes() == len(e_ids)
        paths = []
        for i in range(len(e_ids)):                               # rebuild every node's path from the export
            paths.append((paths[e_par[i]] if e_par[i] >= 0 else ()) + (int(e_ids[i]),))
            assert e_par[i] < i
        assert sorted(paths) == sorted(t.load) and all(t.load[p] == int(l) for p, l in zip(paths, e_loads))
        assert [len(p) for p in paths] == sorted(len(p) for p in paths)          # level order
        assert len(B.tl_pool_prefix_tree(pool, 2)[0]) == min(2, total)
        if step % 3 == 2 and len(resident) > 4:                   # evict something: its nodes and their subtrees go
            victim = int(rng.choice(sorted(resident)))
            for i in sorted(resident):
                if i != victim:
                    B.tl_plan_destroy(B.tl_plan_create(pool, 4, [0, 1], [0, 1], np.array([i], np.uint64), 0))   # refresh the others
                    t.walk([[i]], [1])
            B.tl_pool_release(pool, victim)
            assert B.tl_pool_evict_lru(pool) == victim
            t.evict(victim)
            resident.discard(victim)
            assert B.tl_pool_prefix_tree(pool, 1000)[3] == t.n_nodes()
    B.tl_pool_destroy(pool)


def test_random_batches_every_pair_once_under_every_plan_mode():
    """Random trees of shared prefixes, ragged fills, repeated segments, zero-token and zero-prefix
    requests: whatever the flags, the split size and the number of CUs the planner is told to
    fill, every (token, list entry) pair is covered by exactly one work item or by the one-pass
    rows, and the merge lists name every partial row once."""
    rng = np.random.default_rng(123)
    for case in range(25):
        seg_len = int(rng.choice([64, 128, 256]))
        hkv = int(rng.choice([1, 2, 8]))
        g = int(rng.choice([1, 3, 4, 7, 8]))
        n_req = int(rng.integers(1, 9))
        n_ids = int(rng.integers(4, 40))
        # lists: a common stem, then branches; some ids repeated inside a list
        stem = rng.permutation(n_ids)[:int(rng.integers(0, 4))].tolist()
        lists, ntok = [], []
        for r in range(n_req):
            own = rng.integers(0, n_ids, size=int(rng.integers(0, 7))).tolist()
            lists.append(([] if rng.random() < 0.15 else stem[:int(rng.integers(0, len(stem) + 1))]) + own)
            ntok.append(int(rng.choice([0, 1, 3, 16, 70, 200, 600])))
        ids = sorted(set(x for l in lists for x in l))
        fills = {i: int(rng.integers(1, seg_len + 1)) for i in ids}
        b = wl.Batch(name="random", seed=0, q_heads=hkv * g, kv_heads=hkv, seg_len=seg_len, n_slots=64,
                     req_row_ptr=np.concatenate([[0], np.cumsum(ntok)]).astype(np.int32),
                     req_seg_ptr=np.concatenate([[0], np.cumsum([len(l) for l in lists])]).astype(np.int32),
                     seg_ids=np.array([x for l in lists for x in l], dtype=np.uint64),
                     pool_ids=np.array(ids, dtype=np.uint64),
                     pool_slots=rng.permutation(64)[:len(ids)].astype(np.int32),
                     pool_fills=np.array([fills[i] for i in ids], dtype=np.int32))
        plan_pool[0] = _pool_for(b)
        tok_tile = 256 // g
        for flags in (0, B.TL_PLAN_SELF_BLOCK, B.TL_PLAN_SELF_BLOCK | B.TL_PLAN_NO_SHARING,
                      B.TL_PLAN_SELF_BLOCK | B.TL_PLAN_FUSE_ROWS, B.TL_PLAN_SELF_BLOCK | B.TL_PLAN_FUSE_TAILS,
                      B.TL_PLAN_SELF_BLOCK | B.TL_PLAN_FUSE_ROWS | B.TL_PLAN_FUSE_TAILS):
            for cus in (0, 8, 256):
                if (flags & B.TL_PLAN_FUSE_TAILS) and cus:
                    continue                       # (with a CU count a long private run may be cut instead: not predicted here)
                plan = B.tl_plan_create(plan_pool[0], b.q_heads, b.req_row_ptr, b.req_seg_ptr, b.seg_ids, flags,
                                        int(rng.choice([0, 1, 3])), cus)
                fused = ()
                if flags & B.TL_PLAN_FUSE_ROWS:
                    # the rule as the header states it: more than a token's worth of rows; no segment in
                    # common with another request, or >= 512 rows; and, in a batch of fewer row-tile
                    # workgroups than CUs, a list too short to be cut along the KV
                    wgs = sum(-(-n // tok_tile) * hkv for n in ntok if n > 0)
                    users = {}
                    for r in range(n_req):
                        if ntok[r] > 0:
                            for i in set(lists[r]):
                                users[i] = users.get(i, 0) + 1
                    fused = tuple(r for r in range(n_req)
                                  if ntok[r] * g > 16
                                  and not (wgs < cus and len(lists[r]) > max(1, 2048 // seg_len))
                                  and (ntok[r] * g >= 512 or not any(users[i] > 1 for i in lists[r])))
                tails = ()
                if flags & B.TL_PLAN_FUSE_TAILS:   # every other request with more than a token's worth of rows
                    tails = tuple(r for r in range(n_req) if ntok[r] * g > 16 and r not in fused)
                _check_plan_covers(b, plan, flags, fused_req=fused, tail_req=tails)
                B.tl_plan_destroy(plan)
        B.tl_pool_destroy(plan_pool[0])


def test_binding_checks_tensor_sizes_and_types_against_the_plan():
    """The C ABI takes bare pointers; the Python wrappers compare the tensors they are handed with
    the plan (cached at its first use) before anything is enqueued.  CPU tensors stand in here: the
    checks look at dtype and element count only and fail before any device call."""
    import torch
    b = wl.tiny()
    pool = _pool_for(b)
    plan = B.tl_plan_create(pool, b.q_heads, b.req_row_ptr, b.req_seg_ptr, b.seg_ids, B.TL_PLAN_SELF_BLOCK)
    info = B.tl_plan_get_info(plan)
    T, R, hq, hkv = info.n_tokens, info.n_partial_rows, b.q_heads, b.kv_heads
    q = torch.zeros((T, hq, 128), dtype=torch.bfloat16)
    kn = torch.zeros((T, hkv, 128), dtype=torch.bfloat16)
    outp = torch.zeros((R, hq, 128), dtype=torch.float32)
    lsep = torch.zeros((R, hq), dtype=torch.float32)
    out = torch.zeros((T, hq, 128), dtype=torch.float32)
    with pytest.raises(ValueError):
        B.tl_segment_attn(pool, plan, q, b.scale, outp[:R - 1], lsep)             # a partial row short
    with pytest.raises(TypeError):
        B.tl_segment_attn(pool, plan, q.float(), b.scale, outp, lsep)             # q not bf16
    with pytest.raises(ValueError):
        B.tl_causal_block(plan, q, kn[:T - 1], kn, b.scale, outp, lsep)
    with pytest.raises(TypeError):
        B.tl_merge(plan, outp, lsep, out, True, None)                             # fp32 tensor declared bf16
    with pytest.raises(ValueError):
        B.tl_fused_attn(pool, plan, q, kn, kn, b.scale, out[:T - 1], False, None)
    B.tl_plan_destroy(plan)
    B.tl_pool_destroy(pool)


def test_prefix_tree_starts_over_when_lists_follow_no_tree():
    """Lists that name the same few segments in ever new orders make new tree nodes with every batch; the
    pool clears its tree when it has outgrown 16 nodes per slot, so its size stays bounded, and plans keep
    covering every pair."""
    rng = np.random.default_rng(5)
    n_slots, C = 8, 64
    pool = B.tl_pool_create(n_slots, C, 1, 128, FAKE_K, FAKE_V)
    ids = np.arange(n_slots, dtype=np.uint64) + 10
    B.tl_pool_adopt(pool, ids, np.arange(n_slots), np.full(n_slots, C))
    biggest = 0
    for step in range(60):
        lists = [rng.permutation(ids)[:6].tolist() for _ in range(4)]
        row_ptr = np.arange(5, dtype=np.int32) * 3
        seg_ptr = np.arange(5, dtype=np.int32) * 6
        plan = B.tl_plan_create(pool, 4, row_ptr, seg_ptr, np.array([x for l in lists for x in l], np.uint64), B.TL_PLAN_SELF_BLOCK)
        total = B.tl_pool_prefix_tree(pool, 1)[3]
        assert total <= 16 * n_slots + 24, (step, total)      # at most one batch's nodes over the limit
        biggest = max(biggest, total)
        slots, loads = B.tl_plan_hot_slots(plan, 100)
        assert len(slots) > 0 and loads[0] <= 12
        B.tl_plan_destroy(plan)
    assert biggest > 16 * n_slots - 24                         # the limit was reached, i.e. the tree did start over
    B.tl_pool_destroy(pool)


def test_segment_ids_from_tokens_equal_the_oracles_and_feed_the_planner():
    """tl_segment_ids against the oracle's from-scratch definition, bit for bit, on random sequences
    (negative token values, empty sequences, partly filled tails, salts); then two prompts that agree in
    their first 2.5 segments get ids that share two slots in the pool and one shared run in the plan."""
    rng = np.random.default_rng(31)
    for case in range(40):
        C_ = int(rng.choice([1, 2, 5, 16, 64]))
        toks = rng.integers(-2**31, 2**31, size=int(rng.integers(0, 300)), dtype=np.int64).astype(np.int32)
        salt = int(rng.integers(0, 2**63)) if case % 2 else 0
        got = B.tl_segment_ids(toks, C_, salt)
        assert got.dtype == np.uint64 and got.tolist() == orc.content_segment_ids(toks.tolist(), C_, salt)
    with pytest.raises(B.TokenLakeError):
        B.tl_segment_ids([1, 2, 3], 0)
    C_ = 64
    a = rng.integers(0, 32000, size=4 * C_).tolist()
    b = a[:2 * C_ + C_ // 2] + rng.integers(0, 32000, size=2 * C_).tolist()
    ia, ib = B.tl_segment_ids(a, C_), B.tl_segment_ids(b, C_)
    assert ia[:2].tolist() == ib[:2].tolist() and ia[2] != ib[2]
    pool = B.tl_pool_create(16, C_, 1, 128, FAKE_K, FAKE_V)
    ids = np.unique(np.concatenate([ia, ib]))
    assert len(ids) == len(ia) + len(ib) - 2                       # one copy of the two shared segments
    last_fill = (len(b) - 1) % C_ + 1
    fills = np.array([last_fill if i == ib[-1] else C_ for i in ids], np.int32)
    B.tl_pool_adopt(pool, ids, np.arange(len(ids)), fills)
    lists = [ia.tolist(), ib.tolist()]
    plan = B.tl_plan_create(pool, 4, [0, 20, 40], [0, len(ia), len(ia) + len(ib)], np.array(lists[0] + lists[1], np.uint64),
                            B.TL_PLAN_SELF_BLOCK)
    ex = B.tl_plan_export(plan)
    items = [(ex["item_slots"][ex["item_slot_ptr"][i]:ex["item_slot_ptr"][i + 1]].tolist(),
              sorted(set(ex["item_tokens"][ex["item_tok_ptr"][i]:ex["item_tok_ptr"][i + 1]].tolist())))
             for i in range(len(ex["item_row_base"]))]
    shared = [it for it in items if len(it[1]) == 40]
    assert len(shared) == 1 and shared[0][0] == B.tl_pool_lookup(pool, ia[:2]).tolist()     # the common two segments, read once for both
    B.tl_plan_destroy(plan)
    B.tl_pool_destroy(pool)
