"""GPU parity: the HIP path, called through the C-ABI, against the fp64 oracle on the same
seeded inputs.  Bars: integer/byte work bit-exact; merged O within 2e-2 max-abs and LSE
within 1e-3 (bf16 inputs, fp32 accumulate).  Because |O| itself is ~1e-2 on long diffuse
prefixes, every case also bounds the error relative to max|O*| and the suite includes
peaked / offset variants on which the absolute bar is discriminating."""
import math

import numpy as np
import pytest
import torch

from oracle import tokenlake_oracle as orc
from paper_2508_17219_amd import binding as B
from paper_2508_17219_amd import workloads as wl
from tests import tl_harness as H

pytestmark = pytest.mark.gpu

REL_O = 2e-2


def _say(msg):
    print("[case] " + msg, flush=True)


def _check_all_requests(run, rows_per_req=None, seed=0, reqs=None):
    b = run.batch
    rng = np.random.default_rng(seed)
    worst = {"err_o": 0.0, "err_lse": 0.0, "rel_o": 0.0}
    for r in (range(b.n_req) if reqs is None else reqs):
        lq = int(b.req_row_ptr[r + 1] - b.req_row_ptr[r])
        if lq == 0:
            continue
        rows = None if rows_per_req is None else H.sample_rows(lq, rows_per_req, rng)
        res = H.compare_rows(run, r, rows)
        for k in worst:
            worst[k] = max(worst[k], res[k])
        assert res["err_o"] <= H.TOL_O, "request %d: O max-abs error %.3e" % (r, res["err_o"])
        assert res["err_lse"] <= H.TOL_LSE, "request %d: LSE max-abs error %.3e" % (r, res["err_lse"])
        assert res["rel_o"] <= REL_O, "request %d: O error %.3e relative to max|O*| %.3e" % (r, res["err_o"], res["ref_o"])
    _say("%s worst err_o=%.2e err_lse=%.2e rel_o=%.2e" % (b.name, worst["err_o"], worst["err_lse"], worst["rel_o"]))
    return worst


def _check_every_request(run, rows_per_req, seed, full_heads=(), kv_per_req=2):
    """Every request of a full-size batch: its first, last and tile-boundary rows plus
    rows_per_req random ones (None: all rows), O and LSE, against the oracle on inputs copied back
    from the device tensors that the generator wrote.  Requests in `full_heads` are checked on all
    kv heads, the others on kv_per_req kv heads that rotate with the request index, so that every
    head is covered many times over the batch."""
    b = run.batch
    rng = np.random.default_rng(seed)
    worst = {"err_o": 0.0, "err_lse": 0.0, "rel_o": 0.0}
    n_checked = 0
    for r in range(b.n_req):
        lq = int(b.req_row_ptr[r + 1] - b.req_row_ptr[r])
        if lq == 0:
            continue
        rows = None if rows_per_req is None else H.sample_rows(lq, rows_per_req, rng)
        kv_sel = None if r in full_heads else sorted({(r * 3 + 5 * i) % b.kv_heads for i in range(kv_per_req)})
        res = H.compare_rows_device(run, r, rows, kv_sel)
        n_checked += 1
        for k in worst:
            worst[k] = max(worst[k], res[k])
        assert res["err_o"] <= H.TOL_O, "request %d: O max-abs error %.3e" % (r, res["err_o"])
        assert res["err_lse"] <= H.TOL_LSE, "request %d: LSE max-abs error %.3e" % (r, res["err_lse"])
        assert res["rel_o"] <= REL_O, "request %d: O error %.3e relative to max|O*| %.3e" % (r, res["err_o"], res["ref_o"])
    _say("%s: %d requests, worst err_o=%.2e err_lse=%.2e rel_o=%.2e" % (b.name, n_checked, worst["err_o"], worst["err_lse"], worst["rel_o"]))
    return worst


# ---- integer / byte work -------------------------------------------------------------------
def test_generator_bits_identical_on_device():
    _say("generator cpu vs gpu")
    for stream in (0, 3):
        a = wl.normal_bf16_range(9, stream, 12345, 1 << 16, "cpu")
        g = wl.normal_bf16_range(9, stream, 12345, 1 << 16, "cuda")
        assert np.array_equal(wl.bits_u16(a), wl.bits_u16(g))
    b = wl.tiny()
    kc, vc = b.segment_kv(b.pool_ids, "cpu")
    kg, vg = b.segment_kv(b.pool_ids, "cuda")
    assert np.array_equal(wl.bits_u16(kc), wl.bits_u16(kg)) and np.array_equal(wl.bits_u16(vc), wl.bits_u16(vg))


def test_slot_lookup_and_gather_bit_exact():
    _say("lookup + gather")
    b = wl.prefill(n_req=3, new_tokens=8, lo=300, hi=900, seg_len=128, n_slots=64, n_shared=2)
    pk, pv = H.device_pool(b, poison=False)
    pool = B.tl_pool_create(b.n_slots, b.seg_len, b.kv_heads, b.head_dim, pk, pv)
    B.tl_pool_adopt(pool, b.pool_ids, b.pool_slots, b.pool_fills)
    table = orc.SlotTable(b.n_slots, b.seg_len)
    for sid, s, f in zip(b.pool_ids, b.pool_slots, b.pool_fills):
        table.put(int(sid), int(f), int(s))
    probe = np.concatenate([b.seg_ids, np.array([123456789, 2 ** 63 + 5], dtype=np.uint64)])
    assert np.array_equal(B.tl_pool_lookup(pool, probe), table.lookup(probe))
    slots = table.lookup(b.seg_ids)
    assert np.array_equal(B.tl_pool_fills(pool, slots), table.fill(slots))
    ko = torch.zeros((len(slots),) + tuple(pk.shape[1:]), dtype=torch.bfloat16, device="cuda")
    vo = torch.zeros_like(ko)
    B.tl_pool_gather(pool, slots, ko, vo)
    torch.cuda.synchronize()
    full = np.full(len(slots), b.seg_len)
    gk, gv = orc.gather_segments(wl.bits_u16(pk), wl.bits_u16(pv), slots, full)
    assert np.array_equal(wl.bits_u16(ko).reshape(gk.shape), gk)
    assert np.array_equal(wl.bits_u16(vo).reshape(gv.shape), gv)
    B.tl_pool_destroy(pool)


def test_one_hot_attention_returns_the_slot_sentinel():
    """Integer sentinels through the whole path: V[slot, tok, g, 0] = slot and channel 1 = tok;
    one key per request is aligned with q so strongly that softmax is one-hot in fp32, so the
    merged output must name that key's (slot, token) exactly."""
    _say("one-hot sentinel")
    n_slots, C, hkv, hq, d = 32, 128, 2, 8, 128
    rng = np.random.default_rng(5)
    n_req, segs = 4, 5
    slots = rng.permutation(n_slots)[:n_req * segs].reshape(n_req, segs)
    pk = torch.zeros(n_slots, C, hkv, d, dtype=torch.bfloat16, device="cuda")
    pv = torch.zeros_like(pk)
    pv[:, :, :, 0] = torch.arange(n_slots, device="cuda", dtype=torch.float32)[:, None, None].to(torch.bfloat16)
    pv[:, :, :, 1] = torch.arange(C, device="cuda", dtype=torch.float32)[None, :, None].to(torch.bfloat16)
    q = torch.zeros(n_req, hq, d, dtype=torch.bfloat16, device="cuda")
    q[:, :, 2] = 16.0
    hot = []
    for r in range(n_req):
        s = int(slots[r, rng.integers(segs)])
        t = int(rng.integers(C))
        pk[s, t, :, 2] = 64.0                       # score 16*64/sqrt(128) ~ 90 above the rest
        hot.append((s, t))
    pool = B.tl_pool_create(n_slots, C, hkv, d, pk, pv)
    ids = np.arange(n_req * segs, dtype=np.uint64) + 1000
    B.tl_pool_adopt(pool, ids, slots.reshape(-1), np.full(n_req * segs, C))
    plan = B.tl_plan_create(pool, hq, np.arange(n_req + 1), np.arange(n_req + 1) * segs, ids, 0, 2)
    info = B.tl_plan_get_info(plan)
    outp = torch.zeros(info.n_partial_rows, hq, d, device="cuda")
    lsep = torch.zeros(info.n_partial_rows, hq, device="cuda")
    out = torch.zeros(n_req, hq, d, device="cuda")
    B.tl_segment_attn(pool, plan, q, 1 / math.sqrt(d), outp, lsep)
    B.tl_merge(plan, outp, lsep, out, False, None)
    torch.cuda.synchronize()
    for r, (s, t) in enumerate(hot):
        assert torch.all(out[r, :, 0] == float(s)) and torch.all(out[r, :, 1] == float(t)), (r, s, t, out[r, :, :2])
    B.tl_plan_destroy(plan)
    B.tl_pool_destroy(pool)


# ---- small cases, every row ------------------------------------------------------------------
def test_tiny_config_full_and_partials():
    _say("tiny full")
    b = wl.tiny()
    run = H.run_gpu(b)
    _check_all_requests(run)
    # per-item partials and the self block against the oracle's partials over the same keys
    ex = B.tl_plan_export(run.plan)
    qb, pk, pv, slots, fills, kn, vn = H.host_request_inputs(b, 0)
    slot_pos = {int(s): i for i, s in enumerate(B.tl_pool_lookup(run.pool, b.seg_ids))}
    groups = []
    for i in range(run.info.n_items):
        its = ex["item_slots"][ex["item_slot_ptr"][i]:ex["item_slot_ptr"][i + 1]]
        groups.append([slot_pos[int(s)] for s in its])
    outs, lses = orc.request_partials_by_segment(qb, pk, pv, slots, fills, kn, vn, b.scale, groups)
    for i in range(run.info.n_items):
        r0 = int(ex["item_row_base"][i])
        got_o = run.out_partial[r0:r0 + 32].double().cpu().numpy()
        got_l = run.lse_partial[r0:r0 + 32].double().cpu().numpy()
        assert np.abs(got_o - outs[i]).max() <= H.TOL_O and np.abs(got_l - lses[i]).max() <= H.TOL_LSE
    sb = run.info.self_row_base
    got_o = run.out_partial[sb:sb + 32].double().cpu().numpy()
    got_l = run.lse_partial[sb:sb + 32].double().cpu().numpy()
    assert np.abs(got_o - outs[-1]).max() <= H.TOL_O and np.abs(got_l - lses[-1]).max() <= H.TOL_LSE
    run.close()


def test_tiny_config_scalar_lds_read_variant():
    _say("tiny vread=1")
    B.tl_set_option("vread", 1)
    try:
        run = H.run_gpu(wl.tiny())
        _check_all_requests(run)
        run.close()
    finally:
        B.tl_set_option("vread", 0)


@pytest.mark.parametrize("kw", [
    dict(n_req=3, new_tokens=100, lo=300, hi=900, seg_len=128, n_slots=64, n_shared=2),     # ragged tiles and tails
    dict(n_req=2, new_tokens=70, lo=64, hi=200, seg_len=64, n_slots=16, n_shared=1, hq=8, hkv=8),   # MHA, G=1
    dict(n_req=2, new_tokens=40, lo=500, hi=700, seg_len=256, n_slots=16, n_shared=0, hq=32, hkv=1),  # G=32
    dict(n_req=5, new_tokens=3, lo=100, hi=400, seg_len=128, n_slots=32, n_shared=1, hq=16, hkv=2),   # few rows + sharing
])
def test_small_prefill_shapes_every_row(kw):
    _say("small prefill %r" % (kw,))
    run = H.run_gpu(wl.prefill(seed=11, **kw))
    _check_all_requests(run)
    run.close()


@pytest.mark.parametrize("kw", [
    dict(n_req=6, median=700, sigma=1.0, cap=3000, seg_len=128),
    dict(n_req=4, median=300, sigma=0.5, cap=1000, seg_len=64, hq=8, hkv=2),
    dict(n_req=3, median=900, sigma=0.3, cap=2000, seg_len=256, hq=16, hkv=16),
])
def test_small_decode_shapes_every_row(kw):
    _say("small decode %r" % (kw,))
    for split in (0, 1, 3):
        run = H.run_gpu(wl.decode(seed=12, **kw), split_segments=split)
        assert run.info.n_units > 0 and run.info.n_tiles == 0
        _check_all_requests(run)
        run.close()


def test_peaked_and_offset_variants_are_discriminating():
    _say("peaked / offset variants")
    for maker, kw in [(wl.prefill, dict(n_req=3, new_tokens=100, lo=300, hi=900, seg_len=128, n_slots=64, n_shared=2)),
                      (wl.decode, dict(n_req=6, median=700, cap=3000, seg_len=128))]:
        b = maker(seed=21, k_gain=4.0, v_offset_mod=7, **kw)
        run = H.run_gpu(b)
        w = _check_all_requests(run)
        # on these inputs |O| is O(1): an all-zero or segment-dropping result cannot pass 2e-2
        ref = max(H.compare_rows(run, r)["ref_o"] for r in range(b.n_req))
        assert ref > 0.5
        run.close()


def test_scores_far_from_the_first_blocks_range():
    """The row-tile kernel fixes the exponent's reference point from the first 32 keys of a work
    item and must fall back to its running-maximum path when later scores exceed it by more than
    fp32 can hold (here: keys 32x larger from the third segment on, i.e. scaled scores ~100
    above the first block's), and must stay exact when the first keys dwarf all later ones."""
    _say("late / early score peaks")
    for boost in [(2, 1 << 30, 32.0), (0, 1, 32.0), (3, 4, 32.0)]:
        b = wl.prefill(seed=23, n_req=2, new_tokens=96, lo=700, hi=1100, seg_len=128, n_slots=32, n_shared=1,
                       k_boost=boost, v_offset_mod=7)
        run = H.run_gpu(b)
        assert run.info.n_tiles > 0
        w = _check_all_requests(run)
        assert max(H.compare_rows(run, r)["ref_o"] for r in range(b.n_req)) > 0.5
        run.close()


def test_edge_cases_empty_prefix_zero_tokens_and_no_keys():
    _say("edge cases")
    base = wl.prefill(seed=13, n_req=4, new_tokens=20, lo=200, hi=500, seg_len=128, n_slots=32, n_shared=1)
    # request 1 loses its prefix; request 2 has no new tokens
    seg_ptr = base.req_seg_ptr.copy()
    lens = np.diff(seg_ptr)
    keep = [base.seg_ids[seg_ptr[r]:seg_ptr[r + 1]] for r in range(4)]
    keep[1] = keep[1][:0]
    base.seg_ids = np.concatenate(keep)
    base.req_seg_ptr = np.concatenate([[0], np.cumsum([len(k) for k in keep])]).astype(np.int32)
    base.req_row_ptr = np.array([0, 20, 40, 40, 60], np.int32)
    run = H.run_gpu(base)
    _check_all_requests(run)
    run.close()
    # without the self block a request with no prefix has no keys at all: O = 0, LSE = -inf
    base.self_block = False
    run = H.run_gpu(base)
    t0, t1 = 20, 40
    assert torch.all(run.out[t0:t1] == 0) and torch.all(torch.isneginf(run.lse[t0:t1]))
    _check_all_requests(run, reqs=[0, 3])
    run.close()
    # a batch without any new token: every call returns at once and writes nothing
    base.self_block = True
    base.req_row_ptr = np.zeros(5, np.int32)
    for fuse in (False, True):
        run = H.run_gpu(base, fuse=fuse)
        assert run.info.n_tokens == 0 and run.info.n_partial_rows == 0 and run.info.n_items == 0
        assert torch.isnan(run.out).all() and torch.isnan(run.out_partial).all()
        run.close()


def test_merge_of_long_partial_lists():
    """Split-K with one segment per unit gives a token tens of partials: the merge then runs as
    one workgroup per (token, head) with the list dealt to eight slices.  A request without any
    prefix, in a plan without the self block, has no partial at all: O = 0, LSE = -inf."""
    _say("long merge lists")
    d = wl.decode(seed=71, n_req=4, median=3000, sigma=0.3, cap=6000, seg_len=64, hq=16, hkv=2)
    seg_ptr = d.req_seg_ptr
    keep = [d.seg_ids[seg_ptr[r]:seg_ptr[r + 1]] for r in range(4)]
    keep[2] = keep[2][:0]
    d.seg_ids = np.concatenate(keep)
    d.req_seg_ptr = np.concatenate([[0], np.cumsum([len(k) for k in keep])]).astype(np.int32)
    for self_block in (True, False):
        d.self_block = self_block
        for bf16 in (False, True):
            run = H.run_gpu(d, split_segments=1, out_bf16=bf16)
            ex = B.tl_plan_export(run.plan)
            n_lists = 4 if self_block else 3
            assert len(ex["merge_rows"]) >= 8 * n_lists and run.info.n_units >= 100      # the sliced kernel's case
            if not self_block:
                assert torch.all(run.out[2] == 0) and torch.all(torch.isneginf(run.lse[2]))
            if not bf16:
                _check_all_requests(run, reqs=None if self_block else [0, 1, 3])
            else:
                want = H.run_gpu(d, split_segments=1)
                assert (run.out.float() - want.out).abs().max().item() <= 2.0 ** -8 * max(1.0, want.out.abs().max().item())
                assert torch.equal(run.lse, want.lse)
                want.close()
            run.close()


def test_merge_kernels_on_synthetic_partials():
    """tl_merge alone, on partials that attention would rarely produce: LSEs spread over +-80,
    partials with LSE = -inf (weight 0) mixed in, tokens whose partials are all -inf.  The plan
    gives short lists (plain kernel) and long ones (sliced kernel) in the same call; every
    (token, head) against the oracle's merge, fp32 and bf16 outputs."""
    _say("merge on synthetic partials")
    d = wl.decode(seed=72, n_req=6, median=1500, sigma=0.8, cap=6000, seg_len=64, hq=8, hkv=2)
    pk, pv = H.device_pool(d, poison=False)
    pool = B.tl_pool_create(d.n_slots, d.seg_len, d.kv_heads, d.head_dim, pk, pv)
    B.tl_pool_adopt(pool, d.pool_ids, d.pool_slots, d.pool_fills)
    plan = B.tl_plan_create(pool, d.q_heads, d.req_row_ptr, d.req_seg_ptr, d.seg_ids, B.TL_PLAN_SELF_BLOCK, 2)
    info, ex = B.tl_plan_get_info(plan), B.tl_plan_export(plan)
    counts = np.diff(ex["merge_ptr"])
    assert counts.min() < 8 <= counts.max()                       # both kernels have work
    rng = np.random.default_rng(5)
    R, Hq, D = info.n_partial_rows, d.q_heads, d.head_dim
    outp = rng.standard_normal((R, Hq, D)).astype(np.float32)
    lsep = (rng.standard_normal((R, Hq)) * 30).astype(np.float32)
    lsep[rng.random((R, Hq)) < 0.2] = -np.inf
    dead_tok = int(np.argmax(counts))                             # every partial of the longest list: no keys
    lsep[ex["merge_rows"][ex["merge_ptr"][dead_tok]:ex["merge_ptr"][dead_tok + 1]], 0] = -np.inf
    g_outp, g_lsep = torch.from_numpy(outp).cuda(), torch.from_numpy(lsep).cuda()
    for bf16 in (False, True):
        out = torch.full((info.n_tokens, Hq, D), float("nan"), dtype=torch.bfloat16 if bf16 else torch.float32, device="cuda")
        lse = torch.full((info.n_tokens, Hq), float("nan"), dtype=torch.float32, device="cuda")
        B.tl_merge(plan, g_outp, g_lsep, out, bf16, lse)
        torch.cuda.synchronize()
        got_o, got_l = out.double().cpu().numpy(), lse.double().cpu().numpy()
        for t in range(info.n_tokens):
            rows = ex["merge_rows"][ex["merge_ptr"][t]:ex["merge_ptr"][t + 1]]
            want_o, want_l = orc.merge_partials(outp[rows], lsep[rows])
            both_inf = np.isneginf(want_l) & np.isneginf(got_l[t])
            diff = np.abs(np.where(both_inf, 0.0, got_l[t]) - np.where(both_inf, 0.0, want_l))
            assert np.all(diff <= 1e-4 * np.maximum(1.0, np.abs(np.where(both_inf, 0.0, want_l)))), t
            tol = 2.0 ** -8 * max(1.0, float(np.abs(want_o).max())) if bf16 else 1e-5 * max(1.0, float(np.abs(want_o).max()))
            assert np.abs(got_o[t] - want_o).max() <= tol, (t, bf16)
        assert np.all(got_o[dead_tok, 0] == 0) and np.isneginf(got_l[dead_tok, 0])
    B.tl_plan_destroy(plan)
    B.tl_pool_destroy(pool)


def test_put_path_dedup_and_ragged_fill():
    _say("put path")
    b = wl.prefill(seed=14, n_req=2, new_tokens=33, lo=150, hi=400, seg_len=128, n_slots=16, n_shared=1)
    pool = B.tl_pool_create(b.n_slots, b.seg_len, b.kv_heads, b.head_dim, None, None)   # library-owned memory
    k, v = b.segment_kv(b.pool_ids, "cuda")
    for i, (sid, s, f) in enumerate(zip(b.pool_ids, b.pool_slots, b.pool_fills)):
        got = B.tl_pool_put(pool, int(sid), k[i, :f].contiguous(), v[i, :f].contiguous(), int(f), int(s))
        assert got == int(s)
    # putting a resident id again stores nothing and returns the same slot
    assert B.tl_pool_put(pool, int(b.pool_ids[0]), k[1], v[1], b.seg_len, -1) == int(b.pool_slots[0])
    assert B.tl_pool_used(pool) == len(b.pool_ids)
    plan = B.tl_plan_create(pool, b.q_heads, b.req_row_ptr, b.req_seg_ptr, b.seg_ids)
    info = B.tl_plan_get_info(plan)
    q, kn, vn = b.q("cuda"), b.k_new("cuda"), b.v_new("cuda")
    outp = torch.empty(info.n_partial_rows, b.q_heads, 128, device="cuda")
    lsep = torch.empty(info.n_partial_rows, b.q_heads, device="cuda")
    out = torch.empty(b.n_tokens, b.q_heads, 128, device="cuda")
    lse = torch.empty(b.n_tokens, b.q_heads, device="cuda")
    B.tl_segment_attn(pool, plan, q, b.scale, outp, lsep)
    B.tl_causal_block(plan, q, kn, vn, b.scale, outp, lsep)
    B.tl_merge(plan, outp, lsep, out, False, lse)
    torch.cuda.synchronize()
    run = H.DeviceRun(b, pool, plan, info, q, kn, vn, None, None, outp, lsep, out, lse)
    _check_all_requests(run)
    run.close()


def test_bf16_output_variant():
    _say("bf16 output")
    b = wl.prefill(seed=15, n_req=2, new_tokens=50, lo=300, hi=600, seg_len=128, n_slots=16, n_shared=1, k_gain=4.0)
    r32 = H.run_gpu(b)
    r16 = H.run_gpu(b, out_bf16=True)
    assert torch.equal(r16.out, r32.out.to(torch.bfloat16))
    assert torch.equal(r16.lse, r32.lse)
    r32.close(); r16.close()


def test_sharing_and_no_sharing_plans_agree():
    _say("sharing vs no sharing")
    b = wl.prefill(seed=16, n_req=4, new_tokens=64, lo=600, hi=900, seg_len=128, n_slots=64, n_shared=3)
    a = H.run_gpu(b)
    n = H.run_gpu(b, flags=B.TL_PLAN_SELF_BLOCK | B.TL_PLAN_NO_SHARING)
    assert a.info.n_items > n.info.n_items - 1 and n.info.n_items == 4
    assert (a.out - n.out).abs().max().item() <= 1e-3 and (a.lse - n.lse).abs().max().item() <= 1e-4
    a.close(); n.close()


def test_guard_rows_around_every_output_stay_untouched():
    """Out-of-bounds canaries: partials, LSEs and outputs live inside larger allocations whose rows
    before and after them hold a bit pattern that no kernel may change (three-step and one-pass plans,
    ragged tiles, split-K units)."""
    _say("guard rows")
    b = wl.prefill(seed=19, n_req=4, new_tokens=70, lo=300, hi=900, seg_len=128, n_slots=64, n_shared=2)
    lens = [70, 1, 200, 3]
    b.req_row_ptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    pk, pv = H.device_pool(b)
    pool = B.tl_pool_create(b.n_slots, b.seg_len, b.kv_heads, b.head_dim, pk, pv)
    B.tl_pool_adopt(pool, b.pool_ids, b.pool_slots, b.pool_fills)
    q, kn, vn = b.q("cuda"), b.k_new("cuda"), b.v_new("cuda")
    Hq, D, T, guard = b.q_heads, b.head_dim, b.n_tokens, 8
    canary = -7.25
    for flags in (B.TL_PLAN_SELF_BLOCK, B.TL_PLAN_SELF_BLOCK | B.TL_PLAN_FUSE_ROWS):
        plan = B.tl_plan_create(pool, Hq, b.req_row_ptr, b.req_seg_ptr, b.seg_ids, flags, 1, 0)
        R = B.tl_plan_get_info(plan).n_partial_rows
        big = {name: torch.full((rows + 2 * guard,) + tail, canary, dtype=dt, device="cuda")
               for name, rows, tail, dt in (("outp", R, (Hq, D), torch.float32), ("lsep", R, (Hq,), torch.float32),
                                            ("out", T, (Hq, D), torch.bfloat16), ("lse", T, (Hq,), torch.float32))}
        view = {k: v[guard:v.shape[0] - guard] for k, v in big.items()}
        B.tl_segment_attn(pool, plan, q, b.scale, view["outp"], view["lsep"])
        B.tl_causal_block(plan, q, kn, vn, b.scale, view["outp"], view["lsep"])
        B.tl_merge(plan, view["outp"], view["lsep"], view["out"], True, view["lse"])
        B.tl_fused_attn(pool, plan, q, kn, vn, b.scale, view["out"], True, view["lse"])
        torch.cuda.synchronize()
        for k, v in big.items():
            assert torch.all(v[:guard] == canary) and torch.all(v[v.shape[0] - guard:] == canary), (k, flags)
        assert not torch.any(view["out"] == canary) and not torch.any(view["lse"] == canary)     # and every token was written
        B.tl_plan_destroy(plan)
    B.tl_pool_destroy(pool)


def test_deterministic_bits_run_to_run():
    _say("determinism")
    b = wl.prefill(seed=17, n_req=3, new_tokens=90, lo=300, hi=900, seg_len=128, n_slots=64, n_shared=2)
    r1, r2 = H.run_gpu(b), H.run_gpu(b)
    assert torch.equal(r1.out, r2.out) and torch.equal(r1.lse, r2.lse)
    r1.close(); r2.close()


# ---- the named configurations at full size: every request -------------------------------------------
def test_device_copies_of_oracle_inputs_equal_the_host_generator():
    """The full-size checks below copy the oracle's inputs back from the device tensors that the
    seeded generator filled (regenerating 26 GB on the host would take minutes).  Here: the two
    sources agree bit for bit on a case small enough for both."""
    _say("oracle inputs: device copy vs host generator")
    b = wl.prefill(seed=18, n_req=3, new_tokens=40, lo=300, hi=900, seg_len=128, n_slots=64, n_shared=2)
    run = H.run_gpu(b)
    for r in range(b.n_req):
        host = H.host_request_inputs(b, r)
        dev = H.device_request_inputs(run, r)
        for i in (0, 3, 4, 5, 6):                 # q, slot positions, fills, new K, new V
            assert np.array_equal(host[i], dev[i])
        fills = host[4]
        # the pool: every valid token (beyond a slot's fill the device pool holds its poison)
        for x, y in zip(orc.gather_segments(host[1], host[2], host[3], fills), orc.gather_segments(dev[1], dev[2], dev[3], fills)):
            assert np.array_equal(x, y)
        sub = H.device_request_inputs(run, r, kv_sel=[3, 6])
        gk_h, gv_h = orc.gather_segments(host[1], host[2], host[3], fills)
        gk_d, gv_d = orc.gather_segments(sub[1], sub[2], sub[3], sub[4])
        assert np.array_equal(gk_h[:, [3, 6]], gk_d) and np.array_equal(gv_h[:, [3, 6]], gv_d)
        assert sub[7] == [12, 13, 14, 15, 24, 25, 26, 27] and np.array_equal(host[0][:, sub[7]], sub[0])
    run.close()


def test_full_prefill_config_every_request():
    _say("full prefill (cfg 2)")
    b = wl.prefill()
    L = b.prefix_tokens()
    full = {int(np.argmin(L)), int(np.argmax(L)), 0}
    for fuse in (False, True):
        run = H.run_gpu(b, fuse=fuse)
        assert (run.info.n_fused_tokens == b.n_tokens) == fuse
        _check_every_request(run, rows_per_req=6, seed=1, full_heads=full if not fuse else {5})
        run.close()


def test_full_decode_config_every_request():
    """All 256 tokens of the decode batch: 16 of the 64 q heads each (two kv heads, rotating), all
    64 heads for the shortest, the longest, the median and two more requests."""
    _say("full decode (cfg 3)")
    b = wl.decode()
    run = H.run_gpu(b, poison=False)
    order = np.argsort(b.prefix_tokens())
    full = {int(order[0]), int(order[-1]), int(order[len(order) // 2]), 7, 100}
    _check_every_request(run, rows_per_req=None, seed=2, full_heads=full)
    run.close()


@pytest.mark.parametrize("seed", [3, 33])
def test_full_longctx_config_every_request(seed):
    _say("full long context (cfg 4) seed %d" % seed)
    b = wl.longctx(seed=seed)
    for fuse in (False, True):
        run = H.run_gpu(b, fuse=fuse)
        assert (run.info.n_fused_tokens == b.n_tokens) == fuse
        _check_every_request(run, rows_per_req=3, seed=3, full_heads={2} if (seed == 3 and not fuse) else ())
        run.close()


def test_repeated_segments_walked_once_with_their_multiplicity():
    """Lists that name a segment several times (Zipf draws with replacement): by default a row-tile
    work item walks each distinct slot once and weighs its keys by the multiplicity.  Every row
    against the oracle, which concatenates the list as it stands; with TL_PLAN_WALK_REPEATS the kernel does
    the same as the oracle, and the two settings agree; three-step and one-pass plans; ragged fills
    (the repeated slots' cut-short tiles carry the weight too)."""
    _say("repeated segments")
    b = wl.longctx(seed=77, n_req=3, entries=60, new_tokens=150, seg_len=128, n_ids=12, n_slots=16)
    fills = b.pool_fills.copy()
    fills[::3] = 77                      # a third of the segments end inside their second tile
    b.pool_fills = fills
    counts = [np.unique(b.seg_ids[b.req_seg_ptr[r]:b.req_seg_ptr[r + 1]], return_counts=True)[1] for r in range(b.n_req)]
    assert max(int(c.max()) for c in counts) >= 8
    for fuse in (False, True):
        runs = {}
        for dedupe in (1, 0):
            flags = B.TL_PLAN_SELF_BLOCK | (0 if dedupe else B.TL_PLAN_WALK_REPEATS)
            runs[dedupe] = H.run_gpu(b, flags=flags, fuse=fuse)
            _check_all_requests(runs[dedupe])
        i1, i0 = runs[1].info, runs[0].info
        # one-pass rows walk a request's whole list at once (12 distinct segments of 60 entries); shared runs are
        # walked run by run, and a segment can come back in a later run
        assert i0.tile_pairs == i0.prefix_pairs == i1.prefix_pairs and (3 if fuse else 1) * i1.tile_pairs < i1.prefix_pairs
        assert (runs[1].out - runs[0].out).abs().max().item() <= 8e-3 and (runs[1].lse - runs[0].lse).abs().max().item() <= 1e-4
        runs[0].close(); runs[1].close()


def test_repeated_segments_in_split_k_units_are_walked_once():
    """Decode tokens over lists that name segments several times: a split-K unit walks each distinct
    slot of its run once, with the multiplicity as weight (the run is deduplicated before it is cut
    into chunks); with TL_PLAN_WALK_REPEATS every occurrence is walked.  Both against the oracle,
    which concatenates the list as it stands, and against each other; ragged fills."""
    _say("repeated segments, split-K units")
    b = wl.longctx(seed=78, n_req=6, entries=50, new_tokens=1, seg_len=128, n_ids=9, n_slots=16, hq=16, hkv=2)
    fills = b.pool_fills.copy()
    fills[::2] = 45
    b.pool_fills = fills
    for split in (0, 2):
        runs = {}
        for dedupe in (1, 0):
            flags = B.TL_PLAN_SELF_BLOCK | (0 if dedupe else B.TL_PLAN_WALK_REPEATS)
            runs[dedupe] = H.run_gpu(b, flags=flags, split_segments=split)
            assert runs[dedupe].info.n_units > 0 and runs[dedupe].info.n_tiles == 0
            _check_all_requests(runs[dedupe])
        assert runs[1].info.n_units < runs[0].info.n_units or split == 0       # 9 distinct slots instead of 50 entries
        assert runs[1].info.prefix_pairs == runs[0].info.prefix_pairs
        assert (runs[1].out - runs[0].out).abs().max().item() <= 8e-3 and (runs[1].lse - runs[0].lse).abs().max().item() <= 1e-4
        runs[0].close(); runs[1].close()


@pytest.mark.parametrize("turn", range(8))
def test_full_multiturn_config_every_session(turn):
    """Every session of every turn, three-step plan (the shared prompt as one work item read once
    against all 16384 query tokens, private histories, causal block, merge) and one-pass plan."""
    _say("full multi-turn (cfg 5) turn %d" % turn)
    b = wl.multiturn(turn=turn)
    for fuse in (False, True):
        if fuse and turn not in (0, 3, 7):
            continue
        run = H.run_gpu(b, fuse=fuse)
        assert (run.info.n_fused_tokens == b.n_tokens) == fuse
        if not fuse:
            assert run.info.n_items == (65 if turn else 1)
        _check_every_request(run, rows_per_req=2, seed=4 + turn, full_heads={0, 37, 63} if (turn in (0, 7) and not fuse) else ())
        run.close()


def test_tile_list_longer_than_its_lds_ring_every_row():
    """A work item with more than 512 full tiles: the row-tile kernel keeps a ring of 512 tile
    entries in LDS and refills half of it every 256 tiles.  Every row against the oracle, as
    pool work item (three steps) and as one-pass rows, with a ragged last tile."""
    _say("tile-list ring wrap")
    for fuse, n_new, n_shared in ((False, 70, 3), (True, 130, 3), (True, 70, 0)):
        b = wl.prefill(seed=91, n_req=2, new_tokens=n_new, lo=600 * 64 - 40, hi=600 * 64 - 1, seg_len=64, n_slots=1400,
                       n_shared=n_shared, hq=8, hkv=2)
        run = H.run_gpu(b, fuse=fuse, compute_units=0)
        if fuse:
            assert run.info.n_fused_tokens == b.n_tokens
        else:
            ex = B.tl_plan_export(run.plan)
            assert run.info.n_tiles > 0 and np.diff(ex["item_slot_ptr"]).max() >= 590
        _check_every_request(run, rows_per_req=None, seed=5, full_heads={0, 1})
        run.close()


# ---- one-pass (fused) rows ----------------------------------------------------------------------
def test_fused_rows_small_shapes_every_row():
    """TL_PLAN_FUSE_ROWS: requests with >= 512 rows per kv head, or with no segment in common with
    another request, go through tl_fused_attn alone
    (pool tiles, then their own new tokens, final output written by the kernel); the others
    still take the three steps.  Every row of every request against the oracle, fp32 and bf16
    outputs, with ragged fills, an empty prefix, a request below the threshold and one with
    no new tokens in the same batch."""
    _say("fused rows, small shapes")
    for seed, kw in [(41, dict(n_req=4, new_tokens=150, lo=300, hi=900, seg_len=128, n_slots=64, n_shared=2)),
                     (42, dict(n_req=3, new_tokens=200, lo=64, hi=200, seg_len=64, n_slots=32, n_shared=0)),
                     (43, dict(n_req=5, new_tokens=70, lo=1000, hi=3000, seg_len=256, n_slots=80, n_shared=3, hq=16, hkv=2))]:
        b = wl.prefill(seed=seed, **kw)
        lens = [int(x) for x in np.diff(b.req_row_ptr)]
        lens[-1] = 5                     # stays on the three-step path when it shares segments with the others
        if len(lens) > 3:
            lens[1] = 0                  # no new tokens
        b.req_row_ptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        if seed == 42:                   # first request loses its prefix: self block only
            keep = [b.seg_ids[b.req_seg_ptr[r]:b.req_seg_ptr[r + 1]] for r in range(b.n_req)]
            keep[0] = keep[0][:0]
            b.seg_ids = np.concatenate(keep)
            b.req_seg_ptr = np.concatenate([[0], np.cumsum([len(k) for k in keep])]).astype(np.int32)
        for out_bf16 in (False, True):
            run = H.run_gpu(b, fuse=True, out_bf16=out_bf16)
            g = b.q_heads // b.kv_heads
            private = kw["n_shared"] == 0        # no segment in common: even the 5-token request takes the one pass
            assert run.info.n_fused_tiles > 0
            assert run.info.n_fused_tokens == sum(x for x in lens if x * g >= 512 or (private and x * g > 16))
            _check_all_requests(run)
            run.close()


def test_one_pass_tails_merge_the_shared_runs_partials_every_row():
    """TL_PLAN_FUSE_TAILS: shared runs are work items (read once for all their requesters' rows), each
    request's private end and its new tokens are one-pass rows whose epilogue merges the request's
    partial rows of those items in.  Every row against the oracle: nested sharing (a run shared by
    all, a further run shared by two), a request whose whole list is shared (empty tail), one with no
    prefix, a decode token and a zero-token request in the same batch, ragged fills, fp32 and bf16."""
    _say("one-pass tails")
    S, F, T = B.TL_PLAN_SELF_BLOCK, B.TL_PLAN_FUSE_ROWS, B.TL_PLAN_FUSE_TAILS
    A, Bq, C_, D = 1, 2, 3, 4
    lists = [[A, Bq, C_, 10, 11], [A, Bq, D, 12], [A, Bq, C_, 13, 14, 15], [A, Bq, C_], [A, Bq, C_], [], [A, 16], [A, Bq, 17]]
    ntok = [70, 130, 90, 33, 64, 40, 1, 0]
    ids = sorted(set(x for l in lists for x in l))
    rng = np.random.default_rng(3)
    fills = {i: (64 if i in (A, Bq) else int(rng.integers(1, 65))) for i in ids}
    b = wl.Batch(name="tails", seed=88, q_heads=8, kv_heads=2, seg_len=64, n_slots=32,
                 req_row_ptr=np.concatenate([[0], np.cumsum(ntok)]).astype(np.int32),
                 req_seg_ptr=np.concatenate([[0], np.cumsum([len(l) for l in lists])]).astype(np.int32),
                 seg_ids=np.array([x for l in lists for x in l], dtype=np.uint64), pool_ids=np.array(ids, dtype=np.uint64),
                 pool_slots=rng.permutation(32)[:len(ids)].astype(np.int32),
                 pool_fills=np.array([fills[i] for i in ids], dtype=np.int32))
    for flags in (S | T, S | F | T):
        for out_bf16 in (False, True):
            run = H.run_gpu(b, flags=flags, out_bf16=out_bf16, compute_units=0, split_segments=1)
            i = run.info
            assert i.n_prior_rows >= 8 and i.n_causal_tiles == 0 and i.n_single_tokens == 1 and i.n_units > 0
            assert i.n_fused_tokens == sum(ntok) - 1
            if not out_bf16:
                _check_all_requests(run)
            else:
                want = H.run_gpu(b, flags=flags, compute_units=0, split_segments=1)
                assert torch.equal(run.out, want.out.to(torch.bfloat16)) and torch.equal(run.lse, want.lse)
                want.close()
            run.close()
    # the same batch through the plain three steps gives the same result to rounding
    a3 = H.run_gpu(b, flags=S, compute_units=0)
    at = H.run_gpu(b, flags=S | T, compute_units=0)
    assert (a3.out - at.out).abs().max().item() <= 2e-3 and (a3.lse - at.lse).abs().max().item() <= 1e-4
    a3.close(); at.close()
    # peaked and offset values, and scores far from the first block's range, through the tails
    for kw in [dict(k_gain=4.0, v_offset_mod=7), dict(k_boost=(2, 1 << 30, 32.0), v_offset_mod=7)]:
        pb = wl.prefill(seed=23, n_req=3, new_tokens=100, lo=700, hi=1100, seg_len=128, n_slots=48, n_shared=2, **kw)
        run = H.run_gpu(pb, flags=S | T, compute_units=0)
        assert run.info.n_prior_rows == 3 and run.info.n_fused_tokens == 300
        _check_all_requests(run)
        run.close()


def test_full_multiturn_config_with_one_pass_tails():
    """Turn 7 of the multi-turn workload as the benchmark spec words it: the shared prompt's 16 segments are
    read once against all 16384 query tokens (one work item), each session's history and new tokens
    go through the one-pass kernel, which merges the session's partial rows in."""
    _say("full multi-turn, one-pass tails")
    b = wl.multiturn(turn=7)
    run = H.run_gpu(b, flags=B.TL_PLAN_SELF_BLOCK | B.TL_PLAN_FUSE_TAILS)
    assert run.info.n_items == 1 and run.info.n_prior_rows == 64 and run.info.n_merge_entries == 0
    _check_every_request(run, rows_per_req=2, seed=9, full_heads={0, 63})
    run.close()


def test_only_short_segments_no_full_tile_anywhere():
    """Every segment holds fewer than 64 tokens, so no pool tile is full: the pipelined path never
    runs on the pool (only on the new tokens of the one-pass rows), the masked path does all of it."""
    _say("segments shorter than a tile")
    b = wl.prefill(seed=44, n_req=3, new_tokens=140, lo=600, hi=1200, seg_len=128, n_slots=48, n_shared=2)
    rng = np.random.default_rng(44)
    b.pool_fills = rng.integers(1, 64, size=len(b.pool_fills)).astype(np.int32)
    for fuse in (False, True):
        run = H.run_gpu(b, fuse=fuse)
        assert (run.info.n_fused_tokens > 0) == fuse
        _check_all_requests(run)
        run.close()


def test_fused_rows_peaked_and_far_scores():
    _say("fused rows, peaked / far scores")
    for kw in [dict(k_gain=4.0, v_offset_mod=7), dict(k_boost=(2, 1 << 30, 32.0), v_offset_mod=7),
               dict(k_boost=(0, 1, 32.0), v_offset_mod=7)]:
        b = wl.prefill(seed=23, n_req=2, new_tokens=160, lo=700, hi=1100, seg_len=128, n_slots=32, n_shared=1, **kw)
        run = H.run_gpu(b, fuse=True)
        assert run.info.n_fused_tokens == 320 and run.info.n_tiles == 0
        _check_all_requests(run)
        run.close()


def test_append_rows_grow_chains_like_the_oracle():
    """tl_pool_append against the oracle's append: same slots, same fills, same bytes in the
    pool after every call (bit-exact), and attention over the grown chains within tolerance.
    Rows come from the seeded generator on both sides; the oracle keeps its own numpy pool."""
    _say("append path")
    seed, hq, hkv, C, n_slots, d = 31, 8, 2, 128, 24, 128
    dev = "cuda"
    rng = np.random.default_rng(seed)
    pk = torch.full((n_slots, C, hkv, d), float("nan"), dtype=torch.bfloat16, device=dev)
    pv = torch.full((n_slots, C, hkv, d), float("nan"), dtype=torch.bfloat16, device=dev)
    pool = B.tl_pool_create(n_slots, C, hkv, d, pk, pv)
    opk = np.zeros((n_slots, C, hkv, d), np.uint16)
    opv = np.zeros_like(opk)
    table = orc.SlotTable(n_slots, C)
    cursor = [0]

    def rows(n):                      # n token rows of K and of V, same bits on both devices
        per = hkv * d
        out = []
        for stream in (wl.STREAM_KNEW, wl.STREAM_VNEW):
            g = wl.normal_bf16_range(seed, stream, cursor[0] * per, n * per, dev).view(n, hkv, d)
            c = wl.normal_bf16_range(seed, stream, cursor[0] * per, n * per, "cpu").view(n, hkv, d)
            out += [g, wl.bits_u16(c)]
        cursor[0] += n
        return out

    # two shared, full segments stored with put
    shared = [7, 8]
    for sid in shared:
        kg, kc, vg, vc = rows(C)
        s_lib = B.tl_pool_put(pool, sid, kg, vg, C)
        s_orc = table.put(sid, C)
        assert s_lib == s_orc
        opk[s_orc], opv[s_orc] = kc, vc
    chains = {c: [] for c in range(3)}
    totals = {c: 0 for c in range(3)}
    next_id = 100
    for step in range(14):
        c = step % 3
        n = int(rng.integers(1, 2 * C + 40))
        tail = chains[c][-1] if chains[c] and totals[c] % C else None
        room = C - totals[c] % C if tail is not None else 0
        need = -(-max(0, n - room) // C)
        if B.tl_pool_used(pool) + need > n_slots:
            with pytest.raises(B.TokenLakeError) as e:
                B.tl_pool_append(pool, tail, list(range(next_id, next_id + need)), pk[0], pv[0], n)
            assert e.value.status == B.TL_EFULL
            continue
        ids = list(range(next_id, next_id + need))
        next_id += need
        if need and step % 4 == 1:     # wrong id count is refused and changes nothing
            with pytest.raises(B.TokenLakeError) as e:
                B.tl_pool_append(pool, tail, ids + [next_id], pk[0], pv[0], n)
            assert e.value.status == B.TL_EINVAL
        kg, kc, vg, vc = rows(n)
        new_slots = B.tl_pool_append(pool, tail, ids, kg, vg, n)
        placement = orc.append_rows(opk, opv, table, tail, ids, kc, vc)
        assert new_slots.tolist() == table.lookup(ids).tolist()
        chains[c] += ids
        totals[c] += n
        every = shared + [i for ch in chains.values() for i in ch]
        assert np.array_equal(B.tl_pool_lookup(pool, every), table.lookup(every))
        slots = table.lookup(every)
        assert np.array_equal(B.tl_pool_fills(pool, slots), table.fill(slots))
    assert sum(len(ch) for ch in chains.values()) >= 8
    # bytes: every valid token of every resident segment; tokens beyond the fill of a slot
    # that append created are zero
    every = shared + [i for ch in chains.values() for i in ch]
    slots = table.lookup(every)
    gk = torch.empty((len(slots), C, hkv, d), dtype=torch.bfloat16, device=dev)
    gv = torch.empty_like(gk)
    B.tl_pool_gather(pool, slots, gk, gv)
    torch.cuda.synchronize()
    gkb, gvb = wl.bits_u16(gk), wl.bits_u16(gv)
    for i, (s, f) in enumerate(zip(slots, table.fill(slots))):
        assert np.array_equal(gkb[i, :f], opk[s, :f]) and np.array_equal(gvb[i, :f], opv[s, :f]), "slot %d" % s
        if every[i] >= 100:
            assert not gkb[i, f:].any() and not gvb[i, f:].any()
    # attention of one request per chain over shared + chain segments, plus the self block
    lq = 40
    req_ids = [shared + chains[c] for c in range(3)]
    seg_ptr = np.concatenate([[0], np.cumsum([len(x) for x in req_ids])]).astype(np.int32)
    row_ptr = (np.arange(4) * lq).astype(np.int32)
    plan = B.tl_plan_create(pool, hq, row_ptr, seg_ptr, np.array([i for x in req_ids for i in x], np.uint64))
    info = B.tl_plan_get_info(plan)
    T = 3 * lq
    qg = wl.normal_bf16_range(seed, wl.STREAM_Q, 0, T * hq * d, dev).view(T, hq, d)
    qc = wl.bits_u16(wl.normal_bf16_range(seed, wl.STREAM_Q, 0, T * hq * d, "cpu").view(T, hq, d))
    kng, knc, vng, vnc = rows(T)
    outp = torch.full((info.n_partial_rows, hq, d), float("nan"), dtype=torch.float32, device=dev)
    lsep = torch.full((info.n_partial_rows, hq), float("nan"), dtype=torch.float32, device=dev)
    out = torch.full((T, hq, d), float("nan"), dtype=torch.float32, device=dev)
    lse = torch.full((T, hq), float("nan"), dtype=torch.float32, device=dev)
    scale = 1.0 / math.sqrt(d)
    B.tl_segment_attn(pool, plan, qg, scale, outp, lsep)
    B.tl_causal_block(plan, qg, kng, vng, scale, outp, lsep)
    B.tl_merge(plan, outp, lsep, out, False, lse)
    torch.cuda.synchronize()
    for r in range(3):
        sl = table.lookup(req_ids[r])
        gk_, gv_ = orc.gather_segments(opk, opv, sl, table.fill(sl))
        t0 = r * lq
        k_all = np.concatenate([gk_, knc[t0:t0 + lq]], axis=0)
        v_all = np.concatenate([gv_, vnc[t0:t0 + lq]], axis=0)
        want_o, want_l = orc.partial_attention(qc[t0:t0 + lq], k_all, v_all, scale, n_visible=gk_.shape[0] + np.arange(lq) + 1)
        got_o = out[t0:t0 + lq].double().cpu().numpy()
        got_l = lse[t0:t0 + lq].double().cpu().numpy()
        assert np.abs(got_o - want_o).max() <= H.TOL_O and np.abs(got_l - want_l).max() <= H.TOL_LSE
    B.tl_plan_destroy(plan)
    B.tl_pool_destroy(pool)


def test_batched_append_equals_the_oracles_chain_by_chain_appends():
    """tl_pool_append_batch (all chains of a turn in one call, one launch per 128 destination
    slots) against the oracle appending chain after chain: same slots, fills and pool bytes."""
    _say("batched append")
    seed, hkv, C, n_slots, d = 37, 2, 64, 800, 128
    dev = "cuda"
    rng = np.random.default_rng(seed)
    pk = torch.full((n_slots, C, hkv, d), float("nan"), dtype=torch.bfloat16, device=dev)
    pv = torch.full((n_slots, C, hkv, d), float("nan"), dtype=torch.bfloat16, device=dev)
    pool = B.tl_pool_create(n_slots, C, hkv, d, pk, pv)
    opk = np.zeros((n_slots, C, hkv, d), np.uint16)
    opv = np.zeros_like(opk)
    table = orc.SlotTable(n_slots, C)
    n_chains = 120
    most_chunks = 0
    chains = [[] for _ in range(n_chains)]
    totals = [0] * n_chains
    next_id, cursor = 1000, 0
    per = hkv * d
    for turn in range(3):
        counts = [int(rng.choice([0, 1, C - 1, C, C + 1, 2 * C + 7])) for _ in range(n_chains)]
        tails, ids = [], []
        for c in range(n_chains):
            tail = chains[c][-1] if chains[c] and totals[c] % C else None
            room = C - totals[c] % C if tail is not None else 0
            need = -(-max(0, counts[c] - room) // C)
            tails.append(tail)
            ids.append(list(range(next_id, next_id + need)))
            next_id += need
        most_chunks = max(most_chunks, sum(len(x) for x in ids) + sum(1 for c in range(n_chains) if tails[c] is not None and counts[c]))
        n = sum(counts)
        rows = []
        for stream in (wl.STREAM_KNEW, wl.STREAM_VNEW):
            rows.append(wl.normal_bf16_range(seed, stream, cursor * per, n * per, dev).view(n, hkv, d))
            rows.append(wl.bits_u16(wl.normal_bf16_range(seed, stream, cursor * per, n * per, "cpu").view(n, hkv, d)))
        cursor += n
        kg, kc, vg, vc = rows
        got = B.tl_pool_append_batch(pool, tails, ids, counts, kg, vg)
        r0 = 0
        for c in range(n_chains):
            if counts[c]:
                orc.append_rows(opk, opv, table, tails[c], ids[c], kc[r0:r0 + counts[c]], vc[r0:r0 + counts[c]])
            r0 += counts[c]
            chains[c] += ids[c]
            totals[c] += counts[c]
        flat = [i for x in ids for i in x]
        assert got.tolist() == table.lookup(flat).tolist()
    every = [i for ch in chains for i in ch]
    assert most_chunks > 128                            # at least one call needed a second launch
    slots = table.lookup(every)
    assert np.array_equal(B.tl_pool_lookup(pool, every), slots)
    assert np.array_equal(B.tl_pool_fills(pool, slots), table.fill(slots))
    gk = torch.empty((len(slots), C, hkv, d), dtype=torch.bfloat16, device=dev)
    gv = torch.empty_like(gk)
    B.tl_pool_gather(pool, slots, gk, gv)
    torch.cuda.synchronize()
    gkb, gvb = wl.bits_u16(gk), wl.bits_u16(gv)
    for i, (s_, f) in enumerate(zip(slots, table.fill(slots))):
        assert np.array_equal(gkb[i, :f], opk[s_, :f]) and np.array_equal(gvb[i, :f], opv[s_, :f]), "slot %d" % s_
        assert not gkb[i, f:].any() and not gvb[i, f:].any()
    # the device's fill table is what the attention kernels mask with: a plan over every chain
    lq = 3
    req_ids = [ch for ch in chains if ch]
    b_seg_ptr = np.concatenate([[0], np.cumsum([len(x) for x in req_ids])]).astype(np.int32)
    b_row_ptr = (np.arange(len(req_ids) + 1) * lq).astype(np.int32)
    hq = 2 * hkv
    plan = B.tl_plan_create(pool, hq, b_row_ptr, b_seg_ptr, np.array([i for x in req_ids for i in x], np.uint64), 0)
    info = B.tl_plan_get_info(plan)
    T = lq * len(req_ids)
    qg = wl.normal_bf16_range(seed, wl.STREAM_Q, 0, T * hq * d, dev).view(T, hq, d)
    qc = wl.bits_u16(wl.normal_bf16_range(seed, wl.STREAM_Q, 0, T * hq * d, "cpu").view(T, hq, d))
    outp = torch.full((info.n_partial_rows, hq, d), float("nan"), dtype=torch.float32, device=dev)
    lsep = torch.full((info.n_partial_rows, hq), float("nan"), dtype=torch.float32, device=dev)
    out = torch.full((T, hq, d), float("nan"), dtype=torch.float32, device=dev)
    lse = torch.full((T, hq), float("nan"), dtype=torch.float32, device=dev)
    scale = 1.0 / math.sqrt(d)
    B.tl_segment_attn(pool, plan, qg, scale, outp, lsep)
    B.tl_merge(plan, outp, lsep, out, False, lse)
    torch.cuda.synchronize()
    for r in range(0, len(req_ids), 5):
        sl = table.lookup(req_ids[r])
        want_o, want_l = orc.request_attention(qc[r * lq:(r + 1) * lq], opk, opv, sl, table.fill(sl), None, None, scale)
        got_o = out[r * lq:(r + 1) * lq].double().cpu().numpy()
        got_l = lse[r * lq:(r + 1) * lq].double().cpu().numpy()
        assert np.abs(got_o - want_o).max() <= H.TOL_O and np.abs(got_l - want_l).max() <= H.TOL_LSE
    B.tl_plan_destroy(plan)
    B.tl_pool_destroy(pool)


def test_multi_turn_sessions_as_a_closed_loop_on_the_device():
    """Three turns of four sessions over a shared prompt: every turn plans the batch of new tokens
    over (shared prompt + what the session has appended so far), runs the one-pass attention, checks
    every row against the oracle, and appends the turn's own new-token K/V to the session's chain
    with one tl_pool_append_batch call -- the KV a turn attends to is what earlier turns put there."""
    _say("closed multi-turn loop")
    seed, hq, hkv, C, n_slots, d = 83, 8, 2, 64, 64, 128
    dev = "cuda"
    pk = torch.full((n_slots, C, hkv, d), float("nan"), dtype=torch.bfloat16, device=dev)
    pv = torch.full((n_slots, C, hkv, d), float("nan"), dtype=torch.bfloat16, device=dev)
    pool = B.tl_pool_create(n_slots, C, hkv, d, pk, pv)
    opk = np.zeros((n_slots, C, hkv, d), np.uint16)
    opv = np.zeros_like(opk)
    table = orc.SlotTable(n_slots, C)
    scale = 1.0 / math.sqrt(d)
    cursor = [0]

    def gen(stream, n, heads):        # n rows of `heads` heads, same bits on both devices
        per = heads * d
        g = wl.normal_bf16_range(seed, stream, cursor[0] * hq * d, n * per, dev).view(n, heads, d)
        c = wl.bits_u16(wl.normal_bf16_range(seed, stream, cursor[0] * hq * d, n * per, "cpu").view(n, heads, d))
        return g, c

    shared = [1, 2, 3]
    for sid in shared:                 # the shared prompt: three full segments
        kg, kc = gen(wl.STREAM_POOL_K, C, hkv)
        vg, vc = gen(wl.STREAM_POOL_V, C, hkv)
        cursor[0] += C
        slot = B.tl_pool_put(pool, sid, kg, vg, C)
        assert slot == table.put(sid, C)
        opk[slot], opv[slot] = kc, vc
    n_sess = 4
    chains = [[] for _ in range(n_sess)]
    totals = [0] * n_sess
    next_id = 100
    for turn, lens in enumerate([[70, 150, 40, 200], [33, 64, 130, 1], [129, 20, 65, 90]]):
        T = sum(lens)
        row_ptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        lists = [shared + chains[s_] for s_ in range(n_sess)]
        seg_ptr = np.concatenate([[0], np.cumsum([len(l) for l in lists])]).astype(np.int32)
        ids = np.array([i for l in lists for i in l], np.uint64)
        qg, qc = gen(wl.STREAM_Q, T, hq)
        kng, knc = gen(wl.STREAM_KNEW, T, hkv)
        vng, vnc = gen(wl.STREAM_VNEW, T, hkv)
        cursor[0] += T
        plan = B.tl_plan_create(pool, hq, row_ptr, seg_ptr, ids, B.TL_PLAN_SELF_BLOCK | B.TL_PLAN_FUSE_ROWS, 0, 0)
        info = B.tl_plan_get_info(plan)
        R = max(info.n_partial_rows, 1)
        outp = torch.full((R, hq, d), float("nan"), dtype=torch.float32, device=dev)
        lsep = torch.full((R, hq), float("nan"), dtype=torch.float32, device=dev)
        out = torch.full((T, hq, d), float("nan"), dtype=torch.float32, device=dev)
        lse = torch.full((T, hq), float("nan"), dtype=torch.float32, device=dev)
        B.tl_segment_attn(pool, plan, qg, scale, outp, lsep)
        B.tl_causal_block(plan, qg, kng, vng, scale, outp, lsep)
        B.tl_merge(plan, outp, lsep, out, False, lse)
        B.tl_fused_attn(pool, plan, qg, kng, vng, scale, out, False, lse)
        torch.cuda.synchronize()
        for s_ in range(n_sess):
            t0, t1 = int(row_ptr[s_]), int(row_ptr[s_ + 1])
            sl = table.lookup(lists[s_])
            gk_, gv_ = orc.gather_segments(opk, opv, sl, table.fill(sl))
            k_all = np.concatenate([gk_, knc[t0:t1]], axis=0)
            v_all = np.concatenate([gv_, vnc[t0:t1]], axis=0)
            want_o, want_l = orc.partial_attention(qc[t0:t1], k_all, v_all, scale, n_visible=gk_.shape[0] + np.arange(t1 - t0) + 1)
            err_o = np.abs(out[t0:t1].double().cpu().numpy() - want_o).max()
            err_l = np.abs(lse[t0:t1].double().cpu().numpy() - want_l).max()
            assert err_o <= H.TOL_O and err_l <= H.TOL_LSE, (turn, s_, err_o, err_l)
        B.tl_plan_destroy(plan)
        # the turn's new tokens become prefix: one batched append for all sessions
        tails, new_ids = [], []
        for s_ in range(n_sess):
            tail = chains[s_][-1] if chains[s_] and totals[s_] % C else None
            room = C - totals[s_] % C if tail is not None else 0
            need = -(-max(0, lens[s_] - room) // C)
            tails.append(tail)
            new_ids.append(list(range(next_id, next_id + need)))
            next_id += need
        got = B.tl_pool_append_batch(pool, tails, new_ids, lens, kng, vng)
        for s_ in range(n_sess):
            t0, t1 = int(row_ptr[s_]), int(row_ptr[s_ + 1])
            orc.append_rows(opk, opv, table, tails[s_], new_ids[s_], knc[t0:t1], vnc[t0:t1])
            chains[s_] += new_ids[s_]
            totals[s_] += lens[s_]
        assert got.tolist() == table.lookup([i for x in new_ids for i in x]).tolist()
    assert all(len(ch) >= 3 for ch in chains)
    B.tl_pool_destroy(pool)


def test_evicted_slots_are_reused_and_attended_over():
    """Pool life cycle on the device (paper Section 4.3: eviction by last access time): a full pool,
    releases, a plan that refreshes two segments, LRU evictions (same victims as the oracle), then
    tl_pool_append and tl_pool_put into the freed slots, the stale plan refused, and attention over
    lists that mix old segments with the ones now living in reused slots -- row tiles, one-pass rows
    and split-K units (which read the live fill table) -- against the oracle's own table and pool."""
    _say("evict, reuse, attend")
    seed, hq, hkv, C, n_slots, d = 97, 8, 2, 64, 12, 128
    dev = "cuda"
    pk = torch.full((n_slots, C, hkv, d), float("nan"), dtype=torch.bfloat16, device=dev)
    pv = torch.full((n_slots, C, hkv, d), float("nan"), dtype=torch.bfloat16, device=dev)
    pool = B.tl_pool_create(n_slots, C, hkv, d, pk, pv)
    opk = np.zeros((n_slots, C, hkv, d), np.uint16)
    opv = np.zeros_like(opk)
    table = orc.SlotTable(n_slots, C)
    scale = 1.0 / math.sqrt(d)
    cursor = [0]

    def gen(stream, n, heads):
        per = heads * d
        g = wl.normal_bf16_range(seed, stream, cursor[0] * hq * d, n * per, dev).view(n, heads, d)
        c = wl.bits_u16(wl.normal_bf16_range(seed, stream, cursor[0] * hq * d, n * per, "cpu").view(n, heads, d))
        return g, c

    def put(sid, fill):
        kg, kc = gen(wl.STREAM_POOL_K, fill, hkv)
        vg, vc = gen(wl.STREAM_POOL_V, fill, hkv)
        cursor[0] += fill
        slot = B.tl_pool_put(pool, sid, kg, vg, fill)
        assert slot == table.put(sid, fill)
        opk[slot, :fill], opv[slot, :fill] = kc, vc
        opk[slot, fill:], opv[slot, fill:] = 0, 0
        return slot

    fills = [C, C, 40, C, 17, C, C, 64, 33, C, C, 5]
    for i, f in enumerate(fills):
        assert put(1 + i, f) == i
    with pytest.raises(B.TokenLakeError) as e:
        B.tl_pool_put(pool, 500, pk[0], pv[0], C)
    assert e.value.status == B.TL_EFULL

    def attend(lists, lens, fuse):
        row_ptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        seg_ptr = np.concatenate([[0], np.cumsum([len(l) for l in lists])]).astype(np.int32)
        ids = np.array([i for l in lists for i in l], np.uint64)
        T = int(row_ptr[-1])
        qg, qc = gen(wl.STREAM_Q, T, hq)
        kng, knc = gen(wl.STREAM_KNEW, T, hkv)
        vng, vnc = gen(wl.STREAM_VNEW, T, hkv)
        cursor[0] += T
        flags = B.TL_PLAN_SELF_BLOCK | (B.TL_PLAN_FUSE_ROWS if fuse else 0)
        plan = B.tl_plan_create(pool, hq, row_ptr, seg_ptr, ids, flags, 1, 0)
        table.touch(ids.tolist())
        info = B.tl_plan_get_info(plan)
        R = max(info.n_partial_rows, 1)
        outp = torch.full((R, hq, d), float("nan"), dtype=torch.float32, device=dev)
        lsep = torch.full((R, hq), float("nan"), dtype=torch.float32, device=dev)
        out = torch.full((T, hq, d), float("nan"), dtype=torch.float32, device=dev)
        lse = torch.full((T, hq), float("nan"), dtype=torch.float32, device=dev)
        B.tl_segment_attn(pool, plan, qg, scale, outp, lsep)
        B.tl_causal_block(plan, qg, kng, vng, scale, outp, lsep)
        B.tl_merge(plan, outp, lsep, out, False, lse)
        B.tl_fused_attn(pool, plan, qg, kng, vng, scale, out, False, lse)
        torch.cuda.synchronize()
        for r, l in enumerate(lists):
            t0, t1 = int(row_ptr[r]), int(row_ptr[r + 1])
            sl = table.lookup(l)
            assert (sl >= 0).all()
            gk_, gv_ = orc.gather_segments(opk, opv, sl, table.fill(sl))
            k_all = np.concatenate([gk_, knc[t0:t1]], axis=0)
            v_all = np.concatenate([gv_, vnc[t0:t1]], axis=0)
            want_o, want_l = orc.partial_attention(qc[t0:t1], k_all, v_all, scale, n_visible=gk_.shape[0] + np.arange(t1 - t0) + 1)
            err_o = np.abs(out[t0:t1].double().cpu().numpy() - want_o).max()
            err_l = np.abs(lse[t0:t1].double().cpu().numpy() - want_l).max()
            assert err_o <= H.TOL_O and err_l <= H.TOL_LSE, (fuse, r, err_o, err_l)
        return plan, info, (qg, outp, lsep)

    old_plan, info, (qg, outp, lsep) = attend([[1, 2, 3, 4], [1, 2, 9, 10, 11, 12], [5, 6, 7, 8]], [70, 1, 150], fuse=False)
    assert info.n_units > 0 and info.n_tiles > 0
    # releases; a plan that names 5 and 6 makes them the most recently used of the idle segments
    for sid in (4, 5, 6, 7, 8, 9):
        B.tl_pool_release(pool, sid)
        table.release(sid)
    p2 = B.tl_plan_create(pool, hq, [0, 1], [0, 2], np.array([5, 6], np.uint64), 0)
    B.tl_plan_destroy(p2)
    table.touch([5, 6])
    victims = [B.tl_pool_evict_lru(pool) for _ in range(4)]
    assert victims == [table.evict_lru() for _ in range(4)] and set(victims).isdisjoint({5, 6})
    assert B.tl_pool_used(pool) == 8 == table.n_used()
    # the plan made before the evictions is refused
    with pytest.raises(B.TokenLakeError) as e:
        B.tl_segment_attn(pool, old_plan, qg, scale, outp, lsep)
    assert e.value.status == B.TL_EINVAL
    B.tl_plan_destroy(old_plan)
    # a chain of 2 C + 10 rows takes three of the freed slots, a put the fourth
    n_rows = 2 * C + 10
    kg, kc = gen(wl.STREAM_POOL_K, n_rows, hkv)
    vg, vc = gen(wl.STREAM_POOL_V, n_rows, hkv)
    cursor[0] += n_rows
    new_slots = B.tl_pool_append(pool, None, [100, 101, 102], kg, vg, n_rows)
    orc.append_rows(opk, opv, table, None, [100, 101, 102], kc, vc)
    assert new_slots.tolist() == table.lookup([100, 101, 102]).tolist()
    freed = sorted(i - 1 for i in victims)                     # segment id i lived in slot i - 1
    assert new_slots.tolist() == freed[:3]
    assert put(200, 23) == freed[3]
    # grow the chain's tail (10 of 64 tokens so far) past its end
    kg, kc = gen(wl.STREAM_POOL_K, C, hkv)
    vg, vc = gen(wl.STREAM_POOL_V, C, hkv)
    cursor[0] += C
    with pytest.raises(B.TokenLakeError) as e:
        B.tl_pool_append(pool, 102, [300], kg, vg, C)         # the pool is full again
    assert e.value.status == B.TL_EFULL
    B.tl_pool_append(pool, 102, [], kg, vg, 30)
    orc.append_rows(opk, opv, table, 102, [], kc[:30], vc[:30])
    every = [1, 2, 3, 5, 6, 10, 11, 12, 100, 101, 102, 200]
    slots = table.lookup(every)
    assert np.array_equal(B.tl_pool_lookup(pool, every + victims), table.lookup(every + victims))
    assert np.array_equal(B.tl_pool_fills(pool, np.arange(n_slots)), table.fill(np.arange(n_slots)))
    gk = torch.empty((len(slots), C, hkv, d), dtype=torch.bfloat16, device=dev)
    gv = torch.empty_like(gk)
    B.tl_pool_gather(pool, slots, gk, gv)
    torch.cuda.synchronize()
    gkb, gvb = wl.bits_u16(gk), wl.bits_u16(gv)
    for i, (s_, f) in enumerate(zip(slots, table.fill(slots))):
        assert np.array_equal(gkb[i, :f], opk[s_, :f]) and np.array_equal(gvb[i, :f], opv[s_, :f]), "slot %d" % s_
        assert not gkb[i, f:].any() and not gvb[i, f:].any()      # tails of put / appended slots are cleared
    for fuse in (False, True):
        plan, info, _ = attend([[1, 2, 100, 101, 102], [5, 6, 200, 100], [200, 3, 101, 102, 12], [1, 2, 10]],
                               [70, 1, 150, 3], fuse=fuse)
        assert info.n_units > 0 and (info.n_fused_tiles > 0) == fuse
        B.tl_plan_destroy(plan)
    B.tl_pool_destroy(pool)


@pytest.mark.parametrize("hq,hkv", [(4, 4), (8, 4), (32, 1), (16, 16), (28, 4), (6, 2), (5, 1), (24, 2)])
def test_head_group_sizes_from_mha_to_one_kv_head(hq, hkv):
    """The paper's own model is multi-head (one kv head per q head); the named configurations are
    grouped-query with 4 or 8 q heads per kv head; group sizes that are no power of two (7, 3, 5,
    12) leave the last rows of a 256-row tile or a 16-row unit idle.  Every path (row tiles, one-pass rows, split-K
    units) on both extremes, every row against the oracle."""
    _say("head groups hq=%d hkv=%d" % (hq, hkv))
    g = hq // hkv
    n_new = max(2 * 256 // g + 3, 20)          # a little over two row tiles per request: enough for the one-pass plan
    b = wl.prefill(seed=51, n_req=2, new_tokens=n_new, lo=200, hi=500, seg_len=64, n_slots=24, n_shared=1, hq=hq, hkv=hkv)
    for fuse in (False, True):
        run = H.run_gpu(b, fuse=fuse)
        assert (run.info.n_fused_tiles > 0) == fuse and (run.info.n_tiles > 0) != fuse
        _check_all_requests(run)
        run.close()
    d = wl.decode(seed=52, n_req=5, median=300, cap=900, seg_len=64, hq=hq, hkv=hkv)
    run = H.run_gpu(d)
    assert (run.info.n_units > 0) == (g <= 16)     # a token's rows beyond 16 per kv head go to row tiles
    _check_all_requests(run)
    run.close()


def test_single_long_prompt_is_cut_along_its_kv_and_merged():
    """A batch too small to fill the GPU with row tiles: the plan cuts the slot list into chunks,
    each chunk yields a partial per row, the merge puts them together."""
    _say("single long prompt, KV-chunked work items")
    b = wl.prefill(seed=61, n_req=1, new_tokens=300, lo=8000, hi=8192, seg_len=256, n_slots=40, n_shared=0)
    run = H.run_gpu(b, fuse=True, fill_cus=256)
    assert run.info.n_fused_tiles == 0 and run.info.n_items == 4 and run.info.n_merge_entries == 5 * 300
    _check_all_requests(run, rows_per_req=24, seed=2)
    run.close()


def test_mixed_batch_of_prefill_chunks_and_decode_tokens():
    """One batch with one-pass rows (two prefill chunks), split-K units (single decode tokens, a
    3-token request) and a request of 30 tokens on the row-tile + merge path: the four compute
    calls write disjoint tokens of the same output."""
    _say("mixed prefill / decode batch")
    b = wl.prefill(seed=71, n_req=7, new_tokens=140, lo=500, hi=2500, seg_len=128, n_slots=160, n_shared=2)
    lens = [140, 1, 1, 150, 1, 3, 30]
    b.req_row_ptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    for split in (0, 2):
        run = H.run_gpu(b, fuse=True, split_segments=split)
        i = run.info
        assert i.n_fused_tokens == 290 and i.n_units > 0 and i.n_tiles > 0 and i.n_causal_tiles == 2 and i.n_single_tokens == 3
        _check_all_requests(run)
        run.close()


def test_random_batches_against_the_oracle():
    """Random small batches (shared stems, repeated segments, ragged fills, requests with no
    prefix or no tokens, head groups 1/3/4/7/8) through every plan mode; every row against the oracle."""
    _say("random batches")
    rng = np.random.default_rng(321)
    for case in range(6):
        seg_len = int(rng.choice([64, 128]))
        hkv = int(rng.choice([1, 2]))
        g = int(rng.choice([1, 3, 4, 7, 8]))
        n_req = int(rng.integers(2, 6))
        n_ids = int(rng.integers(6, 20))
        stem = rng.permutation(n_ids)[:int(rng.integers(1, 4))].tolist()
        lists, ntok = [], []
        for r in range(n_req):
            own = rng.integers(0, n_ids, size=int(rng.integers(0, 6))).tolist()
            lists.append(([] if rng.random() < 0.2 else stem[:int(rng.integers(0, len(stem) + 1))]) + own)
            ntok.append(int(rng.choice([0, 1, 5, 40, 150, 530 // g + 1])))
        if sum(ntok) == 0:
            ntok[0] = 7
        ids = sorted(set(x for l in lists for x in l)) or [0]
        fills = {i: int(rng.integers(1, seg_len + 1)) for i in ids}
        b = wl.Batch(name="random%d" % case, seed=100 + case, q_heads=hkv * g, kv_heads=hkv, seg_len=seg_len, n_slots=32,
                     req_row_ptr=np.concatenate([[0], np.cumsum(ntok)]).astype(np.int32),
                     req_seg_ptr=np.concatenate([[0], np.cumsum([len(l) for l in lists])]).astype(np.int32),
                     seg_ids=np.array([x for l in lists for x in l], dtype=np.uint64),
                     pool_ids=np.array(ids, dtype=np.uint64),
                     pool_slots=rng.permutation(32)[:len(ids)].astype(np.int32),
                     pool_fills=np.array([fills[i] for i in ids], dtype=np.int32))
        for kw in (dict(), dict(fuse=True), dict(flags=B.TL_PLAN_SELF_BLOCK | B.TL_PLAN_NO_SHARING, split_segments=1),
                   dict(flags=B.TL_PLAN_SELF_BLOCK | B.TL_PLAN_FUSE_TAILS, compute_units=0)):
            run = H.run_gpu(b, **kw)
            _check_all_requests(run)
            run.close()


def test_random_batches_with_peaked_scores_and_offset_values():
    """The same kind of random batches with what makes rounding show: keys scaled by 4 or 8 (a few keys
    dominate a row), per-segment V offsets of up to +-3 (|O| up to 7), segments of 256 tokens that are
    mostly full (the row-tile kernel's pipelined path), lists of up to 12 segments; every plan mode,
    every row against the oracle."""
    _say("random batches, peaked and offset")
    rng = np.random.default_rng(4242)
    for case in range(10):
        seg_len = int(rng.choice([64, 128, 256]))
        hkv = int(rng.choice([1, 2]))
        g = int(rng.choice([1, 3, 4, 7, 8]))
        n_req = int(rng.integers(2, 6))
        n_ids = int(rng.integers(6, 24))
        stem = rng.permutation(n_ids)[:int(rng.integers(1, 5))].tolist()
        lists, ntok = [], []
        for r in range(n_req):
            own = rng.integers(0, n_ids, size=int(rng.integers(0, 9))).tolist()
            lists.append(([] if rng.random() < 0.2 else stem[:int(rng.integers(0, len(stem) + 1))]) + own)
            ntok.append(int(rng.choice([0, 1, 5, 40, 150, 530 // g + 1, 700 // g])))
        if sum(ntok) == 0:
            ntok[0] = 7
        ids = sorted(set(x for l in lists for x in l)) or [0]
        fills = {i: (seg_len if rng.random() < 0.8 else int(rng.integers(1, seg_len + 1))) for i in ids}
        b = wl.Batch(name="peaked%d" % case, seed=700 + case, q_heads=hkv * g, kv_heads=hkv, seg_len=seg_len, n_slots=32,
                     req_row_ptr=np.concatenate([[0], np.cumsum(ntok)]).astype(np.int32),
                     req_seg_ptr=np.concatenate([[0], np.cumsum([len(l) for l in lists])]).astype(np.int32),
                     seg_ids=np.array([x for l in lists for x in l], dtype=np.uint64),
                     pool_ids=np.array(ids, dtype=np.uint64),
                     pool_slots=rng.permutation(32)[:len(ids)].astype(np.int32),
                     pool_fills=np.array([fills[i] for i in ids], dtype=np.int32),
                     k_gain=float(rng.choice([4.0, 8.0])), v_offset_mod=int(rng.choice([3, 7])))
        for kw in (dict(), dict(fuse=True), dict(flags=B.TL_PLAN_SELF_BLOCK | B.TL_PLAN_NO_SHARING, split_segments=1),
                   dict(flags=B.TL_PLAN_SELF_BLOCK | B.TL_PLAN_FUSE_TAILS, compute_units=0)):
            run = H.run_gpu(b, **kw)
            _check_all_requests(run)
            run.close()


# ---- the step as a HIP graph ----------------------------------------------------------------------
@pytest.mark.parametrize("fuse", [False, True])
def test_step_replays_from_a_hip_graph(fuse):
    """The compute calls only enqueue kernels, so a step can be captured once and replayed.
    Every replay, with eager work and synchronisations in between, must reproduce the eager
    result bit for bit."""
    _say("hip graph replay fuse=%s" % fuse)
    b = wl.prefill(seed=23, n_req=3, new_tokens=100, lo=300, hi=900, seg_len=128, n_slots=64, n_shared=2)
    run = H.run_gpu(b, fuse=fuse)            # eager: also brings the pool's device state up to date
    _check_all_requests(run)
    want_o, want_l = run.out.clone(), run.lse.clone()

    def step():
        B.tl_segment_attn(run.pool, run.plan, run.q, b.scale, run.out_partial, run.lse_partial)
        B.tl_causal_block(run.plan, run.q, run.k_new, run.v_new, b.scale, run.out_partial, run.lse_partial)
        B.tl_merge(run.plan, run.out_partial, run.lse_partial, run.out, False, run.lse)
        if fuse:
            B.tl_fused_attn(run.pool, run.plan, run.q, run.k_new, run.v_new, b.scale, run.out, False, run.lse)

    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for rep in range(3):
        for t in (run.out_partial, run.lse_partial, run.out, run.lse):
            t.fill_(float("nan"))                       # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(run.out, want_o) and torch.equal(run.lse, want_l), "replay %d differs" % rep
    del g
    run.close()
