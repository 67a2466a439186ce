"""Pins for the fp64 oracle: things the mathematics fixes, independent of the oracle's own code.

Each test names the fact it rests on.  The paper (Background, "LLM serving systems"; Section 4,
first paragraph) only states that partial outputs and normalizers of independent segments
combine into the final output, so the pins are closed forms, hand-expanded tiny cases, brute
force with a differently structured evaluator, and library routines (scipy logsumexp/softmax).
"""
import itertools
import math

import numpy as np
import pytest
from scipy.special import logsumexp, softmax

from oracle import tokenlake_oracle as orc


# ---------------------------------------------------------------------------------------
def f64_to_bf16_bits(x):
    """Test helper: values exactly representable in bf16 -> their bit patterns (asserts exactness)."""
    x32 = np.asarray(x, np.float32)
    bits = (x32.view(np.uint32) >> 16).astype(np.uint16)
    assert np.array_equal(orc.bf16_bits_to_f64(bits), np.asarray(x, np.float64)), "value not bf16-exact"
    return bits


def rand_bf16_bits(rng, shape, scale=1.0):
    x = (rng.standard_normal(shape) * scale).astype(np.float32)
    u = x.view(np.uint32)
    u = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)     # round to nearest even
    return u


# ---------------------------------------------------------------------------------------
def test_bf16_bit_patterns_known_values():
    # IEEE: bf16 = sign(1) exp(8) frac(7); 0x3F80 = 1, 0xC000 = -2, 0x3FC0 = 1.5, 0x0080 = 2^-126,
    # 0x0001 = 2^-133 (subnormal), 0x7F80 = +inf, 0x4049 = 3.140625
    bits = np.array([0x3F80, 0xC000, 0x3FC0, 0x0080, 0x0001, 0x7F80, 0x4049, 0x0000, 0x8000], np.uint16)
    want = [1.0, -2.0, 1.5, 2.0 ** -126, 2.0 ** -133, math.inf, 3.140625, 0.0, -0.0]
    got = orc.bf16_bits_to_f64(bits)
    assert got.dtype == np.float64
    assert np.array_equal(got, np.array(want))
    assert math.copysign(1.0, got[-1]) == -1.0


def test_hand_expanded_three_keys():
    """scale=1, q=(1,0), k_j=(ln a_j, .) with a=(1,2,3): softmax weights are exactly 1/6, 2/6, 3/6.
    v_j = (6,0), (0,6), (12,-6)  ->  O = (1+0+6, 0+2-3) = (7,-1);  LSE = ln 6."""
    q = np.array([[1.0, 0.0]])
    k = np.array([[math.log(1.0), 5.0], [math.log(2.0), -7.0], [math.log(3.0), 11.0]])
    v = np.array([[6.0, 0.0], [0.0, 6.0], [12.0, -6.0]])
    o, lse = orc.attention_rows(q, k, v, 1.0)
    assert np.allclose(o, [[7.0, -1.0]], rtol=0, atol=1e-12)
    assert abs(lse[0] - math.log(6.0)) < 1e-12


def test_hand_expanded_causal_eight_tokens():
    """8 tokens, every score equal to ln 2 * 0 = 0 except key j has score ln(j+1) for every row:
    row i sees keys 0..i, so Z_i = 1+2+..+(i+1) = (i+1)(i+2)/2 and O_i = sum_j (j+1) v_j / Z_i.
    With v_j = j (one channel): O_i = sum_{j<=i} (j+1) j / Z_i = (i(i+1)(i+2)/3) / Z_i = 2i/3."""
    n = 8
    q = np.ones((n, 1))
    k = np.log(np.arange(1, n + 1, dtype=np.float64))[:, None]
    v = np.arange(n, dtype=np.float64)[:, None]
    o, lse = orc.attention_rows(q, k, v, 1.0, n_visible=np.arange(1, n + 1))
    for i in range(n):
        assert abs(o[i, 0] - 2.0 * i / 3.0) < 1e-12
        assert abs(lse[i] - math.log((i + 1) * (i + 2) / 2.0)) < 1e-12


def test_hand_expanded_bf16_integer_case():
    """Through the bf16 entry point, GQA 2 q-heads on 1 kv-head, d=2, scale=0.5.
    q0=(2,0): scores (0, 1*... ) -- keys (0,0),(2,0),(4,2): s = 0.5*(0,4,8) = (0,2,4)
    q1=(0,2): s = 0.5*(0,0,4) = (0,0,2).  Expected weights typed from e^0, e^2, e^4."""
    qb = f64_to_bf16_bits(np.array([[[2.0, 0.0], [0.0, 2.0]]]))           # [1 tok, 2 heads, 2]
    kb = f64_to_bf16_bits(np.array([[[0.0, 0.0]], [[2.0, 0.0]], [[4.0, 2.0]]]))
    vb = f64_to_bf16_bits(np.array([[[1.0, -1.0]], [[3.0, 0.5]], [[-2.0, 8.0]]]))
    o, lse = orc.partial_attention(qb, kb, vb, 0.5)
    e2, e4 = 7.38905609893065, 54.598150033144236            # e^2, e^4 to 15 digits (tables)
    z0 = 1.0 + e2 + e4
    z1 = 1.0 + 1.0 + e2
    want0 = [(1.0 + 3.0 * e2 - 2.0 * e4) / z0, (-1.0 + 0.5 * e2 + 8.0 * e4) / z0]
    want1 = [(1.0 + 3.0 - 2.0 * e2) / z1, (-1.0 + 0.5 + 8.0 * e2) / z1]
    assert np.allclose(o[0, 0], want0, rtol=0, atol=1e-12)
    assert np.allclose(o[0, 1], want1, rtol=0, atol=1e-12)
    assert abs(lse[0, 0] - math.log(z0)) < 1e-12 and abs(lse[0, 1] - math.log(z1)) < 1e-12


# ---------------------------------------------------------------------------------------
def brute_attention(q, k, v, scale, n_vis=None):
    """Differently structured evaluator: python loops, math.exp, no max subtraction."""
    nq, nk, d = len(q), len(k), len(v[0])
    out = [[0.0] * d for _ in range(nq)]
    lse = [0.0] * nq
    for i in range(nq):
        vis = nk if n_vis is None else n_vis[i]
        ws = []
        for j in range(vis):
            s = 0.0
            for c in range(len(q[i])):
                s += q[i][c] * k[j][c]
            ws.append(math.exp(s * scale))
        z = math.fsum(ws)
        lse[i] = math.log(z)
        for c in range(d):
            out[i][c] = math.fsum(w * v[j][c] for j, w in enumerate(ws)) / z
    return np.array(out), np.array(lse)


def test_brute_force_small_random():
    rng = np.random.default_rng(7)
    for nq, nk, d in [(1, 1, 1), (3, 5, 4), (6, 8, 3), (8, 8, 2)]:
        q, k, v = rng.standard_normal((nq, d)), rng.standard_normal((nk, d)), rng.standard_normal((nk, d))
        o, l = orc.attention_rows(q, k, v, 0.37)
        bo, bl = brute_attention(q.tolist(), k.tolist(), v.tolist(), 0.37)
        assert np.allclose(o, bo, rtol=0, atol=1e-12) and np.allclose(l, bl, rtol=0, atol=1e-12)
    q, k, v = rng.standard_normal((8, 4)), rng.standard_normal((8, 4)), rng.standard_normal((8, 4))
    nv = list(range(1, 9))
    o, l = orc.attention_rows(q, k, v, 0.5, n_visible=nv)
    bo, bl = brute_attention(q.tolist(), k.tolist(), v.tolist(), 0.5, nv)
    assert np.allclose(o, bo, rtol=0, atol=1e-12) and np.allclose(l, bl, rtol=0, atol=1e-12)


def test_brute_force_request_with_pool_and_gqa():
    """Whole-request definition against explicit loops over (slot, token, head): checks slot
    indexing, fills, list order, GQA head map, causal visibility and scale in one go."""
    rng = np.random.default_rng(11)
    n_slots, C, hkv, hq, d, lq = 5, 3, 2, 4, 2, 4
    pk = rand_bf16_bits(rng, (n_slots, C, hkv, d))
    pv = rand_bf16_bits(rng, (n_slots, C, hkv, d))
    qb = rand_bf16_bits(rng, (lq, hq, d))
    kn = rand_bf16_bits(rng, (lq, hkv, d))
    vn = rand_bf16_bits(rng, (lq, hkv, d))
    slots, fills, scale = [3, 0, 4], [3, 2, 1], 0.8
    o, lse = orc.request_attention(qb, pk, pv, slots, fills, kn, vn, scale)
    P_k, P_v = orc.bf16_bits_to_f64(pk), orc.bf16_bits_to_f64(pv)
    Q, KN, VN = orc.bf16_bits_to_f64(qb), orc.bf16_bits_to_f64(kn), orc.bf16_bits_to_f64(vn)
    for i in range(lq):
        for h in range(hq):
            g = h // (hq // hkv)
            keys, vals = [], []
            for s, f in zip(slots, fills):
                for t in range(f):
                    keys.append(P_k[s, t, g].tolist())
                    vals.append(P_v[s, t, g].tolist())
            for j in range(i + 1):
                keys.append(KN[j, g].tolist())
                vals.append(VN[j, g].tolist())
            bo, bl = brute_attention([Q[i, h].tolist()], keys, vals, scale)
            assert np.allclose(o[i, h], bo[0], rtol=0, atol=1e-12)
            assert abs(lse[i, h] - bl[0]) < 1e-12


# ---------------------------------------------------------------------------------------
def test_closed_forms():
    rng = np.random.default_rng(3)
    d, n = 5, 9
    v = rng.standard_normal((n, d))
    q = rng.standard_normal((4, d))
    # identical keys: LSE = s + ln n, O = mean(V)
    k1 = rng.standard_normal(d)
    k = np.tile(k1, (n, 1))
    o, l = orc.attention_rows(q, k, v, 0.3)
    assert np.allclose(o, np.tile(v.mean(0), (4, 1)), atol=1e-12)
    assert np.allclose(l, 0.3 * q @ k1 + math.log(n), atol=1e-12)
    # q = 0: LSE = ln n, O = mean(V)
    o, l = orc.attention_rows(np.zeros((2, d)), rng.standard_normal((n, d)), v, 1.7)
    assert np.allclose(o, np.tile(v.mean(0), (2, 1)), atol=1e-12) and np.allclose(l, math.log(n), atol=1e-12)
    # bounds and convexity
    k = rng.standard_normal((n, d))
    o, l = orc.attention_rows(q, k, v, 0.9)
    s = 0.9 * q @ k.T
    assert np.all(l >= s.max(1) - 1e-12) and np.all(l <= s.max(1) + math.log(n) + 1e-12)
    assert np.all(o <= v.max(0) + 1e-12) and np.all(o >= v.min(0) - 1e-12)
    # constant V
    o, _ = orc.attention_rows(q, k, np.full((n, d), 2.5), 0.9)
    assert np.allclose(o, 2.5, atol=1e-12)
    # one dominating key (+40 over the rest): O -> its v
    kd = np.zeros((n, 1)); kd[4, 0] = 40.0
    o, l = orc.attention_rows(np.ones((1, 1)), kd, v, 1.0)
    assert np.allclose(o[0], v[4], atol=1e-12 * 1e5) and abs(l[0] - 40.0) < 1e-12 * 1e5
    # library routine: scipy softmax / logsumexp
    o, l = orc.attention_rows(q, k, v, 0.9)
    assert np.allclose(o, softmax(s, axis=1) @ v, atol=1e-12)
    assert np.allclose(l, logsumexp(s, axis=1), atol=1e-12)


def test_shift_and_duplication():
    rng = np.random.default_rng(5)
    d, n = 4, 7
    q, k, v = rng.standard_normal((3, d)), rng.standard_normal((n, d)), rng.standard_normal((n, d))
    o, l = orc.attention_rows(q, k, v, 0.6)
    # extra channel: q gets 1, every key gets c/scale -> all scores + c
    c = 2.25
    q2 = np.concatenate([q, np.ones((3, 1))], 1)
    k2 = np.concatenate([k, np.full((n, 1), c / 0.6)], 1)
    o2, l2 = orc.attention_rows(q2, k2, v, 0.6)
    assert np.allclose(o2, o, atol=1e-12) and np.allclose(l2, l + c, atol=1e-12)
    # keys listed twice: same O, LSE + ln 2
    o3, l3 = orc.attention_rows(q, np.concatenate([k, k]), np.concatenate([v, v]), 0.6)
    assert np.allclose(o3, o, atol=1e-12) and np.allclose(l3, l + math.log(2.0), atol=1e-12)


def test_empty_and_masked_rows():
    o, l = orc.attention_rows(np.ones((2, 3)), np.zeros((0, 3)), np.zeros((0, 3)), 1.0)
    assert o.shape == (2, 3) and np.all(o == 0) and np.all(np.isneginf(l))
    o, l = orc.attention_rows(np.ones((2, 3)), np.ones((4, 3)), np.ones((4, 3)), 1.0, n_visible=[0, 2])
    assert np.all(o[0] == 0) and np.isneginf(l[0]) and np.allclose(o[1], 1.0)
    assert abs(l[1] - (3.0 + math.log(2.0))) < 1e-12
    # merge: -inf partials carry weight 0; all -inf stays (0, -inf); no NaN anywhere
    outs = np.stack([np.zeros((2, 3)), np.full((2, 3), 4.0)])
    lses = np.array([[-np.inf, -np.inf], [1.5, -np.inf]])
    mo, ml = orc.merge_partials(outs, lses)
    assert np.allclose(mo[0], 4.0) and ml[0] == 1.5
    assert np.all(mo[1] == 0) and np.isneginf(ml[1]) and not np.isnan(mo).any()


# ---------------------------------------------------------------------------------------
def _request_case(rng, n_list=5, C=4, hkv=2, hq=4, d=8, lq=5, n_slots=9):
    pk = rand_bf16_bits(rng, (n_slots, C, hkv, d))
    pv = rand_bf16_bits(rng, (n_slots, C, hkv, d))
    qb = rand_bf16_bits(rng, (lq, hq, d))
    kn = rand_bf16_bits(rng, (lq, hkv, d))
    vn = rand_bf16_bits(rng, (lq, hkv, d))
    slots = rng.permutation(n_slots)[:n_list]
    fills = rng.integers(1, C + 1, size=n_list)
    return qb, pk, pv, slots, fills, kn, vn


def test_merge_of_partials_equals_full_any_partition_any_order():
    rng = np.random.default_rng(13)
    qb, pk, pv, slots, fills, kn, vn = _request_case(rng)
    scale = 1.0 / math.sqrt(8)
    full_o, full_l = orc.request_attention(qb, pk, pv, slots, fills, kn, vn, scale)
    n = len(slots)
    for trial in range(12):
        # random partition of the list into 1..n groups (not necessarily contiguous), random order
        n_groups = int(rng.integers(1, n + 1))
        labels = rng.integers(0, n_groups, size=n)
        groups = [np.flatnonzero(labels == g).tolist() for g in range(n_groups)]
        groups = [g for g in groups if g]
        outs, lses = orc.request_partials_by_segment(qb, pk, pv, slots, fills, kn, vn, scale, groups)
        perm = rng.permutation(len(outs))
        mo, ml = orc.merge_partials(outs[perm], lses[perm])
        assert np.allclose(mo, full_o, rtol=0, atol=1e-12)
        assert np.allclose(ml, full_l, rtol=0, atol=1e-12)


def test_merge_split_points_inside_segments_and_associativity():
    rng = np.random.default_rng(17)
    d, n = 6, 23
    q, k, v = rng.standard_normal((4, d)), rng.standard_normal((n, d)), rng.standard_normal((n, d))
    full_o, full_l = orc.attention_rows(q, k, v, 0.41)
    for trial in range(10):
        cuts = np.sort(rng.choice(np.arange(1, n), size=int(rng.integers(1, 6)), replace=False))
        edges = [0] + cuts.tolist() + [n]
        parts = [orc.attention_rows(q, k[a:b], v[a:b], 0.41) for a, b in zip(edges[:-1], edges[1:])]
        outs = np.stack([p[0] for p in parts]); lses = np.stack([p[1] for p in parts])
        mo, ml = orc.merge_partials(outs, lses)
        assert np.allclose(mo, full_o, atol=1e-12) and np.allclose(ml, full_l, atol=1e-12)
        # pairwise tree == flat
        acc_o, acc_l = outs[0], lses[0]
        for j in range(1, len(outs)):
            acc_o, acc_l = orc.merge_partials(np.stack([acc_o, outs[j]]), np.stack([acc_l, lses[j]]))
        assert np.allclose(acc_o, full_o, atol=1e-12) and np.allclose(acc_l, full_l, atol=1e-12)


def test_single_segment_reduces_to_plain_attention():
    rng = np.random.default_rng(19)
    C, hkv, hq, d, lq = 6, 1, 1, 8, 3
    pk = rand_bf16_bits(rng, (2, C, hkv, d)); pv = rand_bf16_bits(rng, (2, C, hkv, d))
    qb = rand_bf16_bits(rng, (lq, hq, d))
    o, l = orc.request_attention(qb, pk, pv, [1], [C], None, None, 0.25)
    Q = orc.bf16_bits_to_f64(qb)[:, 0]; K = orc.bf16_bits_to_f64(pk)[1, :, 0]; V = orc.bf16_bits_to_f64(pv)[1, :, 0]
    s = 0.25 * Q @ K.T
    assert np.allclose(o[:, 0], softmax(s, axis=1) @ V, atol=1e-12)
    assert np.allclose(l[:, 0], logsumexp(s, axis=1), atol=1e-12)


def test_slot_placement_does_not_change_any_bit():
    rng = np.random.default_rng(23)
    qb, pk, pv, slots, fills, kn, vn = _request_case(rng)
    o1, l1 = orc.request_attention(qb, pk, pv, slots, fills, kn, vn, 0.3)
    perm = rng.permutation(pk.shape[0])                 # slot s moves to perm[s]
    pk2 = np.empty_like(pk); pv2 = np.empty_like(pv)
    pk2[perm] = pk; pv2[perm] = pv
    o2, l2 = orc.request_attention(qb, pk2, pv2, perm[slots], fills, kn, vn, 0.3)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)


def test_gqa_equals_mha_with_replicated_kv_heads():
    rng = np.random.default_rng(29)
    qb, pk, pv, slots, fills, kn, vn = _request_case(rng, hkv=2, hq=6)
    o1, l1 = orc.request_attention(qb, pk, pv, slots, fills, kn, vn, 0.3)
    rep = lambda x: np.repeat(x, 3, axis=-2)
    o2, l2 = orc.request_attention(qb, rep(pk), rep(pv), slots, fills, rep(kn), rep(vn), 0.3)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)


def test_gather_brute_force_and_slot_table():
    rng = np.random.default_rng(31)
    n_slots, C, hkv, d = 6, 3, 2, 4
    pk = rng.integers(0, 65536, size=(n_slots, C, hkv, d)).astype(np.uint16)
    pv = rng.integers(0, 65536, size=(n_slots, C, hkv, d)).astype(np.uint16)
    slots, fills = [5, 2, 2, 0], [3, 1, 1, 2]
    gk, gv = orc.gather_segments(pk, pv, slots, fills)
    row = 0
    for s, f in zip(slots, fills):
        for t in range(f):
            for h in range(hkv):
                for c in range(d):
                    assert gk[row, h, c] == pk[s, t, h, c] and gv[row, h, c] == pv[s, t, h, c]
            row += 1
    assert row == gk.shape[0] == 7
    tab = orc.SlotTable(4, 8)
    assert tab.put(100, 8, want_slot=2) == 2
    assert tab.put(7, 3) == 0            # lowest free
    assert tab.put(100, 5) == 2          # dedup: existing id keeps slot and fill
    assert tab.put(9, 8) == 1
    assert list(tab.lookup([7, 100, 55, 9])) == [0, 2, -1, 1]
    assert list(tab.fill([0, 2, 1])) == [3, 8, 8]
    tab.put(1, 1)
    with pytest.raises(MemoryError):
        tab.put(2, 1)


def test_duplicate_slot_counts_twice():
    rng = np.random.default_rng(37)
    qb, pk, pv, slots, fills, kn, vn = _request_case(rng, n_list=1)
    o1, l1 = orc.request_attention(qb, pk, pv, slots, fills, None, None, 0.3)
    o2, l2 = orc.request_attention(qb, pk, pv, list(slots) * 2, list(fills) * 2, None, None, 0.3)
    assert np.allclose(o1, o2, atol=1e-12) and np.allclose(l2, l1 + math.log(2.0), atol=1e-12)


def test_append_chain_equals_concatenation_of_rows():
    """Pin for SlotTable.append / append_rows: whatever the sizes of the appends, reading a
    chain's segments back in order gives exactly the rows that were appended, in order; every
    segment but the last is full; new segments take the lowest free slot; a refused call
    changes nothing.  (The check keeps its own per-chain list of rows and never looks at the
    placement arithmetic.)"""
    rng = np.random.default_rng(5)
    n_slots, C, hkv, d = 24, 8, 2, 4
    pk = np.zeros((n_slots, C, hkv, d), np.uint16)
    pv = np.zeros_like(pk)
    table = orc.SlotTable(n_slots, C)
    table.put(1000, C, want_slot=0)          # two unrelated residents, so that slot choice is visible
    table.put(1001, 3, want_slot=2)
    chains = {c: {"ids": [], "rows_k": [], "rows_v": []} for c in range(3)}
    next_id = 1
    for step in range(40):
        c = int(rng.integers(0, 3))
        ch = chains[c]
        n = int(rng.integers(0, 2 * C + 3))
        k = rng.integers(0, 1 << 16, size=(n, hkv, d), dtype=np.uint16)
        v = rng.integers(0, 1 << 16, size=(n, hkv, d), dtype=np.uint16)
        total = sum(len(x) for x in ch["rows_k"])
        tail = ch["ids"][-1] if ch["ids"] and total % C else None
        room = (C - total % C) if tail is not None else 0
        need = -(-max(0, n - room) // C)
        used_before = set(np.flatnonzero(table._used).tolist())
        if used_before.__len__() + need > n_slots:
            with pytest.raises(MemoryError):
                orc.append_rows(pk, pv, table, tail, [10 ** 6 + i for i in range(need)], k, v)
            assert set(np.flatnonzero(table._used).tolist()) == used_before
            continue
        if need and step % 7 == 0:            # wrong id count: refused, nothing changes
            fills_before = table._fill.copy()
            with pytest.raises(ValueError):
                orc.append_rows(pk, pv, table, tail, list(range(next_id, next_id + need + 1)), k, v)
            assert np.array_equal(table._fill, fills_before)
        ids = list(range(next_id, next_id + need))
        next_id += need
        placement = orc.append_rows(pk, pv, table, tail, ids, k, v)
        new_slots = [p[0] for p in placement if p[0] not in used_before]
        free_sorted = sorted(set(range(n_slots)) - used_before)
        assert new_slots == free_sorted[:len(new_slots)]          # lowest free slots, in order
        ch["ids"] += ids
        ch["rows_k"].append(k)
        ch["rows_v"].append(v)
        for cc in chains.values():                                    # every chain, after every step
            if not cc["ids"]:
                continue
            slots = table.lookup(cc["ids"])
            assert (slots >= 0).all() and len(set(slots.tolist())) == len(slots)
            fills = table.fill(slots)
            assert (fills[:-1] == C).all() and 1 <= fills[-1] <= C
            gk, gv = orc.gather_segments(pk, pv, slots, fills)
            assert np.array_equal(gk, np.concatenate(cc["rows_k"], axis=0))
            assert np.array_equal(gv, np.concatenate(cc["rows_v"], axis=0))
    assert sum(len(c["ids"]) for c in chains.values()) > 10
    # the unrelated residents were never touched
    assert table.lookup([1000, 1001]).tolist() == [0, 2] and table.fill([0, 2]).tolist() == [C, 3]


def test_segment_loads_hand_case_and_invariants():
    """Pin for segment_loads: a case counted by hand, then invariants on random lists."""
    # requests: A = [s1, s2, s3] with 5 new tokens, B = [s1, s2, s9] with 2, C = [s7] with 4, D = [s1, s1] with 1
    got = orc.segment_loads([[1, 2, 3], [1, 2, 9], [7], [1, 1]], [5, 2, 4, 1])
    # s1: 5 + 2 + 1 + 1 = 9; s2: 5 + 2 = 7; s3: 5; s7: 4; s9: 2 -- and s3 before s7? no: 5 > 4
    assert got == [(1, 9), (2, 7), (3, 5), (7, 4), (9, 2)]
    # ties keep first appearance: s3 (request A) before s9 (request B) when both carry 3
    assert orc.segment_loads([[3], [9]], [3, 3]) == [(3, 3), (9, 3)]
    rng = np.random.default_rng(8)
    lists = [rng.integers(0, 30, size=int(rng.integers(0, 12))).tolist() for _ in range(20)]
    ntok = rng.integers(0, 50, size=20).tolist()
    got = orc.segment_loads(lists, ntok)
    assert sum(l for _, l in got) == sum(len(ids) * n for ids, n in zip(lists, ntok))     # every listing counted once
    assert [l for _, l in got] == sorted((l for _, l in got), reverse=True)
    assert set(i for i, _ in got) == set(x for ids in lists for x in ids)
    for sid, l in got:                                                                    # brute force per id
        assert l == sum(ids.count(sid) * n for ids, n in zip(lists, ntok))


def test_release_and_lru_eviction_hand_case_and_independent_model():
    """Pin for SlotTable.release / touch / evict_lru (paper Section 4.3: global LRU on the
    recorded last access time).  First a case worked by hand, then random operation sequences
    against a model of a different shape (a plain list of records scanned with min())."""
    t = orc.SlotTable(4, 8)
    assert [t.put(10, 8), t.put(11, 8), t.put(12, 3)] == [0, 1, 2]        # access times 1, 2, 3
    t.touch([10])                                                          # 10 accessed at 4
    with pytest.raises(LookupError):
        t.evict_lru()                                                      # everybody is held
    t.release(11)
    t.release(12)
    assert t.evict_lru() == 11                                             # time 2 is older than time 3
    assert t.lookup([10, 11, 12]).tolist() == [0, -1, 2] and t.fill([1]).tolist() == [0]
    assert t.put(13, 5) == 1                                               # the freed slot is the lowest free one
    t.release(10)
    assert t.evict_lru() == 12                                             # 12 (time 3) before 10 (time 4)
    assert t.evict_lru() == 10
    with pytest.raises(LookupError):
        t.evict_lru()                                                      # 13 is still held
    assert t.n_used() == 1
    # a second put of a resident id adds a holder: one release is not enough
    assert t.put(13, 5) == 1 and t.holders(13) == 2
    t.release(13)
    with pytest.raises(LookupError):
        t.evict_lru()
    t.release(13)
    with pytest.raises(ValueError):
        t.release(13)                                                      # nobody left to release
    with pytest.raises(KeyError):
        t.release(99)
    # one touch gives equal times: the lower slot goes first; a later touch of one id saves it
    a, b = t.put(20, 8), t.put(21, 8)                                      # slots 0 and 2
    assert (a, b) == (0, 2)
    for i in (20, 21):
        t.release(i)
    t.touch([21, 20, 13])
    assert t.evict_lru() == 20 and t.evict_lru() == 13 and t.evict_lru() == 21
    # a tail that somebody else also holds does not grow; neither does one nobody holds
    t = orc.SlotTable(4, 8)
    t.put(1, 3)
    t.put(1, 3)
    with pytest.raises(ValueError):
        t.append(1, [], 2)
    t.release(1)
    assert t.append(1, [], 2) == [(0, 3, 2, 0)]
    t.release(1)
    with pytest.raises(ValueError):
        t.append(1, [], 1)

    # random sequences against an independent model
    rng = np.random.default_rng(17)
    for trial in range(20):
        n_slots = int(rng.integers(2, 9))
        t = orc.SlotTable(n_slots, 8)
        model = []                      # records [id, slot, holders, time]
        clock = 0
        for step in range(200):
            op = rng.choice(["put", "touch", "release", "evict"], p=[0.35, 0.2, 0.3, 0.15])
            ids_in = [m[0] for m in model]
            if op == "put":
                sid = int(rng.integers(0, 12))
                rec = next((m for m in model if m[0] == sid), None)
                if rec is None and len(model) == n_slots:
                    with pytest.raises(MemoryError):
                        t.put(sid, 8)
                    continue
                clock += 1
                if rec is None:
                    slot = min(set(range(n_slots)) - {m[1] for m in model})
                    model.append([sid, slot, 1, clock])
                else:
                    slot = rec[1]
                    rec[2] += 1
                    rec[3] = clock
                assert t.put(sid, 8) == slot
            elif op == "touch" and ids_in:
                pick = rng.choice(ids_in, size=int(rng.integers(1, len(ids_in) + 1)), replace=False).tolist()
                clock += 1
                for m in model:
                    if m[0] in pick:
                        m[3] = clock
                t.touch(pick)
            elif op == "release" and ids_in:
                sid = int(rng.choice(ids_in))
                rec = next(m for m in model if m[0] == sid)
                if rec[2] == 0:
                    with pytest.raises(ValueError):
                        t.release(sid)
                else:
                    rec[2] -= 1
                    t.release(sid)
            elif op == "evict":
                idle = [m for m in model if m[2] == 0]
                if not idle:
                    with pytest.raises(LookupError):
                        t.evict_lru()
                else:
                    victim = min(idle, key=lambda m: (m[3], m[1]))
                    assert t.evict_lru() == victim[0]
                    model.remove(victim)
            assert t.n_used() == len(model)
            assert t.lookup(list(range(12))).tolist() == [next((m[1] for m in model if m[0] == i), -1) for i in range(12)]


def test_prefix_tree_hand_case_and_invariants():
    """Pin for PrefixTree: a batch counted by hand, then invariants on random batches (a node is never
    more loaded than its parent; the loads of all nodes of an id add up to segment_loads' figure for
    that id; eviction removes a node with everything below it and nothing else)."""
    t = orc.PrefixTree()
    # A = [1, 2, 3] x 5 tokens, B = [1, 2, 9] x 2, C = [7] x 4, D = [1, 1] x 1
    batch = t.walk([[1, 2, 3], [1, 2, 9], [7], [1, 1]], [5, 2, 4, 1])
    # node (1): 5 + 2 + 1 = 8; (1,2): 7; (1,2,3): 5; (7): 4; (1,2,9): 2; (1,1): 1
    assert t.ranked(batch) == [((1,), 8), ((1, 2), 7), ((1, 2, 3), 5), ((7,), 4), ((1, 2, 9), 2), ((1, 1), 1)]
    assert t.hot(2) == [((1,), 8), ((1, 2), 7)]
    # a second batch adds to the same nodes; its own loads start from zero
    batch2 = t.walk([[7, 8], [1, 2, 3]], [10, 1])
    assert t.ranked(batch2) == [((7,), 10), ((7, 8), 10), ((1,), 1), ((1, 2), 1), ((1, 2, 3), 1)]
    assert t.hot(3) == [((7,), 14), ((7, 8), 10), ((1,), 9)]
    # equal loads: the older node first (here the parent)
    assert [p for p, _ in t.hot()][:2] == [(7,), (7, 8)]
    t.evict(2)                                   # (1,2), (1,2,3), (1,2,9) go; (1), (1,1), (7), (7,8) stay
    assert sorted(t.load) == [(1,), (1, 1), (7,), (7, 8)]
    rng = np.random.default_rng(12)
    for trial in range(10):
        t = orc.PrefixTree()
        stems = [rng.integers(0, 6, size=int(rng.integers(1, 5))).tolist() for _ in range(3)]
        for b in range(3):
            lists = [stems[int(rng.integers(0, 3))][:int(rng.integers(0, 5))] + rng.integers(0, 6, size=int(rng.integers(0, 4))).tolist()
                     for _ in range(8)]
            ntok = rng.integers(0, 20, size=8).tolist()
            batch = t.walk(lists, ntok)
            for path, l in batch.items():
                if len(path) > 1:
                    assert batch[path[:-1]] >= l and t.load[path[:-1]] >= t.load[path]
            per_id = {}
            for path, l in batch.items():
                per_id[path[-1]] = per_id.get(path[-1], 0) + l
            assert per_id == dict(orc.segment_loads(lists, ntok))
            r = t.ranked(batch)
            assert [l for _, l in r] == sorted((l for _, l in r), reverse=True)
            for i, (path, _) in enumerate(r):                       # a parent always precedes its children
                if len(path) > 1:
                    assert path[:-1] in [p for p, _ in r[:i]]
        victim = int(rng.integers(0, 6))
        before = dict(t.load)
        t.evict(victim)
        assert set(t.load) == {p for p in before if victim not in p}


def test_content_segment_ids_follow_the_published_hash_and_the_prefix_rule():
    """Pins of the content-derived ids (Section 3.1, tree keyed by tokens): the byte hash against the
    published FNV-1a test vectors; two sequences get equal ids exactly for the whole segments of their common
    prefix; an id depends on every earlier token; a partly filled last segment has an id of its own."""
    assert orc.fnv1a64(b"") == 0xCBF29CE484222325
    assert orc.fnv1a64(b"a") == 0xAF63DC4C8601EC8C
    assert orc.fnv1a64(b"foobar") == 0x85944171F73967E8
    # tokens are hashed as 4 little-endian bytes each: one token 0x61 is the bytes "a\0\0\0"
    assert orc.content_segment_ids([0x61], 4) == [orc.fnv1a64(b"a\x00\x00\x00")]
    assert orc.content_segment_ids([0x6F6F66, 0x726162], 2) == [orc.fnv1a64(b"foo\x00bar\x00")]
    rng = np.random.default_rng(8)
    for case in range(20):
        C = int(rng.choice([1, 2, 3, 8]))
        a = rng.integers(0, 50000, size=int(rng.integers(0, 40))).tolist()
        lcp = int(rng.integers(0, len(a) + 1))
        b = a[:lcp] + rng.integers(50000, 60000, size=int(rng.integers(1, 20))).tolist()     # differs from a at position lcp
        ia, ib = orc.content_segment_ids(a, C), orc.content_segment_ids(b, C)
        assert len(ia) == (len(a) + C - 1) // C and len(ib) == (len(b) + C - 1) // C
        same = lcp // C                                    # whole segments inside the common prefix
        assert ia[:same] == ib[:same]
        assert all(x != y for x, y in zip(ia[same:], ib[same:]))          # (a 64-bit collision is not expected here)
        assert len(set(ia)) == len(ia)
        if a:
            c = [a[0] ^ 1] + a[1:]
            assert all(x != y for x, y in zip(ia, orc.content_segment_ids(c, C)))
            assert orc.content_segment_ids(a, C, salt=7) != ia
    # a partly filled tail: the id of [1, 2, 3] in segments of 2 is (hash of 1 2), (hash of 1 2 3)
    assert orc.content_segment_ids([1, 2, 3], 2)[1] == orc.content_segment_ids([1, 2, 3], 3)[0]
