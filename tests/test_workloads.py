"""Seeded input generators: determinism, shapes, and the statistics the configs call for."""
import numpy as np
import torch

from paper_2508_17219_amd import workloads as wl


def test_generator_is_random_access_and_deterministic():
    a = wl.normal_bf16_range(5, 2, 1000, 4096)
    b = wl.normal_bf16_range(5, 2, 1000 + 100, 50)
    assert torch.equal(a[100:150], b)
    c = wl.normal_bf16_range(5, 3, 1000, 4096)
    assert not torch.equal(a, c)
    x = wl.normal_bf16_range(1, 0, 0, 1 << 20).float()
    assert abs(float(x.mean())) < 5e-3 and abs(float(x.std()) - 1.0) < 5e-3
    # known first values keep the generator from drifting between machines
    ref = wl.bits_u16(wl.normal_bf16_range(0, 0, 0, 4))
    assert ref.dtype == np.uint16 and ref.shape == (4,)


def test_tiny_shape():
    b = wl.tiny()
    assert (b.q_heads, b.kv_heads, b.seg_len, b.n_slots, b.n_tokens, b.n_req) == (8, 2, 128, 8, 32, 1)
    assert len(b.seg_ids) == 4 and len(set(b.pool_slots.tolist())) == 4 and list(b.pool_fills) == [128] * 4
    assert b.q().shape == (32, 8, 128) and b.k_new().shape == (32, 2, 128)


def test_prefill_shape():
    b = wl.prefill()
    L = b.prefix_tokens()
    assert b.n_req == 16 and b.n_tokens == 16 * 512 and L.min() >= 8192 and L.max() <= 32768
    for r in range(16):
        ids = b.seg_ids[b.req_seg_ptr[r]:b.req_seg_ptr[r + 1]]
        assert list(ids[:8]) == list(range(8))
        assert len(ids) == -(-int(L[r]) // 256)
    assert len(np.unique(b.pool_slots)) == len(b.pool_ids) <= 4096
    assert (b.pool_fills < 256).sum() >= 1            # ragged tails exist


def test_decode_shape():
    b = wl.decode()
    L = b.prefix_tokens()
    assert b.n_req == 256 and b.n_tokens == 256 and L.max() <= 131072 and L.min() >= 1
    assert 8000 < np.median(L) < 32000
    assert len(b.pool_ids) == len(b.seg_ids)          # all private


def test_longctx_dedup():
    b = wl.longctx()
    assert b.n_req == 4 and len(b.seg_ids) == 1024 and len(b.pool_ids) < 1024 and len(b.pool_ids) <= 1000
    assert b.prefix_tokens().tolist() == [131072] * 4


def test_multiturn_slots_persist_across_turns():
    b0, b3, b7 = wl.multiturn(turn=0), wl.multiturn(turn=3), wl.multiturn(turn=7)
    assert b0.n_tokens == 64 * 256 and len(b0.pool_ids) == 16 and len(b7.pool_ids) == 16 + 64 * 28
    s3 = dict(zip(b3.pool_ids.tolist(), b3.pool_slots.tolist()))
    s7 = dict(zip(b7.pool_ids.tolist(), b7.pool_slots.tolist()))
    assert all(s7[k] == v for k, v in s3.items())
    assert b3.prefix_tokens().tolist() == [4096 + 3 * 1024] * 64


def test_segment_contents_depend_on_id_only():
    b = wl.tiny()
    k1, v1 = b.segment_kv(b.pool_ids[:2])
    k2, v2 = b.segment_kv(b.pool_ids[1:2])
    assert torch.equal(k1[1], k2[0]) and torch.equal(v1[1], v2[0])
    pk = torch.zeros(b.n_slots, b.seg_len, b.kv_heads, b.head_dim, dtype=torch.bfloat16)
    pv = torch.zeros_like(pk)
    b.fill_pool(pk, pv)
    assert torch.equal(pk[int(b.pool_slots[1])], k2[0])
