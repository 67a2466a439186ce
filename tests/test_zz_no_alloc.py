"""tl_fused_attn_static, the entry point for callers that cannot allocate device memory: the same
kernels as tl_fused_attn with the plan's work lists staged in a static device buffer.  Its output
must equal tl_fused_attn's bit for bit, on two calls in a row that share the buffer, the second
with a smaller input; and it must refuse a plan whose work lists do not fit."""
import numpy as np
import pytest
import torch

from paper_2508_17219_amd import binding as B
from paper_2508_17219_amd import workloads as wl
from tests import tl_harness as H

FAKE_K, FAKE_V = 0x100000, 0x200000


@pytest.mark.gpu
def test_static_buffer_variant_equals_fused_attn_on_two_calls_in_a_row():
    print("[case] tl_fused_attn_static vs tl_fused_attn", flush=True)
    big = wl.prefill(seed=45, n_req=4, new_tokens=150, lo=2000, hi=6000, seg_len=128, n_slots=256, n_shared=2)
    small = wl.prefill(seed=46, n_req=2, new_tokens=130, lo=200, hi=500, seg_len=64, n_slots=32, n_shared=0, hq=8, hkv=2)
    runs = [H.run_gpu(b, fuse=True, out_bf16=bf16) for b, bf16 in ((big, False), (small, True))]
    outs = []
    for run in runs:                         # back to back on one stream: the second call overwrites the first one's lists
        b = run.batch
        assert run.info.n_fused_tokens == b.n_tokens
        out = torch.full_like(run.out, float("nan"))
        lse = torch.full_like(run.lse, float("nan"))
        B.tl_fused_attn_static(run.pool, run.plan, run.q, run.k_new, run.v_new, b.scale, out, out.dtype == torch.bfloat16, lse)
        outs.append((out, lse))
    torch.cuda.synchronize()
    for run, (out, lse) in zip(runs, outs):
        assert torch.equal(out, run.out) and torch.equal(lse, run.lse)
        assert not torch.isnan(out.float()).any()
    # and against the oracle, to the usual bar (the fp32 run)
    res = H.compare_rows_device(runs[0], 1, np.array([0, 63, 64, 149]))
    assert res["ok"], res
    # once more on the first, larger plan: the buffer now holds the small plan's lists
    run = runs[0]
    out = torch.full_like(run.out, float("nan"))
    lse = torch.full_like(run.lse, float("nan"))
    B.tl_fused_attn_static(run.pool, run.plan, run.q, run.k_new, run.v_new, run.batch.scale, out, False, lse)
    torch.cuda.synchronize()
    assert torch.equal(out, run.out) and torch.equal(lse, run.lse)
    for run in runs:
        run.close()


def test_static_buffer_variant_refuses_lists_beyond_its_buffer():
    """Checked before any device call, so fake pointers do: 1500 requests x 700 segments of one tile
    each give 4.2 MB of tile lists, more than the 4 MiB buffer."""
    n_seg, n_req, C = 700, 1500, 64
    pool = B.tl_pool_create(n_seg, C, 1, 128, FAKE_K, FAKE_V)
    ids = np.arange(n_seg, dtype=np.uint64) + 10
    B.tl_pool_adopt(pool, ids, np.arange(n_seg), np.full(n_seg, C))
    row_ptr = (np.arange(n_req + 1) * 64).astype(np.int32)            # 64 tokens x 8 q heads = 512 rows: one-pass rows
    seg_ptr = (np.arange(n_req + 1) * n_seg).astype(np.int32)
    plan = B.tl_plan_create(pool, 8, row_ptr, seg_ptr, np.tile(ids, n_req), B.TL_PLAN_SELF_BLOCK | B.TL_PLAN_FUSE_ROWS)
    assert B.tl_plan_get_info(plan).n_fused_tokens == n_req * 64
    lib = B.load_library()
    rc = lib.tl_fused_attn_static(pool, plan, FAKE_K, FAKE_K, FAKE_V, 0.1, None, None, FAKE_K, 0, None, None)
    assert rc == B.TL_EINVAL and b"static buffer holds" in lib.tl_last_error()
    B.tl_plan_destroy(plan)
    B.tl_pool_destroy(pool)
