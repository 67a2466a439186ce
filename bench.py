#!/usr/bin/env python3
"""Benchmark of the segment-attention hot path on one MI355X.

A "step" is one pass of the whole path over one batch, with all inputs already resident in
HBM: tl_segment_attn (partial attention of every work item over its pool slots) +
tl_causal_block (self block of the new tokens) + tl_merge (LSE recombination) + tl_fused_attn
(the same three in one pass for requests whose rows fill whole row tiles; the plan decides,
TL_PLAN_FUSE_ROWS).  `--three-step` plans without the one-pass kernel.

Default workload: "prefill" (Llama-3-8B layer shape, 16 requests x 512 new tokens, prefixes
8k-32k tokens, first 2k shared) -- the configuration the prefill MFMA target is quoted on.
`--workload decode` times the 70B-shape decode batch (HBM-bound); by default a short decode
measurement is appended to the same JSON line under "decode".

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E


def measured_traffic(kernel, workload):
    """HBM bytes per launch of `kernel` on `workload`, from the rocprofv3 --pmc FETCH_SIZE /
    WRITE_SIZE runs summarised under profiles/ (scaled by a plain copy of known size); None if
    that pair has not been profiled."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as f:
            table = json.load(f)
    except (OSError, ValueError):
        return None
    ent = table.get("%s@%s" % (kernel, workload))
    return ent["hbm_bytes_per_launch"] if ent else None


def calibrate_copy(torch, n_bytes=1 << 30):
    """A plain device copy of known size, for scaling the FETCH_SIZE / WRITE_SIZE counters."""
    src = torch.ones(n_bytes // 2, dtype=torch.bfloat16, device="cuda")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"calibrate_copy_bytes_read": n_bytes, "calibrate_copy_bytes_written": n_bytes,
                      "kernel": "torch elementwise copy (bf16)", "launches": 3}))


def _setup(batch, torch, B):
    dev = "cuda"
    shape = (batch.n_slots, batch.seg_len, batch.kv_heads, batch.head_dim)
    pk = torch.zeros(shape, dtype=torch.bfloat16, device=dev)
    pv = torch.zeros(shape, dtype=torch.bfloat16, device=dev)
    batch.fill_pool(pk, pv)
    pool = B.tl_pool_create(batch.n_slots, batch.seg_len, batch.kv_heads, batch.head_dim, pk, pv)
    B.tl_pool_adopt(pool, batch.pool_ids, batch.pool_slots, batch.pool_fills)
    return pk, pv, pool


def run_workload(batch, steps, warmup, torch, B, split_segments=0, fuse=True, extra_flags=0, graph=False):
    """Times `steps` passes of the whole path; returns timings and the plan's work counters."""
    pk, pv, pool = _setup(batch, torch, B)
    plan_flags = B.TL_PLAN_SELF_BLOCK | (B.TL_PLAN_FUSE_ROWS if fuse else 0) | extra_flags
    t_plan = []
    for _ in range(3):       # host-side cost of a plan (built once per iteration, used by every layer)
        t0 = time.perf_counter()
        plan = B.tl_plan_create(pool, batch.q_heads, batch.req_row_ptr, batch.req_seg_ptr, batch.seg_ids, plan_flags,
                                split_segments)
        t_plan.append((time.perf_counter() - t0) * 1e3)
        if len(t_plan) < 3:
            B.tl_plan_destroy(plan)
    info = B.tl_plan_get_info(plan)
    dev = "cuda"
    q, kn, vn = batch.q(dev), batch.k_new(dev), batch.v_new(dev)
    H, D = batch.q_heads, batch.head_dim
    outp = torch.empty((max(info.n_partial_rows, 1), H, D), dtype=torch.float32, device=dev)
    lsep = torch.empty((max(info.n_partial_rows, 1), H), dtype=torch.float32, device=dev)
    out = torch.empty((info.n_tokens, H, D), dtype=torch.bfloat16, device=dev)
    lse = torch.empty((info.n_tokens, H), dtype=torch.float32, device=dev)
    scale = batch.scale

    # In the timed region only the dominant call is bracketed by HIP events (every event is a marker
    # in the stream and costs the GPU a few microseconds); the other calls are timed in a short loop
    # of their own afterwards.
    all_fused = info.n_fused_tokens == info.n_tokens and info.n_tokens > 0 and info.n_items == 0
    dom = 3 if all_fused else 0           # index of the dominant call: tl_fused_attn or tl_segment_attn
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(steps)]

    def step(marks=None, which=None):
        calls = (lambda: B.tl_segment_attn(pool, plan, q, scale, outp, lsep),
                 lambda: B.tl_causal_block(plan, q, kn, vn, scale, outp, lsep),
                 lambda: B.tl_merge(plan, outp, lsep, out, True, lse),
                 lambda: B.tl_fused_attn(pool, plan, q, kn, vn, scale, out, True, lse, prior_partial=outp, prior_lse=lsep))
        if marks and which is None: marks[0].record()          # five marks: one before, one after every call
        for i, call in enumerate(calls):
            if marks and which == i: marks[0].record()         # two marks: around call `which` only
            call()
            if marks and which is None: marks[i + 1].record()
            if marks and which == i: marks[1].record()

    for _ in range(max(warmup, 1)):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(ev[i], dom)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    dom_ms = sum(e[0].elapsed_time(e[1]) for e in ev) / steps
    n_side = min(steps, 20)
    ev5 = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(n_side)]
    for i in range(n_side):
        step(ev5[i])
    torch.cuda.synchronize()
    seg_ms = sum(e[0].elapsed_time(e[1]) for e in ev5) / n_side
    causal_ms = sum(e[1].elapsed_time(e[2]) for e in ev5) / n_side
    merge_ms = sum(e[2].elapsed_time(e[3]) for e in ev5) / n_side
    fused_ms = sum(e[3].elapsed_time(e[4]) for e in ev5) / n_side
    if dom == 3:
        fused_ms = dom_ms                 # the dominant call's time is the one from the timed region
    else:
        seg_ms = dom_ms
    res = {
        "ms_per_step": (t1 - t0) * 1e3 / steps,
        "segment_attn_ms": seg_ms, "causal_block_ms": causal_ms, "merge_ms": merge_ms, "fused_attn_ms": fused_ms,
        "info": {n: getattr(info, n) for n, _ in info._fields_},
        "plan_create_ms": min(t_plan),
        "checksum": float(out.float().abs().mean().item()),
    }
    if graph:
        # the same step captured once as a HIP graph and replayed: what the launches cost the host
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step()
        g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            g.replay()
        torch.cuda.synchronize()
        res["graph_ms_per_step"] = (time.perf_counter() - t0) * 1e3 / steps
        res["graph_checksum"] = float(out.float().abs().mean().item())
        del g
    B.tl_plan_destroy(plan)
    B.tl_pool_destroy(pool)
    del pk, pv, outp, lsep, out, lse, q, kn, vn
    torch.cuda.empty_cache()
    return res


_probe_lib = None


def _probe():
    """libtlprobe.so: a kernel of MFMAs only.  A measurement aid of this benchmark, built beside the
    library by paper_2508_17219_amd.build and loaded here alone (no part of the C ABI)."""
    global _probe_lib
    if _probe_lib is None:
        import ctypes as C
        from paper_2508_17219_amd import build as _build
        if not os.path.exists(_build.PROBE_LIB):
            _build.build_probe(verbose=False)
        lib = C.CDLL(_build.PROBE_LIB)
        lib.tlprobe_mfma.restype = C.c_int32
        lib.tlprobe_mfma.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.POINTER(C.c_double), C.c_void_p]
        lib.tlprobe_mfma_kind.restype = C.c_int32
        lib.tlprobe_mfma_kind.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.POINTER(C.c_double), C.c_void_p]
        lib.tlprobe_issue.restype = C.c_int32
        lib.tlprobe_issue.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_double)]
        _probe_lib = lib
    return _probe_lib


def mfma_sustained(torch, random_operands, iters=2000, reps=3, kind=None, idle_every=0, times=None):
    """TFLOP/s of the matrix unit alone (no memory, LDS or vector work), best of `reps` launches.
    kind/idle_every select one of the probe's operand and throttling variants instead."""
    import ctypes as C
    lib = _probe()
    scratch = torch.zeros(16, dtype=torch.float32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream or None
    best = 0.0
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fl = C.c_double(0.0)
        e0.record()
        if kind is None:
            rc = lib.tlprobe_mfma(int(bool(random_operands)), iters, scratch.data_ptr(), C.byref(fl), st)
        else:
            rc = lib.tlprobe_mfma_kind(kind, idle_every, iters, scratch.data_ptr(), C.byref(fl), st)
        e1.record()
        torch.cuda.synchronize()
        if rc != 0:
            raise RuntimeError("tlprobe_mfma failed (%d)" % rc)
        if times is not None:
            times.append(e0.elapsed_time(e1))
        best = max(best, fl.value / (e0.elapsed_time(e1) * 1e-3) / 1e12)
    return best


def probe_mfma(torch, iters=8000, reps=5):
    """Sustained rate of the matrix unit alone, with constant and with changing operands: context
    for the published peak the roofline fractions are taken against."""
    out = {}
    for name, rnd in (("constant_operands", False), ("changing_random_operands", True)):
        best = mfma_sustained(torch, rnd, iters, reps)
        out[name] = {"TFLOP/s": best, "frac_of_peak": best / PEAK_BF16_TFLOPS}
    # what the power of the matrix unit depends on: the values inside an instruction or the change between instructions
    kinds = {}
    for name, kind in (("random_operands_that_never_change", 0), ("plus_minus_one_random_signs", 1),
                       ("random_mantissas_one_exponent_positive", 2), ("A_changing_B_one", 3), ("A_one_B_changing", 4),
                       ("both_changing", 5)):
        kinds[name] = round(mfma_sustained(torch, True, 3000, 3, kind=kind), 1)
    # the same instructions on the same operands made to take more cycles (the wave idles after every n-th MFMA)
    throttled = []
    for idle in (32, 16, 8, 4, 2):
        ts = []
        mfma_sustained(torch, True, 3000, 4, kind=5, idle_every=idle, times=ts)
        throttled.append({"idle_after_every": idle, "ms": round(min(ts[1:]), 4)})
    print(json.dumps({"probe": "mfma_f32_32x32x16_bf16 only, 1024 workgroups x 8 waves, %d x 32 instructions per wave, "
                               "best of %d launches" % (iters, reps), "peak_TFLOP/s": PEAK_BF16_TFLOPS, **out,
                      "operand_kinds_TFLOP/s": kinds, "throttled_one_wave_per_simd": throttled}))


def probe_issue(torch, iters=20000):
    """Issue cycles of an MFMA and of the softmax's vector instructions on one SIMD, alone and together, with one
    and two waves per SIMD (cycle counter per wave; a group = a quarter of a loop iteration)."""
    import ctypes as C
    lib = _probe()
    torch.zeros(1, device="cuda")
    rows = []
    for name, mode, waves in (("8 v_fma_f32", 0, 1), ("8 v_add_f32", 1, 1), ("8 v_exp_f32", 2, 1), ("8 v_cvt_pk_bf16_f32", 3, 1),
                              ("8 v_max3_f32", 4, 1), ("8 v_perm_b32", 5, 1), ("1 MFMA 32x32x16 bf16", 10, 1), ("1 MFMA", 10, 2),
                              ("1 MFMA + one element's fma, exp, add, half a convert", 11, 1), ("the same", 11, 2),
                              ("1 MFMA + two elements' softmax", 12, 1), ("the same", 12, 2),
                              ("waves 0-3: 1 MFMA; waves 4-7: 8 v_fma_f32", 20, 2)):
        a, b = C.c_double(0.0), C.c_double(0.0)
        rc = lib.tlprobe_issue(mode, waves, iters, C.byref(a), C.byref(b))
        if rc != 0:
            raise RuntimeError("tlprobe_issue failed (%d)" % rc)
        rows.append({"per_group": name, "waves_per_simd": waves, "cycles_waves_0_3": round(a.value, 1),
                     "cycles_waves_4_7": round(b.value, 1) if waves == 2 else None})
    print(json.dumps({"probe": "issue cycles per group on one SIMD (256 workgroups, one per CU; loop overhead included)", "rows": rows}))


def run_session_loop(steps, warmup, torch, B, wl, per_chain_append=False):
    """The multi-turn workload as one closed loop on the device: for turn 0..7, plan the batch of
    all sessions' new tokens over (shared prompt + the history appended so far), run the step,
    then append each session's next 1024 KV rows (4 segments) to its chain (tl_pool_append_batch:
    all 64 chains in one call; `per_chain_append`: 64 calls of tl_pool_append).
    Returns per-turn times (HIP events; host clock for the plans) averaged over `steps` passes."""
    import numpy as np
    turns = [wl.multiturn(turn=t) for t in range(8)]
    b0 = turns[0]
    dev = "cuda"
    shape = (b0.n_slots, b0.seg_len, b0.kv_heads, b0.head_dim)
    pk = torch.zeros(shape, dtype=torch.bfloat16, device=dev)
    pv = torch.zeros(shape, dtype=torch.bfloat16, device=dev)
    b0.fill_pool(pk, pv)                                   # the shared prompt's 16 segments
    n_s, grow = b0.n_req, 4 * b0.seg_len
    H, D = b0.q_heads, b0.head_dim
    qs = [(t.q(dev), t.k_new(dev), t.v_new(dev)) for t in turns]
    # rows each session appends after a turn (its 256 new tokens + 768 filler tokens): seeded noise
    rows_k = wl.normal_bf16_range(b0.seed, wl.STREAM_KNEW, 1 << 40, n_s * grow * b0.kv_heads * D, dev).view(n_s, grow, b0.kv_heads, D)
    rows_v = wl.normal_bf16_range(b0.seed, wl.STREAM_VNEW, 1 << 40, n_s * grow * b0.kv_heads * D, dev).view(n_s, grow, b0.kv_heads, D)
    out = torch.empty((b0.n_tokens, H, D), dtype=torch.bfloat16, device=dev)
    lse = torch.empty((b0.n_tokens, H), dtype=torch.float32, device=dev)
    flags = B.TL_PLAN_SELF_BLOCK | B.TL_PLAN_FUSE_ROWS
    shared = [int(x) for x in b0.pool_ids]
    row_ptr = b0.req_row_ptr
    acc = {"attn_ms": np.zeros(8), "append_ms": np.zeros(8), "plan_ms": np.zeros(8), "flops": np.zeros(8)}
    wall = 0.0
    for rep in range(warmup + steps):
        pool = B.tl_pool_create(b0.n_slots, b0.seg_len, b0.kv_heads, D, pk, pv)
        B.tl_pool_adopt(pool, b0.pool_ids, b0.pool_slots, b0.pool_fills)
        chains = [[] for _ in range(n_s)]
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(8)]
        plan_ms, flops, plans = [], [], []
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        for t in range(8):
            lists = [shared + c for c in chains]
            seg_ptr = np.concatenate([[0], np.cumsum([len(l) for l in lists])]).astype(np.int32)
            ids = np.array([i for l in lists for i in l], dtype=np.uint64)
            t0 = time.perf_counter()
            plan = B.tl_plan_create(pool, H, row_ptr, seg_ptr, ids, flags, 0)
            plan_ms.append((time.perf_counter() - t0) * 1e3)
            info = B.tl_plan_get_info(plan)
            assert info.n_fused_tokens == b0.n_tokens      # every request takes the one-pass kernel
            flops.append(4.0 * H * D * (info.prefix_pairs + info.self_pairs))
            q, kn, vn = qs[t]
            ev[t][0].record()
            B.tl_fused_attn(pool, plan, q, kn, vn, b0.scale, out, True, lse)
            ev[t][1].record()
            new_ids = [[wl._private_id(s_, len(shared) + len(chains[s_]) + j) for j in range(4)] for s_ in range(n_s)]
            if per_chain_append:
                for s_ in range(n_s):
                    B.tl_pool_append(pool, None, new_ids[s_], rows_k[s_], rows_v[s_], grow)
            else:
                B.tl_pool_append_batch(pool, [None] * n_s, new_ids, [grow] * n_s, rows_k, rows_v)
            for s_ in range(n_s):
                chains[s_] += new_ids[s_]
            ev[t][2].record()
            plans.append(plan)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t_start
        if rep >= warmup:
            wall += dt
            acc["attn_ms"] += [e[0].elapsed_time(e[1]) for e in ev]
            acc["append_ms"] += [e[1].elapsed_time(e[2]) for e in ev]
            acc["plan_ms"] += plan_ms
            acc["flops"] = np.array(flops)
        for plan in plans:
            B.tl_plan_destroy(plan)
        B.tl_pool_destroy(pool)
    for k in ("attn_ms", "append_ms", "plan_ms"):
        acc[k] = acc[k] / steps
    acc["wall_ms"] = wall * 1e3 / steps
    acc["tokens"] = 8 * b0.n_tokens
    acc["append_bytes_per_turn"] = 2.0 * 2 * n_s * grow * b0.kv_heads * D * 2     # K and V, read + written
    acc["checksum"] = float(out.float().abs().mean().item())
    return acc


def algorithmic_work(batch, info):
    """Flops and minimum HBM bytes of one pass (what the method must do)."""
    hq, hkv, d = batch.q_heads, batch.kv_heads, batch.head_dim
    flops_prefix = 4.0 * hq * d * info["prefix_pairs"]
    flops_self = 4.0 * hq * d * info["self_pairs"]
    kv_bytes = 4.0 * hkv * d * info["unique_kv_tokens"]          # K and V, bf16, each unique slot once
    q_bytes = 2.0 * hq * d * info["n_tokens"]
    part_rows = info["n_partial_rows"] - (info["n_tokens"] if info["self_row_base"] >= 0 else 0)
    part_bytes = part_rows * hq * (d + 1) * 4.0
    # one-pass rows: K/V of the new tokens are read, the final bf16 output and fp32 LSE are written
    fused_io_bytes = info["n_fused_tokens"] * (4.0 * hkv * d + hq * (2.0 * d + 4.0))
    return {"flops_prefix": flops_prefix, "flops_self": flops_self, "flops_tiles": 4.0 * hq * d * info.get("tile_pairs", 0), "kv_bytes": kv_bytes, "q_bytes": q_bytes,
            "partial_bytes": part_bytes, "fused_io_bytes": fused_io_bytes}


def three_step_report(b, r, w):
    """Per-kernel times and roofline fractions of a plan that keeps shared runs as work items:
    tl_segment_attn (row tiles over the pool work items), then either tl_causal_block + tl_merge
    (plain three steps) or tl_fused_attn over each request's private end and new tokens, merging the
    work items' partials in (TL_PLAN_FUSE_TAILS)."""
    info = r["info"]
    hq, d = b.q_heads, b.head_dim
    item_flops = 4.0 * hq * d * info["item_pairs"]
    seg = item_flops / (r["segment_attn_ms"] * 1e-3) / 1e12
    out = {"ms_per_step": r["ms_per_step"], "merged_tok_s": b.n_tokens / (r["ms_per_step"] * 1e-3),
           "work_items": info["n_items"], "row_tiles": info["n_tiles"], "causal_tiles": info["n_causal_tiles"],
           "one_pass_tiles": info["n_fused_tiles"], "prior_rows_merged_in_kernel": info["n_prior_rows"],
           "segment_attn": {"ms": r["segment_attn_ms"], "bound": "mfma", "achieved": seg, "unit": "TFLOP/s",
                            "frac": seg / PEAK_BF16_TFLOPS}}
    if info["n_causal_tiles"] > 0:
        cau = w["flops_self"] / (r["causal_block_ms"] * 1e-3) / 1e12
        out["causal_block"] = {"ms": r["causal_block_ms"], "bound": "mfma", "achieved": cau, "unit": "TFLOP/s",
                               "frac": cau / PEAK_BF16_TFLOPS}
    if info["n_merge_entries"] > 0:
        merge_bytes = info["n_merge_entries"] * hq * (d + 1) * 4.0 + info["n_tokens"] * hq * (2.0 * d + 4.0)
        mer = merge_bytes / (r["merge_ms"] * 1e-3) / 1e9
        out["merge"] = {"ms": r["merge_ms"], "bound": "hbm", "achieved": mer, "unit": "GB/s", "frac": mer / PEAK_HBM_GBS,
                        "algorithmic_bytes": merge_bytes}
    if info["n_fused_tiles"] > 0:
        fl = w["flops_prefix"] - item_flops + w["flops_self"]
        fu = fl / (r["fused_attn_ms"] * 1e-3) / 1e12
        out["fused_attn"] = {"ms": r["fused_attn_ms"], "bound": "mfma", "achieved": fu, "unit": "TFLOP/s",
                             "frac": fu / PEAK_BF16_TFLOPS}
    return out


def cpu_baseline(batch, budget_s=15.0):
    """The fp64 oracle, as it stands, timed on this host on a bounded sample of the workload:
    whole new tokens (all heads, full prefix + self block), taking requests in order of
    distance from the batch's median prefix length until the time budget is used."""
    import numpy as np
    from threadpoolctl import threadpool_info
    from tests import tl_harness as H      # test-side glue around oracle/ (generator -> oracle inputs)
    from oracle import tokenlake_oracle as orc
    L = batch.prefix_tokens()
    order = np.argsort(np.abs(L - np.median(L)), kind="stable")
    n_done, t_used, used_reqs = 0, 0.0, []
    for r in order:
        if t_used >= budget_s:
            break
        r = int(r)
        qb, pk, pv, slots, fills, kn, vn = H.host_request_inputs(batch, r)     # input generation: untimed
        lq = qb.shape[0]
        if lq == 0:
            continue
        used_reqs.append(r)
        done_r, n = 0, min(2, lq)
        while done_r < lq and t_used < budget_s:
            rows = np.arange(done_r, min(lq, done_r + n))
            t0 = time.perf_counter()
            gk, gv = orc.gather_segments(pk, pv, slots, fills)
            k_all = np.concatenate([gk, kn], axis=0)
            v_all = np.concatenate([gv, vn], axis=0)
            orc.partial_attention(qb[rows], k_all, v_all, batch.scale, n_visible=gk.shape[0] + rows + 1)
            dt = time.perf_counter() - t0
            t_used += dt
            done_r += len(rows)
            # next chunk: aim at a quarter of what is left of the budget
            per_row = dt / len(rows)
            n = int(max(1, min(lq - done_r, (budget_s - t_used) / 4 / max(per_row, 1e-6))))
        n_done += done_r
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    # cores: what this process may run on; numpy's BLAS pool (the only threads the oracle uses) is
    # sized from the environment and never exceeds it on the boxes this runs on
    avail = len(os.sched_getaffinity(0))
    return {"value": n_done / t_used, "unit": "tok/s", "cores": int(min(avail, threads)), "cores_available": avail,
            "blas_threads": int(threads), "kind": "oracle",
            "sample": "%d new tokens (all %d heads) of %d request(s) nearest the batch's median prefix length "
                      "(requests %s, prefixes %s tokens), full prefix + causal self block, numpy fp64, %.1f s"
                      % (n_done, batch.q_heads, len(used_reqs), used_reqs, [int(L[r]) for r in used_reqs], t_used)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="prefill", choices=["prefill", "decode", "longctx", "multiturn", "tiny"])
    ap.add_argument("--turn", type=int, default=7, help="turn of the multi-turn workload (0..7)")
    ap.add_argument("--split-segments", type=int, default=0)
    ap.add_argument("--n-req", type=int, default=0, help="decode workload only: number of requests (default 256)")
    ap.add_argument("--median-prefix", type=int, default=0, help="decode workload only: median prefix length (default 16384)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sharing", action="store_true", help="plan with TL_PLAN_NO_SHARING (one item chain per request)")
    ap.add_argument("--three-step", action="store_true",
                    help="plan without TL_PLAN_FUSE_ROWS: every request goes through partials and the merge")
    ap.add_argument("--tails", action="store_true",
                    help="plan with TL_PLAN_FUSE_TAILS alone: shared runs as work items read once, private ends and new "
                         "tokens in one pass that merges the shared runs' partials in")
    ap.add_argument("--no-decode", action="store_true", help="skip the appended decode measurement")
    ap.add_argument("--no-extra", action="store_true",
                    help="skip the appended short measurements (three-step plan, other named workloads, MFMA-only rate)")
    ap.add_argument("--session-loop", action="store_true",
                    help="multi-turn workload as a closed loop: 8 turns of plan + attention + tl_pool_append")
    ap.add_argument("--per-chain-append", action="store_true",
                    help="with --session-loop: one tl_pool_append call per session instead of one batched call per turn")
    ap.add_argument("--graph", action="store_true",
                    help="also time the step replayed from a HIP graph (reported as graph_ms_per_step)")
    ap.add_argument("--probe-mfma", action="store_true",
                    help="only run the MFMA-only probe kernel (constant and changing operands) and exit")
    ap.add_argument("--probe-issue", action="store_true",
                    help="only run the issue-cycle microbenchmark (MFMA and softmax vector instructions on one SIMD) and exit")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a 1 GiB device copy (to scale rocprofv3 FETCH_SIZE/WRITE_SIZE) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding or collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2508_17219_amd import binding as B
    from paper_2508_17219_amd import workloads as wl
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    from paper_2508_17219_amd import build as _build
    _build.ensure_built(verbose=False)       # builds only if no library is there
    B.load_library()
    if args.probe_issue:
        probe_issue(torch)
        return
    if args.probe_mfma:
        probe_mfma(torch)
        return
    if args.calibrate_copy:
        calibrate_copy(torch)
        return

    if args.session_loop:
        r = run_session_loop(args.steps, max(args.warmup, 1), torch, B, wl, args.per_chain_append)
        gpu_ms = float(r["attn_ms"].sum() + r["append_ms"].sum())
        ach = float(r["flops"].sum()) / (float(r["attn_ms"].sum()) * 1e-3) / 1e12
        print(json.dumps({
            "metric": "merged tok/s (one layer; 8 turns of 64 sessions: plan, one-pass attention, append of the turn's KV)",
            "value": r["tokens"] / (r["wall_ms"] * 1e-3), "unit": "tok/s", "n_gpus": 1, "steps": args.steps,
            "warmup": max(args.warmup, 1), "ms_per_step": r["wall_ms"], "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "multiturn[closed loop, turns 0-7]", "new_tokens": r["tokens"]},
            "roofline": {"kernel": "row_tile_attn_kernel<one pass>", "bound": "mfma", "achieved": ach,
                         "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS, "traffic": None,
                         "algorithmic_flops": float(r["flops"].sum()), "avg_kernel_ms": float(r["attn_ms"].mean())},
            "per_turn_ms": {"attention": [round(float(x), 4) for x in r["attn_ms"]],
                            "append": [round(float(x), 4) for x in r["append_ms"]],
                            "plan_host": [round(float(x), 4) for x in r["plan_ms"]]},
            "gpu_ms_per_pass": gpu_ms,
            "append": {"bytes_per_turn": r["append_bytes_per_turn"],
                       "GB_per_s": r["append_bytes_per_turn"] / (float(r["append_ms"].mean()) * 1e-3) / 1e9,
                       "launches_per_turn": 64 if args.per_chain_append else 2},
        }))
        return

    decode_kw = {}
    if args.n_req:
        decode_kw["n_req"] = args.n_req
    if args.median_prefix:
        decode_kw["median"] = args.median_prefix
    maker = {"prefill": wl.prefill, "decode": lambda: wl.decode(**decode_kw), "longctx": wl.longctx, "tiny": wl.tiny,
             "multiturn": lambda: wl.multiturn(turn=args.turn)}[args.workload]
    batch = maker()
    if args.workload == "decode" and decode_kw:
        batch.name = "decode[%s]" % ", ".join("%s=%d" % kv for kv in sorted(decode_kw.items()))
    res = run_workload(batch, args.steps, args.warmup, torch, B, args.split_segments, fuse=not (args.three_step or args.tails),
                       extra_flags=(B.TL_PLAN_NO_SHARING if args.no_sharing else 0) | (B.TL_PLAN_FUSE_TAILS if args.tails else 0),
                       graph=args.graph)
    work = algorithmic_work(batch, res["info"])
    tok_s = batch.n_tokens / (res["ms_per_step"] * 1e-3)

    def roofline_for(b, r, w):
        seg_s = r["segment_attn_ms"] * 1e-3
        if b.name.startswith("decode"):
            by = w["kv_bytes"] + w["q_bytes"] + w["partial_bytes"]
            ach = by / seg_s / 1e9
            return {"kernel": "splitk_unit_attn_kernel", "bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": ach / PEAK_HBM_GBS,
                    "traffic": measured_traffic("splitk_unit_attn_kernel", b.name),
                    "algorithmic_bytes": by, "avg_kernel_ms": r["segment_attn_ms"]}
        if r["info"]["n_fused_tokens"] == r["info"]["n_tokens"] and r["info"]["n_items"] == 0:
            # every request takes the one-pass kernel: pool tiles and causal block in one launch
            fl = w["flops_prefix"] + w["flops_self"]
            ach = fl / (r["fused_attn_ms"] * 1e-3) / 1e12
            return {"kernel": "row_tile_attn_kernel<one pass>", "bound": "mfma", "achieved": ach, "peak": PEAK_BF16_TFLOPS,
                    "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS,
                    "traffic": measured_traffic("row_tile_attn_kernel<one pass>", b.name),
                    "algorithmic_flops": fl, "algorithmic_bytes": w["kv_bytes"] + w["q_bytes"] + w["fused_io_bytes"],
                    # what the matrix unit was given: a slot that a list names m times is walked once, weighted m
                    "executed_flops": w["flops_tiles"] + w["flops_self"],
                    "executed_tflops": (w["flops_tiles"] + w["flops_self"]) / (r["fused_attn_ms"] * 1e-3) / 1e12,
                    "avg_kernel_ms": r["fused_attn_ms"]}
        item_flops = 4.0 * b.q_heads * b.head_dim * r["info"]["item_pairs"]      # the work items' share of the prefix flops
        ach = item_flops / seg_s / 1e12
        return {"kernel": "row_tile_attn_kernel", "bound": "mfma", "achieved": ach, "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS,
                "traffic": measured_traffic("row_tile_attn_kernel", b.name),
                "algorithmic_flops": item_flops, "avg_kernel_ms": r["segment_attn_ms"]}

    line = {
        "metric": "merged tok/s (one layer: attention over the segment pool + causal self block, partials merged)",
        "value": tok_s, "unit": "tok/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": batch.name, "n_req": batch.n_req, "new_tokens": batch.n_tokens,
                   "q_heads": batch.q_heads, "kv_heads": batch.kv_heads, "head_dim": batch.head_dim,
                   "seg_len": batch.seg_len, "prefix_tokens_total": int(batch.prefix_tokens().sum()),
                   "seed": batch.seed},
        "roofline": roofline_for(batch, res, work),
        "kernels_ms": {"segment_attn": res["segment_attn_ms"], "causal_block": res["causal_block_ms"],
                       "merge": res["merge_ms"], "fused_attn": res["fused_attn_ms"]},
        "plan": {"fused_tokens": res["info"]["n_fused_tokens"], "row_tiles": res["info"]["n_tiles"],
                 "split_k_units": res["info"]["n_units"], "causal_tiles": res["info"]["n_causal_tiles"],
                 "fused_row_tiles": res["info"]["n_fused_tiles"], "host_ms_to_build": res["plan_create_ms"]},
        "attn_tflops": (work["flops_prefix"] + work["flops_self"]) /
                       ((res["segment_attn_ms"] + res["causal_block_ms"] + res["fused_attn_ms"]) * 1e-3) / 1e12,
    }
    if args.graph:
        line["hip_graph"] = {"ms_per_step": res["graph_ms_per_step"],
                             "same_output": res["graph_checksum"] == res["checksum"]}
    if args.workload == "prefill" and not args.no_extra:
        # the matrix unit's own sustained rate on this machine in this run: what tells a slow box from a slow kernel
        rl = line["roofline"]
        rl["mfma_sustained"] = {"constant_operands_TFLOP/s": mfma_sustained(torch, False),
                                "changing_operands_TFLOP/s": mfma_sustained(torch, True),
                                "note": "a kernel of MFMAs only (no memory, LDS or vector work), best of 3 launches"}
        rl["frac_of_sustained_changing"] = rl["achieved"] / rl["mfma_sustained"]["changing_operands_TFLOP/s"]
        # the named three-step path on the same workload: partials of every work item, causal block, merge
        side_steps = max(5, min(args.steps, 20))
        r3 = run_workload(batch, side_steps, 3, torch, B, args.split_segments, fuse=False)
        line["three_step"] = three_step_report(batch, r3, algorithmic_work(batch, r3["info"]))
        # hot segments read once for all their requesters' rows, private ends and new tokens in one pass
        # that merges the shared runs' partials in (TL_PLAN_FUSE_TAILS): this workload and multi-turn turn 7
        line["shared_runs_once"] = []
        for sb in (batch, wl.multiturn(turn=7)):
            rt = run_workload(sb, side_steps, 3, torch, B, args.split_segments, fuse=False, extra_flags=B.TL_PLAN_FUSE_TAILS)
            rep_ = three_step_report(sb, rt, algorithmic_work(sb, rt["info"]))
            rep_["workload"] = sb.name
            line["shared_runs_once"].append(rep_)
        # the other named workloads, short runs, default plan
        line["configs"] = []
        for mk in (wl.tiny, wl.longctx, lambda: wl.multiturn(turn=0), lambda: wl.multiturn(turn=7)):
            ob = mk()
            orr = run_workload(ob, side_steps, 3, torch, B, args.split_segments, fuse=True)
            orl = roofline_for(ob, orr, algorithmic_work(ob, orr["info"]))
            # `achieved` counts flops per list entry (what the method asks for); `frac` is what the matrix
            # unit was given (a slot that a list names m times is walked once, weighted) over the peak
            ex_t = orl.get("executed_tflops", orl["achieved"])
            line["configs"].append({"workload": ob.name, "new_tokens": ob.n_tokens, "ms_per_step": orr["ms_per_step"],
                                    "merged_tok_s": ob.n_tokens / (orr["ms_per_step"] * 1e-3), "kernel": orl["kernel"],
                                    "achieved": orl["achieved"], "executed": ex_t, "unit": orl["unit"],
                                    "frac": ex_t / orl["peak"], "steps": side_steps})
    if args.workload != "decode" and not args.no_decode:
        db = wl.decode()
        dres = run_workload(db, max(3, args.steps // 4), 1, torch, B, args.split_segments, fuse=not args.three_step)
        dwork = algorithmic_work(db, dres["info"])
        line["decode"] = {"workload": db.name, "ms_per_step": dres["ms_per_step"],
                          "merged_tok_s": db.n_tokens / (dres["ms_per_step"] * 1e-3),
                          "roofline": roofline_for(db, dres, dwork),
                          "kernels_ms": {"segment_attn": dres["segment_attn_ms"], "causal_block": dres["causal_block_ms"],
                                         "merge": dres["merge_ms"], "fused_attn": dres["fused_attn_ms"]}}
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(batch)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
