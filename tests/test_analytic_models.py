"""Pins of oracle/analytic_oracle.py against what the paper prints, and the library's
tl_model_* calls against that oracle (host-only code: runs without a GPU)."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import analytic_oracle as ao
from paper_2508_17219_amd import binding as B

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_analytic_figures.txt")


def _golden():
    out = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].split()
        if line:
            out[line[0]] = (float(line[1]), line[2])
    return out


# the paper's testbed: A100-80GB (dense 16-bit 312 TFLOP/s, HBM2e ~2.0 TB/s)
A100_FLOPS, A100_MEM = 312e12, 2.0e12


def test_kv_bytes_per_token_is_the_papers_16_kib():
    g = _golden()
    d = int(g["hidden_size"][0])
    assert ao.kv_bytes_per_token(d) == g["kv_bytes_per_request_per_layer"][0] * 1024


def test_threshold_and_overhead_printed_by_the_paper_are_mutually_consistent():
    """The paper prints C ~ 568 tokens and, at that size, 4.66 us of communication; it does not
    print its network latency.  At the threshold T_comp(C) = T_comm, so the two figures fix
    k_comp = 4.66 us / 568 = 8.2 ns per token, which must be what the formula gives for the
    paper's GPU and model: 4 d / B_mem with d = 4096 and the A100's ~2 TB/s (the compute side,
    4 d / F, is 150 times smaller).  A dropped factor of two anywhere (2d for 4d, one-way
    latency, one message) breaks one of the assertions."""
    g = _golden()
    d = int(g["hidden_size"][0])
    c_paper, t_paper = g["segment_threshold"][0], g["comm_overhead"][0] * 1e-6
    k = ao.segment_time_per_token(d, Fraction(A100_FLOPS), Fraction(A100_MEM))
    assert float(k) == pytest.approx(t_paper / c_paper, rel=5e-3)           # 8.19 vs 8.20 ns
    assert float(Fraction(4 * d) / Fraction(A100_FLOPS)) < float(k) / 100    # memory-bound side decides
    # the latency that reproduces 4.66 us with the printed link bandwidth ...
    bw = g["nvlink_bandwidth"][0] * 1e9
    alpha = (Fraction(t_paper) - Fraction(4 * d) / Fraction(bw)) / 2
    assert 2e-6 < float(alpha) < 2.5e-6                                       # a plausible one-way NVLink/NCCL latency
    assert float(ao.comm_time(d, alpha, Fraction(bw))) == pytest.approx(t_paper, rel=1e-12)
    # ... gives the printed threshold
    c = ao.segment_threshold(d, Fraction(A100_FLOPS), Fraction(A100_MEM), alpha, Fraction(bw))
    assert abs(float(c) - c_paper) <= 1.0
    # and at the threshold the two times are equal, below it communication costs more
    assert ao.segment_time(c, d, Fraction(A100_FLOPS), Fraction(A100_MEM)) == ao.comm_time(d, alpha, Fraction(bw))
    assert ao.segment_time(c / 2, d, Fraction(A100_FLOPS), Fraction(A100_MEM)) < ao.comm_time(d, alpha, Fraction(bw))


def test_segment_time_takes_the_slower_roofline():
    # compute-bound when flops are scarce: 4 d C / F
    assert ao.segment_time(10, 8, 16, 10 ** 9) == Fraction(4 * 8 * 10, 16)
    assert ao.segment_time(10, 8, 10 ** 9, 64) == Fraction(4 * 8 * 10, 64)


def test_cache_load_hand_cases():
    """Integer cases worked by hand.  One request, d = 1, prefix 20, input 5:
    M = 4 (20 + 5) = 100 bytes, F = 2 * 20 * 5 = 200 flop.  With N B T = 100 the memory share is
    100 / 200 = 1/2; with N F T = 600 the compute share is 200 / 800 = 1/4; L is the larger."""
    assert ao.cache_traffic_and_flops(1, [20], [5]) == (100, 200)
    assert ao.cache_load(1, [20], [5], n_gpus=2, mem_bw=10, flops=60, t_ideal=5) == Fraction(1, 2)
    # compute side larger: N F T = 200 -> 1/2 ; N B T = 900 -> 1/10
    assert ao.cache_load(1, [20], [5], n_gpus=1, mem_bw=90, flops=20, t_ideal=10) == Fraction(1, 2)
    # two requests add up: M = 4*3*(7+1) + 4*3*(2+2) = 96 + 48 = 144 ; F = 2*3*7 + 2*3*4 = 42 + 24 = 66
    assert ao.cache_traffic_and_flops(3, [7, 2], [1, 2]) == (144, 66)
    # limits: no time -> the cache takes everything; unbounded time -> nothing
    assert ao.cache_load(1, [20], [5], 1, 1, 1, 0) == 1
    assert float(ao.cache_load(1, [20], [5], 1, 1, 1, 10 ** 12)) < 1e-9
    # no prefix: no cache flops, only the new tokens' KV traffic
    assert ao.cache_traffic_and_flops(2, [0], [9]) == (72, 0)


# ---- the library's calculators against the oracle ------------------------------------------
def test_library_calculators_match_the_oracle():
    rng = np.random.default_rng(0)
    for _ in range(200):
        dq = int(rng.integers(1, 16384))
        dkv = dq if rng.random() < 0.5 else int(rng.integers(1, dq + 1))
        F, Bm = float(rng.uniform(1e12, 5e15)), float(rng.uniform(1e11, 1e13))
        a, Bn = float(rng.uniform(1e-7, 1e-4)), float(rng.uniform(1e9, 1e12))
        Ctok = float(rng.integers(1, 100000))
        t = B.tl_model_segment_time(Ctok, dq, dkv, F, Bm)
        want = max(Fraction(4 * dq) / Fraction(F), Fraction(4 * dkv) / Fraction(Bm)) * Fraction(Ctok)
        assert t == pytest.approx(float(want), rel=1e-12)
        if dq == dkv:
            assert t == pytest.approx(float(ao.segment_time(Fraction(Ctok), dq, Fraction(F), Fraction(Bm))), rel=1e-12)
            thr = B.tl_model_segment_threshold(dq, dkv, F, Bm, a, Bn)
            assert thr == pytest.approx(float(ao.segment_threshold(dq, Fraction(F), Fraction(Bm), Fraction(a), Fraction(Bn))), rel=1e-12)
        assert B.tl_model_comm_time(dq, a, Bn) == pytest.approx(float(ao.comm_time(dq, Fraction(a), Fraction(Bn))), rel=1e-12)
    for _ in range(50):
        n = int(rng.integers(1, 20))
        d = int(rng.integers(1, 8192))
        pl = rng.integers(0, 200000, size=n)
        il = rng.integers(1, 4096, size=n)
        N, Bm, F, T = int(rng.integers(1, 64)), float(rng.uniform(1e11, 1e13)), float(rng.uniform(1e12, 5e15)), float(rng.uniform(1e-4, 1.0))
        m, f, L = B.tl_model_cache_load(d, pl, il, N, Bm, F, T)
        wm, wf = ao.cache_traffic_and_flops(d, pl.tolist(), il.tolist())
        assert m == pytest.approx(float(wm), rel=1e-12) and f == pytest.approx(float(wf), rel=1e-12)
        assert L == pytest.approx(float(ao.cache_load(d, pl.tolist(), il.tolist(), N, Fraction(Bm), Fraction(F), Fraction(T))), rel=1e-12)


def test_library_calculators_reject_bad_arguments():
    for call in [lambda: B.tl_model_segment_time(10, 0, 1, 1e12, 1e12), lambda: B.tl_model_segment_time(10, 8, 8, 0, 1e12),
                 lambda: B.tl_model_comm_time(8, -1e-6, 1e9), lambda: B.tl_model_segment_threshold(8, 8, 1e12, 1e12, 1e-6, 0),
                 lambda: B.tl_model_cache_load(8, [1, 2], [1], 1, 1e12, 1e12, 1.0),
                 lambda: B.tl_model_cache_load(8, [1], [1], 0, 1e12, 1e12, 1.0),
                 lambda: B.tl_model_cache_load(8, [-1], [1], 1, 1e12, 1e12, 1.0)]:
        with pytest.raises((B.TokenLakeError, ValueError)):
            call()


def test_mi355x_parameters_give_a_threshold_well_below_the_segment_sizes_used():
    """The same formula with MI355X / xGMI figures (8 TB/s HBM, 2.5 PFLOP/s, one xGMI link
    ~153 GB/s, 2 us of latency) for a Llama-3-8B layer (Hq*dh = 4096, Hkv*dh = 1024): a decode
    token is memory-bound at 0.51 ns per prefix token, sixteen times less than on the paper's
    testbed, so with the same latency the segment size from which a remote partial attention
    pays off is about 8k tokens rather than 568."""
    t = B.tl_model_segment_threshold(4096, 1024, 2.5e15, 8e12, 2e-6, 153e9)
    k = max(4 * 4096 / 2.5e15, 4 * 1024 / 8e12)
    assert k == 4 * 1024 / 8e12
    assert t == pytest.approx((2 * 2e-6 + 4 * 4096 / 153e9) / k, rel=1e-12)
    assert 7500 < t < 8500
