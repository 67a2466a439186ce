"""Plain definitions of the paper's analytic models (TEST INFRASTRUCTURE ONLY, like the rest
of oracle/: nothing on the product path imports this file).

* Section 4.1 (segment size trade-off): time to attend to a segment of C tokens on one GPU,
  the round-trip communication time of a remote partial attention, and the segment size from
  which going remote pays off.
* Section 3.3 (last paragraph): bytes of KV cache produced per decoded token per layer.
* Section 5.1 (cache load isolation): memory traffic M_r and flops F_r of the cache-side work
  of a batch, and the fraction L of the GPUs' capacity they take during an iteration of
  ideal duration T_r.

Units: seconds, bytes, flop/s, bytes/s, tokens.  `d` is the hidden size the paper uses (its
model is multi-head, so one d serves for query and KV widths); 16-bit elements throughout, as
in the paper.  Pins: tests/test_analytic_models.py checks these functions against the three
figures the paper prints for its own testbed (16 KB per request per layer, a threshold of about
568 tokens, 4.66 us of communication at that size -- see tests/golden/paper_analytic_figures.txt)
and against hand-worked integer cases of the load formula.  The paper prints no worked example
of the load formula: get_cache_load is pinned by those hand cases and limits only.
"""
from __future__ import annotations

from fractions import Fraction


def kv_bytes_per_token(d):
    """K and V rows of one token of one layer at 16 bit: 2 tensors x d elements x 2 bytes."""
    return 4 * d


def segment_time_per_token(d, flops, mem_bw):
    """k_comp of Section 4.1: per prefix token, a query token costs 4d flop (2d for q.k, 2d
    for p.v) and the GPU reads 4d bytes of KV; the slower of the two rooflines decides."""
    return max(Fraction(4 * d) / Fraction(flops), Fraction(4 * d) / Fraction(mem_bw))


def segment_time(C, d, flops, mem_bw):
    """T_comp(C) = k_comp * C."""
    return segment_time_per_token(d, flops, mem_bw) * C


def comm_time(d, net_latency, net_bw):
    """T_comm = two messages' latency (query out, partial result back) plus 2d bytes each way
    (16-bit query row; 16-bit partial output row, the normalizer being negligible)."""
    return 2 * Fraction(net_latency) + Fraction(4 * d) / Fraction(net_bw)


def segment_threshold(d, flops, mem_bw, net_latency, net_bw):
    """Smallest segment size C (real-valued) with T_comp(C) >= T_comm."""
    return comm_time(d, net_latency, net_bw) / segment_time_per_token(d, flops, mem_bw)


def cache_traffic_and_flops(d, prefix_lens, input_lens):
    """M_r and F_r of Section 5.1 for a batch, as the paper prints them."""
    m = sum(4 * d * (p + i) for p, i in zip(prefix_lens, input_lens))
    f = sum(2 * d * p * i for p, i in zip(prefix_lens, input_lens))
    return m, f


def cache_load(d, prefix_lens, input_lens, n_gpus, mem_bw, flops, t_ideal):
    """L of Section 5.1: the larger of the memory-side and the compute-side share."""
    m, f = cache_traffic_and_flops(d, prefix_lens, input_lens)
    cap_m = Fraction(n_gpus) * Fraction(mem_bw) * Fraction(t_ideal)
    cap_f = Fraction(n_gpus) * Fraction(flops) * Fraction(t_ideal)
    share_m = Fraction(m) / (Fraction(m) + cap_m) if m + cap_m else Fraction(0)
    share_f = Fraction(f) / (Fraction(f) + cap_f) if f + cap_f else Fraction(0)
    return max(share_m, share_f)
