// Analytic models of the paper (host arithmetic only; no device code):
//   Section 4.1  segment-size trade-off: T_comp(C) = max(4 C d / F, 4 C d / B_mem),
//                T_comm = 2 alpha + 4 d / B_net, and the segment size where the two meet;
//   Section 5.1  get_cache_load: M_r, F_r and the share L of the GPUs they take.
// The paper's model is multi-head, so it has one width d; with grouped-query attention the
// flops follow the query width (q_heads * head_dim) and the KV bytes the KV width
// (kv_heads * head_dim), hence the two arguments d_q and d_kv.
#include <cmath>

#include "tl_internal.h"

using namespace tl;

namespace {

bool positive(double x) { return std::isfinite(x) && x > 0.0; }

double per_token(double d_q, double d_kv, double flops, double mem_bw) {
  const double by_compute = 4.0 * d_q / flops, by_memory = 4.0 * d_kv / mem_bw;
  return by_compute > by_memory ? by_compute : by_memory;
}

}  // namespace

extern "C" {

tl_status tl_model_segment_time(double n_tokens, double d_q, double d_kv, double flops, double mem_bw, double* seconds_out) {
  if (!seconds_out) TL_FAIL(TL_EINVAL, "tl_model_segment_time: null out");
  if (!(n_tokens >= 0.0) || !positive(d_q) || !positive(d_kv) || !positive(flops) || !positive(mem_bw))
    TL_FAIL(TL_EINVAL, "tl_model_segment_time: sizes and rates must be positive");
  *seconds_out = per_token(d_q, d_kv, flops, mem_bw) * n_tokens;
  return TL_OK;
}

tl_status tl_model_comm_time(double d_q, double net_latency, double net_bw, double* seconds_out) {
  if (!seconds_out) TL_FAIL(TL_EINVAL, "tl_model_comm_time: null out");
  if (!positive(d_q) || !(net_latency >= 0.0) || !std::isfinite(net_latency) || !positive(net_bw))
    TL_FAIL(TL_EINVAL, "tl_model_comm_time: width and bandwidth must be positive, latency non-negative");
  *seconds_out = 2.0 * net_latency + 4.0 * d_q / net_bw;
  return TL_OK;
}

tl_status tl_model_segment_threshold(double d_q, double d_kv, double flops, double mem_bw, double net_latency,
                                     double net_bw, double* tokens_out) {
  if (!tokens_out) TL_FAIL(TL_EINVAL, "tl_model_segment_threshold: null out");
  double t_comm = 0.0;
  tl_status rc = tl_model_comm_time(d_q, net_latency, net_bw, &t_comm);
  if (rc != TL_OK) return rc;
  if (!positive(d_kv) || !positive(flops) || !positive(mem_bw))
    TL_FAIL(TL_EINVAL, "tl_model_segment_threshold: sizes and rates must be positive");
  *tokens_out = t_comm / per_token(d_q, d_kv, flops, mem_bw);
  return TL_OK;
}

tl_status tl_model_cache_load(double d, const int64_t* prefix_len, const int64_t* input_len, int32_t n, int32_t n_gpus,
                              double mem_bw, double flops, double t_ideal, double* traffic_out, double* flops_out,
                              double* load_out) {
  if (n < 0 || (n > 0 && (!prefix_len || !input_len))) TL_FAIL(TL_EINVAL, "tl_model_cache_load: bad request arrays");
  if (!positive(d) || n_gpus < 1 || !positive(mem_bw) || !positive(flops) || !(t_ideal >= 0.0) || !std::isfinite(t_ideal))
    TL_FAIL(TL_EINVAL, "tl_model_cache_load: width, GPU count and rates must be positive, time non-negative");
  // sums in long double: exact for any realistic batch (terms are integers below 2^63)
  long double m = 0.0L, f = 0.0L;
  for (int32_t i = 0; i < n; ++i) {
    if (prefix_len[i] < 0 || input_len[i] < 0) TL_FAIL(TL_EINVAL, "tl_model_cache_load: negative length in request %d", i);
    m += 4.0L * (long double)d * ((long double)prefix_len[i] + (long double)input_len[i]);
    f += 2.0L * (long double)d * (long double)prefix_len[i] * (long double)input_len[i];
  }
  const long double cap_m = (long double)n_gpus * (long double)mem_bw * (long double)t_ideal;
  const long double cap_f = (long double)n_gpus * (long double)flops * (long double)t_ideal;
  const long double share_m = m + cap_m > 0.0L ? m / (m + cap_m) : 0.0L;
  const long double share_f = f + cap_f > 0.0L ? f / (f + cap_f) : 0.0L;
  if (traffic_out) *traffic_out = (double)m;
  if (flops_out) *flops_out = (double)f;
  if (load_out) *load_out = (double)(share_m > share_f ? share_m : share_f);
  return TL_OK;
}

// Content-derived segment ids: one pass over the tokens, the hash state carried from segment to segment
// (FNV-1a is sequential, so the running value at a segment's end is the hash of everything before it).
tl_status tl_segment_ids(const int32_t* tokens, int64_t n_tokens, int32_t seg_len, uint64_t salt, uint64_t* ids_out) {
  if (seg_len <= 0 || n_tokens < 0) TL_FAIL(TL_EINVAL, "tl_segment_ids: seg_len must be positive, n_tokens non-negative");
  if (n_tokens > 0 && (!tokens || !ids_out)) TL_FAIL(TL_EINVAL, "tl_segment_ids: null argument");
  uint64_t h = 0xCBF29CE484222325ull ^ salt;
  for (int64_t i = 0; i < n_tokens; ++i) {
    const uint32_t t = (uint32_t)tokens[i];
    for (int b = 0; b < 4; ++b) h = (h ^ ((t >> (8 * b)) & 0xFFu)) * 0x100000001B3ull;
    if ((i + 1) % seg_len == 0 || i + 1 == n_tokens) ids_out[i / seg_len] = h;
  }
  return TL_OK;
}

}  // extern "C"
