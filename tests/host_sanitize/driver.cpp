// Host-only exercise of the C ABI for a build with AddressSanitizer and UndefinedBehaviorSanitizer
// on the host pass: pool bookkeeping, plan building over random batches (every flag combination,
// repeated segments, empty lists, zero-token requests), exports, heavy hitters, append validation
// and the analytic models.  No call here enqueues device work: the pool is given (fake) pointers
// that are never dereferenced, and plans make their device copies only on first use.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "tokenlake.h"

#define CHECK(cond)                                                                  \
  do {                                                                               \
    if (!(cond)) {                                                                   \
      std::fprintf(stderr, "driver: line %d: %s failed (%s)\n", __LINE__, #cond, tl_last_error()); \
      std::exit(1);                                                                  \
    }                                                                                \
  } while (0)

int main() {
  std::mt19937_64 rng(12345);
  auto pick = [&](int lo, int hi) { return (int)(lo + rng() % (uint64_t)(hi - lo + 1)); };
  void* fake_k = (void*)0x1000;
  void* fake_v = (void*)0x2000;
  int n_plans = 0;
  for (int round = 0; round < 40; ++round) {
    const int seg_len = 64 << pick(0, 2), kv_heads = 1 << pick(0, 3), n_slots = 64;
    const int group = (int[]){1, 3, 4, 7, 8}[pick(0, 4)];
    tl_pool* pool = nullptr;
    CHECK(tl_pool_create(&pool, n_slots, seg_len, kv_heads, 128, fake_k, fake_v) == TL_OK);
    const int n_ids = pick(4, 40);
    std::vector<uint64_t> ids(n_ids);
    std::vector<int32_t> slots(n_ids), fills(n_ids);
    std::vector<int32_t> perm(n_slots);
    for (int i = 0; i < n_slots; ++i) perm[i] = i;
    for (int i = n_slots - 1; i > 0; --i) std::swap(perm[i], perm[pick(0, i)]);
    for (int i = 0; i < n_ids; ++i) {
      ids[i] = 1000 + (uint64_t)i * 7;
      slots[i] = perm[i];
      fills[i] = pick(1, seg_len);
    }
    CHECK(tl_pool_adopt(pool, ids.data(), slots.data(), fills.data(), n_ids, nullptr) == TL_OK);
    CHECK(tl_pool_adopt(pool, ids.data(), slots.data(), fills.data(), 1, nullptr) == TL_EINVAL);   // already there
    std::vector<int32_t> looked(n_ids);
    CHECK(tl_pool_lookup(pool, ids.data(), n_ids, looked.data()) == TL_OK);
    for (int i = 0; i < n_ids; ++i) CHECK(looked[i] == slots[i]);
    uint64_t missing = 5;
    int32_t miss_slot = 0;
    CHECK(tl_pool_lookup(pool, &missing, 1, &miss_slot) == TL_OK && miss_slot == -1);

    // random batch: a common stem, then own entries (with repeats), some requests empty either way
    const int n_req = pick(1, 8);
    std::vector<int32_t> row_ptr(1, 0), seg_ptr(1, 0);
    std::vector<uint64_t> seg_ids;
    const int stem = pick(0, 3);
    const int tok_choices[] = {0, 1, 3, 16, 70, 200, 600};
    for (int r = 0; r < n_req; ++r) {
      if (pick(0, 6) != 0)
        for (int i = 0; i < stem && i < n_ids; ++i) seg_ids.push_back(ids[i]);
      const int own = pick(0, 6);
      for (int i = 0; i < own; ++i) seg_ids.push_back(ids[pick(0, n_ids - 1)]);
      seg_ptr.push_back((int32_t)seg_ids.size());
      row_ptr.push_back(row_ptr.back() + tok_choices[pick(0, 6)]);
    }
    const int flag_sets[] = {0, TL_PLAN_SELF_BLOCK, TL_PLAN_SELF_BLOCK | TL_PLAN_NO_SHARING,
                             TL_PLAN_SELF_BLOCK | TL_PLAN_FUSE_ROWS, TL_PLAN_SELF_BLOCK | TL_PLAN_FUSE_ROWS | TL_PLAN_NO_SHARING,
                             TL_PLAN_SELF_BLOCK | TL_PLAN_FUSE_TAILS, TL_PLAN_SELF_BLOCK | TL_PLAN_FUSE_TAILS | TL_PLAN_FUSE_ROWS};
    for (int flags : flag_sets)
      for (int cus : {0, 8, 256})
        for (int dedupe : {0, 1}) {
          tl_plan* plan = nullptr;
          CHECK(tl_plan_create(&plan, pool, kv_heads * group, n_req, row_ptr.data(), seg_ptr.data(),
                               seg_ids.empty() ? nullptr : seg_ids.data(), flags | (dedupe ? 0 : TL_PLAN_WALK_REPEATS),
                               pick(0, 3), cus) == TL_OK);
          tl_plan_info info;
          CHECK(tl_plan_get_info(plan, &info) == TL_OK);
          CHECK(info.n_tokens == row_ptr.back() && info.n_req == n_req);
          CHECK(info.tile_pairs <= info.prefix_pairs);
          int32_t n_item_tokens = 0, n_item_slots = 0;
          CHECK(tl_plan_export_sizes(plan, &n_item_tokens, &n_item_slots) == TL_OK);
          std::vector<int32_t> row_base(info.n_items + 1), tok_ptr(info.n_items + 1), toks(n_item_tokens + 1),
              slot_ptr(info.n_items + 1), islots(n_item_slots + 1), mptr(info.n_tokens + 1), mrows(info.n_merge_entries + 1);
          CHECK(tl_plan_export(plan, row_base.data(), tok_ptr.data(), toks.data(), slot_ptr.data(), islots.data(),
                               mptr.data(), mrows.data()) == TL_OK);
          CHECK(mptr[info.n_tokens] == info.n_merge_entries);
          std::vector<int32_t> hot(8);
          std::vector<int64_t> load(8);
          int32_t n_hot = 0;
          CHECK(tl_plan_hot_slots(plan, 8, hot.data(), load.data(), &n_hot) == TL_OK && n_hot <= 8);
          for (int i = 1; i < n_hot; ++i) CHECK(load[i - 1] >= load[i]);
          CHECK(tl_plan_destroy(plan) == TL_OK);
          ++n_plans;
        }
    tl_plan* bad = nullptr;
    uint64_t unknown = 3;
    int32_t one_row[2] = {0, 1}, one_seg[2] = {0, 1};
    CHECK(tl_plan_create(&bad, pool, kv_heads * group, 1, one_row, one_seg, &unknown, 0, 0, -1) == TL_ENOTFOUND && bad == nullptr);

    // append validation (refused before any device work), release, eviction
    uint64_t new_id = 999999;
    CHECK(tl_pool_append(pool, 1, 424242, nullptr, 0, fake_k, fake_v, 1, nullptr, nullptr) == TL_ENOTFOUND);
    CHECK(tl_pool_append(pool, 0, 0, &new_id, 1, fake_k, fake_v, 2 * seg_len, nullptr, nullptr) == TL_EINVAL);   // needs two ids
    CHECK(tl_pool_append(pool, 0, 0, &ids[0], 1, fake_k, fake_v, 1, nullptr, nullptr) == TL_EINVAL);             // id resident
    int32_t used = 0;
    CHECK(tl_pool_used(pool, &used) == TL_OK && used == n_ids);
    uint64_t evicted = 0;
    CHECK(tl_pool_evict_lru(pool, &evicted) == TL_ENOTFOUND);                 // everything is referenced
    for (int i = 0; i < n_ids; i += 2) CHECK(tl_pool_release(pool, ids[i]) == TL_OK);
    CHECK(tl_pool_release(pool, ids[0]) == TL_EINVAL);
    int n_evicted = 0;
    while (tl_pool_evict_lru(pool, &evicted) == TL_OK) ++n_evicted;
    CHECK(n_evicted == (n_ids + 1) / 2);
    CHECK(tl_pool_used(pool, &used) == TL_OK && used == n_ids - n_evicted);
    CHECK(tl_pool_destroy(pool) == TL_OK);
  }
  double t = 0, thr = 0, tr = 0, fl = 0, ld = 0;
  CHECK(tl_model_segment_time(568, 4096, 4096, 312e12, 2e12, &t) == TL_OK && t > 0);
  CHECK(tl_model_comm_time(4096, 2.3e-6, 400e9, &t) == TL_OK && t > 0);
  CHECK(tl_model_segment_threshold(4096, 4096, 312e12, 2e12, 2.3e-6, 400e9, &thr) == TL_OK && thr > 0);
  const int64_t pre[3] = {1000, 20000, 0}, inp[3] = {128, 1, 512};
  CHECK(tl_model_cache_load(4096, pre, inp, 3, 8, 2e12, 312e12, 0.05, &tr, &fl, &ld) == TL_OK && ld > 0 && ld < 1);
  CHECK(tl_model_cache_load(0, pre, inp, 3, 8, 2e12, 312e12, 0.05, &tr, &fl, &ld) == TL_EINVAL);
  std::printf("host sanitizer driver: %d plans built and checked, all statuses as expected\n", n_plans);
  return 0;
}
