// Internal declarations shared by the host side of the library (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <unordered_map>
#include <vector>

#include "prefix_tree.h"
#include "tokenlake.h"

namespace tl {

void set_error(const char* fmt, ...) __attribute__((format(printf, 1, 2)));

#define TL_FAIL(code, ...)        \
  do {                            \
    ::tl::set_error(__VA_ARGS__); \
    return (code);                \
  } while (0)

#define TL_HIP(expr)                                                          \
  do {                                                                        \
    hipError_t e_ = (expr);                                                   \
    if (e_ != hipSuccess) {                                                   \
      ::tl::set_error("%s failed: %s", #expr, hipGetErrorString(e_));         \
      return TL_EHIP;                                                         \
    }                                                                         \
  } while (0)

constexpr int kHeadDim = 128;
constexpr int kKvTile = 64;      // kv tokens per LDS tile of the row-tile kernel
constexpr int kTreeNodesPerSlot = 16;   // the pool's prefix tree is cleared when it outgrows this many nodes per slot
constexpr int kMergeFixInts = 8;   // ints of a short merge list's fixed record: the token, then up to 7 partial rows
constexpr int kLongMergeList = 8;  // partials per token from which the merge deals the list to slices
constexpr int kRowTile = 256;    // query rows (token x head-in-group) per workgroup
constexpr int kUnitRows = 16;    // max rows per kv head of a split-K unit
// A request is planned for the one-pass kernel from this many query rows per kv head: it then
// does 512 flop per KV byte it reads by itself (4 * 128 flop per row and 512-byte K+V token),
// about twice the machine balance of the measured rooflines (1.2 PFLOP/s : 6 TB/s = 200), so
// that giving up the sharing of hot segments between requests cannot make it bandwidth-bound.
constexpr int kFuseRows = 2 * kRowTile;
constexpr int kComputeUnits = 256;   // MI355X (tl_plan_create's default; the plan builder makes no HIP call)

// One unit of kernel work.  Its query tokens are tok[tok_off .. tok_off+n_tok) (batch token
// indices), its partial rows out_row .. out_row+n_tok-1.
//  pool work:   split-K units: kv_off/kv_len index the plan's unit slot list (with unit_lm[]);
//               row tiles: the item's kv tokens are listed as tiles of 64: full_off/n_full index tile_base[]
//               (first kv row of each completely filled tile), part_off/n_part index
//               part_tile[] (first kv row, valid tokens) for the tiles cut short by a fill.
//  causal work: kv_off = first new token of the request, kv_len = new tokens visible to the
//               last row of the tile; tokens of the tile are consecutive.
//  one-pass rows: both of the above (tile lists of the request's pool part, new tokens as causal
//               work; out_row = the tile's first token) and prior_off/n_prior: entries of the plan's
//               prior_rows[], each the partial row that the request's FIRST new token has in a work
//               item above it (row of this tile's first token = entry + out_row - kv_off), which the
//               epilogue merges into the result.
struct Work {
  int32_t tok_off, n_tok, out_row, kv_off, kv_len, full_off, n_full, part_off, n_part, prior_off, n_prior;
};

int get_option_vread();

}  // namespace tl

struct tl_pool {
  int32_t n_slots, seg_len, kv_heads, head_dim;
  void* k_dev;
  void* v_dev;
  bool owns_kv;
  std::unordered_map<uint64_t, int32_t> slot_of;
  std::vector<uint64_t> id_of;
  std::vector<int32_t> fill;     // 0 = free
  std::vector<int32_t> refcnt;
  mutable std::vector<uint64_t> stamp;
  mutable uint64_t clock;
  int32_t n_used;
  int32_t free_hint;             // no free slot below this index
  uint64_t generation;           // goes up whenever a slot's content, fill or owner changes (put of a new id,
                                 // append, adopt, evict): a plan is valid for the generation it was built in
  mutable tl::PrefixTree tree;   // grows as plans walk their requests' lists; loses a segment's nodes on eviction
  // device mirror of fill[]
  mutable int32_t* fill_dev;
  mutable bool fill_dirty;
};

struct tl_plan {
  const tl_pool* pool;           // identity only after creation (never dereferenced: the pool may be gone)
  int32_t q_heads, kv_heads, group, n_req, n_tokens, flags;
  tl_plan_info info;
  std::vector<int32_t> item_row_base, item_tok_ptr, item_tokens, item_slot_ptr, item_slots;
  std::vector<int32_t> merge_ptr, merge_rows;
  std::vector<tl::Work> tiles, units, ctiles, ftiles;   // ftiles: fused rows (pool tiles + causal block in one pass)
  std::vector<int32_t> merge_fix;  // the short lists again, one fixed record of 8 ints per token: {token, rows..., -1 padding}
  std::vector<int32_t> merge_tok;  // tokens that tl_merge writes (all but the fused ones): n_merge_short with short
                                   // lists first, then those with kLongMergeList or more partials
  int32_t n_merge_short = 0;
  std::vector<int32_t> single_tok; // the new token of every request that has exactly one (not fused): self block = one key
  // the part of the pool's prefix tree that this batch walked, nodes in order of first visit (a node's
  // parent comes before it): what tl_plan_hot_slots searches, from the root side, without the pool
  std::vector<int32_t> bt_slot, bt_first_child, bt_next_sib, bt_roots;
  std::vector<int64_t> bt_load;
  std::vector<int32_t> tok;      // token index array referenced by Work::tok_off
  std::vector<int32_t> tile_base;  // Work::full_off
  std::vector<int32_t> part_tile;  // Work::part_off, pairs (first kv row, valid tokens)
  bool any_repeat = false;              // some work item's list names a slot more than once
  std::vector<float> tile_lm, part_lm;  // log2 of how often the tile's slot is listed (parallel to tile_base / part_tile pairs)
  std::vector<int32_t> prior_rows;      // Work::prior_off
  std::vector<int32_t> unit_slots;      // split-K units: Work::kv_off/kv_len, each distinct slot of a chunk once ...
  std::vector<float> unit_lm;           // ... with log2 of the number of times the run lists it
  bool any_unit_repeat = false;
  uint64_t pool_generation;      // the pool's generation when the plan was built
  int32_t pool_n_slots;
  // Everything the kernels read, laid out once at creation as one block of host memory (each array
  // starts on a 256-byte boundary); the device copy is made on first use, in one transfer.
  std::vector<char> blob_host;
  struct {
    size_t tiles, units, ctiles, ftiles, tok, slots, merge_ptr, merge_rows, tile_base, part_tile, merge_tok, single_tok,
        tile_lm, part_lm, prior_rows, unit_lm, merge_fix;
  } off;
  void* blob_dev;                // hipMalloc'd copy of blob_host, or null
};

namespace tl {

// Device addresses of a plan's arrays inside a copy of its block that starts at `base`.
struct PlanDev {
  const Work *tiles, *units, *ctiles, *ftiles;
  const int32_t *tok, *slots, *merge_ptr, *merge_rows, *tile_base, *part_tile, *merge_tok, *single_tok;
  const float *tile_lm, *part_lm;
  const int32_t* prior_rows;
  const float* unit_lm;
  const int32_t* merge_fix;
};
inline PlanDev plan_dev(const tl_plan* p, const void* base) {
  const char* b = (const char*)base;
  PlanDev d;
  d.tiles = (const Work*)(b + p->off.tiles);
  d.units = (const Work*)(b + p->off.units);
  d.ctiles = (const Work*)(b + p->off.ctiles);
  d.ftiles = (const Work*)(b + p->off.ftiles);
  d.tok = (const int32_t*)(b + p->off.tok);
  d.slots = (const int32_t*)(b + p->off.slots);
  d.merge_ptr = (const int32_t*)(b + p->off.merge_ptr);
  d.merge_rows = (const int32_t*)(b + p->off.merge_rows);
  d.tile_base = (const int32_t*)(b + p->off.tile_base);
  d.part_tile = (const int32_t*)(b + p->off.part_tile);
  d.merge_tok = (const int32_t*)(b + p->off.merge_tok);
  d.single_tok = (const int32_t*)(b + p->off.single_tok);
  d.tile_lm = (const float*)(b + p->off.tile_lm);
  d.part_lm = (const float*)(b + p->off.part_lm);
  d.prior_rows = (const int32_t*)(b + p->off.prior_rows);
  d.unit_lm = (const float*)(b + p->off.unit_lm);
  d.merge_fix = (const int32_t*)(b + p->off.merge_fix);
  return d;
}

tl_status pool_device_ready(const tl_pool* pool, hipStream_t stream);
// Makes the plan's device copy if there is none yet: one hipMalloc and one copy enqueued on `stream`.
tl_status plan_device_ready(tl_plan* plan, hipStream_t stream);
// TL_EINVAL if the pool has changed since the plan was built.
tl_status plan_is_current(const tl_plan* plan, const tl_pool* pool, const char* who);
}  // namespace tl
