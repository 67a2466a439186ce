// Segment pool: id -> slot table, per-slot fill / reference count / last-use stamp on the
// host; K/V slots and a mirror of fill[] on the device.  (Paper Section 3.1: fixed-size
// segments in cache slots; Section 1 and 4: one copy per segment; Section 4.3: eviction by
// last access time.)
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>

#include "tl_internal.h"

namespace tl {

static thread_local char g_err[512] = "";
static int g_opt_vread = 0;

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

int get_option_vread() { return g_opt_vread; }

// Slot numbers of one gather launch: they travel in the kernel arguments (no device buffer to
// allocate, fill and free).
constexpr int kGatherPerLaunch = 512;
struct GatherSlots {
  int32_t slot[kGatherPerLaunch];
};

// out[(first + i, :)] = pool[(slots.slot[i], :)], slot16 uint4 per slot; one block column per slot.
__global__ void gather_slots_kernel(uint4* __restrict__ out, const uint4* __restrict__ pool, const GatherSlots slots,
                                    int first, size_t slot16) {
  const int32_t s = slots.slot[blockIdx.y];
  const uint4* src = pool + (size_t)s * slot16;
  uint4* dst = out + (size_t)(first + blockIdx.y) * slot16;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < slot16; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}

// Destination chunks of one append launch: rows [src_row, src_row + n) of the source go to
// tokens [tok, tok + n) of `slot`; `zero_to` > tok + n asks for tokens [tok + n, zero_to) to be
// cleared; new_fill is stored in fill[slot].
struct AppendChunk {
  int32_t slot, tok, n, src_row, zero_to, new_fill;
};
constexpr int kAppendChunks = 128;   // 3 KB of kernel arguments
struct AppendArgs {
  AppendChunk c[kAppendChunks];
};

// blockIdx.y = chunk; the blocks of a column stride over the chunk's 16-byte pieces.
__global__ void append_rows_kernel(uint4* __restrict__ pool_k, uint4* __restrict__ pool_v,
                                   const uint4* __restrict__ src_k, const uint4* __restrict__ src_v,
                                   int32_t* __restrict__ fill, const AppendArgs args, size_t row16, size_t slot16) {
  const AppendChunk c = args.c[blockIdx.y];
  const size_t dst0 = (size_t)c.slot * slot16 + (size_t)c.tok * row16;
  const size_t src0 = (size_t)c.src_row * row16;
  const size_t n16 = (size_t)c.n * row16;
  const size_t z16 = c.zero_to > c.tok + c.n ? (size_t)(c.zero_to - c.tok - c.n) * row16 : 0;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) {
    pool_k[dst0 + i] = src_k[src0 + i];
    pool_v[dst0 + i] = src_v[src0 + i];
  }
  const uint4 z = make_uint4(0, 0, 0, 0);
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < z16; i += stride) {
    pool_k[dst0 + n16 + i] = z;
    pool_v[dst0 + n16 + i] = z;
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) fill[c.slot] = c.new_fill;
}

tl_status pool_device_ready(const tl_pool* pool, hipStream_t stream) {
  if (!pool->fill_dev) {
    int32_t* p = nullptr;
    TL_HIP(hipMalloc((void**)&p, sizeof(int32_t) * (size_t)pool->n_slots));
    pool->fill_dev = p;
    pool->fill_dirty = true;
  }
  if (pool->fill_dirty) {
    TL_HIP(hipMemcpyAsync(pool->fill_dev, pool->fill.data(), sizeof(int32_t) * (size_t)pool->n_slots,
                          hipMemcpyHostToDevice, stream));
    pool->fill_dirty = false;
  }
  return TL_OK;
}

}  // namespace tl

using namespace tl;

extern "C" {

const char* tl_status_str(tl_status s) {
  switch (s) {
    case TL_OK: return "ok";
    case TL_EINVAL: return "invalid argument";
    case TL_ENOMEM: return "out of memory";
    case TL_EFULL: return "pool full";
    case TL_ENOTFOUND: return "segment not found";
    case TL_EHIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

const char* tl_last_error(void) { return g_err; }

tl_status tl_set_option(const char* knob, int32_t value) {
  if (!knob) TL_FAIL(TL_EINVAL, "tl_set_option: null knob");
  if (!strcmp(knob, "vread")) {
    if (value < 0 || value > 1) TL_FAIL(TL_EINVAL, "tl_set_option: vread must be 0 or 1");
    g_opt_vread = value;
    return TL_OK;
  }
  TL_FAIL(TL_EINVAL, "tl_set_option: unknown knob '%s'", knob);
}

tl_status tl_pool_create(tl_pool** out, int32_t n_slots, int32_t seg_len, int32_t kv_heads, int32_t head_dim,
                         void* k_dev, void* v_dev) {
  if (!out) TL_FAIL(TL_EINVAL, "tl_pool_create: null out");
  *out = nullptr;
  if (n_slots <= 0 || seg_len <= 0 || kv_heads <= 0) TL_FAIL(TL_EINVAL, "tl_pool_create: non-positive size");
  if (head_dim != kHeadDim) TL_FAIL(TL_EINVAL, "tl_pool_create: head_dim must be %d", kHeadDim);
  if (seg_len % kKvTile) TL_FAIL(TL_EINVAL, "tl_pool_create: seg_len must be a multiple of %d", kKvTile);
  if ((int64_t)n_slots * seg_len > (int64_t)INT32_MAX)
    TL_FAIL(TL_EINVAL, "tl_pool_create: n_slots * seg_len exceeds 2^31-1 tokens");
  if ((k_dev == nullptr) != (v_dev == nullptr)) TL_FAIL(TL_EINVAL, "tl_pool_create: give both k_dev and v_dev or neither");
  tl_pool* p = new (std::nothrow) tl_pool();
  if (!p) TL_FAIL(TL_ENOMEM, "tl_pool_create: host allocation failed");
  p->n_slots = n_slots;
  p->seg_len = seg_len;
  p->kv_heads = kv_heads;
  p->head_dim = head_dim;
  p->k_dev = k_dev;
  p->v_dev = v_dev;
  p->owns_kv = false;
  p->clock = 0;
  p->n_used = 0;
  p->free_hint = 0;
  p->generation = 0;
  p->fill_dev = nullptr;
  p->fill_dirty = true;
  try {
    p->id_of.assign(n_slots, 0);
    p->fill.assign(n_slots, 0);
    p->refcnt.assign(n_slots, 0);
    p->stamp.assign(n_slots, 0);
    p->tree.reset(n_slots);
  } catch (...) {
    delete p;
    TL_FAIL(TL_ENOMEM, "tl_pool_create: host allocation failed");
  }
  if (!k_dev) {
    size_t bytes = (size_t)n_slots * seg_len * kv_heads * head_dim * 2;
    hipError_t e = hipMalloc(&p->k_dev, bytes);
    if (e == hipSuccess) e = hipMalloc(&p->v_dev, bytes);
    if (e != hipSuccess) {
      if (p->k_dev) (void)hipFree(p->k_dev);
      delete p;
      set_error("tl_pool_create: hipMalloc of %zu bytes x2 failed: %s", bytes, hipGetErrorString(e));
      return e == hipErrorOutOfMemory ? TL_ENOMEM : TL_EHIP;
    }
    p->owns_kv = true;
  }
  *out = p;
  return TL_OK;
}

tl_status tl_pool_destroy(tl_pool* pool) {
  if (!pool) return TL_OK;
  if (pool->fill_dev) (void)hipFree(pool->fill_dev);
  if (pool->owns_kv) {
    (void)hipFree(pool->k_dev);
    (void)hipFree(pool->v_dev);
  }
  delete pool;
  return TL_OK;
}

static int32_t take_slot(tl_pool* p, int32_t want) {
  if (want >= 0) return want;
  int32_t s = p->free_hint;
  while (s < p->n_slots && p->fill[s] != 0) ++s;
  p->free_hint = s;
  return s < p->n_slots ? s : -1;
}

static void occupy(tl_pool* p, int32_t slot, uint64_t id, int32_t fill) {
  p->slot_of.emplace(id, slot);
  p->id_of[slot] = id;
  p->fill[slot] = fill;
  p->refcnt[slot] = 1;
  p->stamp[slot] = ++p->clock;
  p->n_used++;
  p->generation++;
}

tl_status tl_pool_put(tl_pool* pool, uint64_t segment_id, const void* k_src_dev, const void* v_src_dev, int32_t fill,
                      int32_t want_slot, int32_t* slot_out, void* stream) {
  if (!pool) TL_FAIL(TL_EINVAL, "tl_pool_put: null pool");
  auto it = pool->slot_of.find(segment_id);
  if (it != pool->slot_of.end()) {
    int32_t s = it->second;
    pool->refcnt[s]++;
    pool->stamp[s] = ++pool->clock;
    if (slot_out) *slot_out = s;
    return TL_OK;
  }
  if (!k_src_dev || !v_src_dev) TL_FAIL(TL_EINVAL, "tl_pool_put: null source");
  if (fill < 1 || fill > pool->seg_len) TL_FAIL(TL_EINVAL, "tl_pool_put: fill %d outside 1..%d", fill, pool->seg_len);
  if (want_slot >= pool->n_slots || want_slot < -1) TL_FAIL(TL_EINVAL, "tl_pool_put: slot %d out of range", want_slot);
  if (want_slot >= 0 && pool->fill[want_slot] != 0) TL_FAIL(TL_EINVAL, "tl_pool_put: slot %d is taken", want_slot);
  int32_t s = take_slot(pool, want_slot);
  if (s < 0) TL_FAIL(TL_EFULL, "tl_pool_put: no free slot (%d in use)", pool->n_used);
  hipStream_t st = (hipStream_t)stream;
  tl_status rc = pool_device_ready(pool, st);
  if (rc != TL_OK) return rc;
  // one launch: copy the fill rows, clear the rest of the slot, store the slot's fill
  const size_t row16 = (size_t)pool->kv_heads * pool->head_dim * 2 / 16;
  const size_t slot16 = row16 * pool->seg_len;
  AppendArgs args;
  memset(&args, 0, sizeof(args));
  args.c[0] = AppendChunk{s, 0, fill, 0, pool->seg_len, fill};
  const unsigned bx = (unsigned)(slot16 / 256 > 32 ? 32 : (slot16 + 255) / 256);
  hipLaunchKernelGGL(append_rows_kernel, dim3(bx, 1), dim3(256), 0, st, (uint4*)pool->k_dev, (uint4*)pool->v_dev,
                     (const uint4*)k_src_dev, (const uint4*)v_src_dev, pool->fill_dev, args, row16, slot16);
  TL_HIP(hipGetLastError());
  occupy(pool, s, segment_id, fill);
  if (slot_out) *slot_out = s;
  return TL_OK;
}

tl_status tl_pool_append_batch(tl_pool* pool, int32_t n_chains, const int32_t* has_tail, const uint64_t* tail_ids,
                               const int32_t* new_ptr, const uint64_t* new_ids, const int32_t* row_ptr,
                               const void* k_rows_dev, const void* v_rows_dev, int32_t* new_slots_out, void* stream) {
  if (!pool || n_chains < 0) TL_FAIL(TL_EINVAL, "tl_pool_append: bad argument");
  if (n_chains == 0) return TL_OK;
  if (!has_tail || !new_ptr || !row_ptr) TL_FAIL(TL_EINVAL, "tl_pool_append: null chain arrays");
  if (new_ptr[0] != 0 || row_ptr[0] != 0) TL_FAIL(TL_EINVAL, "tl_pool_append: offsets must start at 0");
  for (int32_t c = 0; c < n_chains; ++c) {
    if (new_ptr[c + 1] < new_ptr[c] || row_ptr[c + 1] < row_ptr[c]) TL_FAIL(TL_EINVAL, "tl_pool_append: offsets must not decrease");
    if (has_tail[c] && !tail_ids) TL_FAIL(TL_EINVAL, "tl_pool_append: null tail ids");
  }
  const int32_t n_new_all = new_ptr[n_chains], n_rows_all = row_ptr[n_chains];
  if (n_new_all > 0 && !new_ids) TL_FAIL(TL_EINVAL, "tl_pool_append: null new ids");
  if (n_rows_all > 0 && (!k_rows_dev || !v_rows_dev)) TL_FAIL(TL_EINVAL, "tl_pool_append: null source");
  const int32_t C = pool->seg_len;
  // ---- validate every chain first ----
  std::vector<int32_t> tail_slot(n_chains, -1), room(n_chains, 0);
  {
    std::unordered_map<int32_t, int> tails;
    for (int32_t c = 0; c < n_chains; ++c) {
      const int32_t n_rows = row_ptr[c + 1] - row_ptr[c], n_new = new_ptr[c + 1] - new_ptr[c];
      if (has_tail[c]) {
        auto it = pool->slot_of.find(tail_ids[c]);
        if (it == pool->slot_of.end())
          TL_FAIL(TL_ENOTFOUND, "tl_pool_append: tail id %llu not resident", (unsigned long long)tail_ids[c]);
        tail_slot[c] = it->second;
        if (pool->refcnt[tail_slot[c]] != 1)
          TL_FAIL(TL_EINVAL, "tl_pool_append: tail id %llu has %d references, a shared segment does not grow",
                  (unsigned long long)tail_ids[c], pool->refcnt[tail_slot[c]]);
        if (n_rows > 0 && !tails.emplace(tail_slot[c], c).second)
          TL_FAIL(TL_EINVAL, "tl_pool_append: tail id %llu is the tail of two chains", (unsigned long long)tail_ids[c]);
        room[c] = C - pool->fill[tail_slot[c]];
      }
      const int32_t rest = n_rows > room[c] ? n_rows - room[c] : 0;
      const int32_t need = (rest + C - 1) / C;
      if (n_new != need)
        TL_FAIL(TL_EINVAL, "tl_pool_append: %d rows need exactly %d new segments, %d given", n_rows, need, n_new);
    }
    std::unordered_map<uint64_t, int> seen;
    for (int32_t i = 0; i < n_new_all; ++i) {
      if (pool->slot_of.count(new_ids[i])) TL_FAIL(TL_EINVAL, "tl_pool_append: id %llu already resident", (unsigned long long)new_ids[i]);
      if (!seen.emplace(new_ids[i], i).second) TL_FAIL(TL_EINVAL, "tl_pool_append: id %llu listed twice", (unsigned long long)new_ids[i]);
    }
  }
  if (pool->n_slots - pool->n_used < n_new_all)
    TL_FAIL(TL_EFULL, "tl_pool_append: %d free slots, %d needed", pool->n_slots - pool->n_used, n_new_all);
  if (n_rows_all == 0) return TL_OK;
  hipStream_t st = (hipStream_t)stream;
  tl_status rc = pool_device_ready(pool, st);
  if (rc != TL_OK) return rc;

  // ---- place the rows (host state changes from here on; no failure path below but HIP's) ----
  std::vector<AppendChunk> chunks;
  for (int32_t c = 0; c < n_chains; ++c) {
    const int32_t n_rows = row_ptr[c + 1] - row_ptr[c];
    int32_t row = 0;
    if (has_tail[c] && room[c] > 0 && n_rows > 0) {
      const int32_t ts = tail_slot[c];
      const int32_t n = n_rows < room[c] ? n_rows : room[c];
      chunks.push_back(AppendChunk{ts, pool->fill[ts], n, row_ptr[c], 0, pool->fill[ts] + n});
      pool->fill[ts] += n;
      pool->stamp[ts] = ++pool->clock;
      pool->generation++;
      row = n;
    }
    for (int32_t i = new_ptr[c]; i < new_ptr[c + 1]; ++i) {
      const int32_t n = n_rows - row < C ? n_rows - row : C;
      const int32_t s = take_slot(pool, -1);
      occupy(pool, s, new_ids[i], n);
      chunks.push_back(AppendChunk{s, 0, n, row_ptr[c] + row, C, n});
      if (new_slots_out) new_slots_out[i] = s;
      row += n;
    }
  }
  const size_t row16 = (size_t)pool->kv_heads * pool->head_dim * 2 / 16;
  const size_t slot16 = row16 * C;
  for (size_t c0 = 0; c0 < chunks.size(); c0 += kAppendChunks) {
    const size_t nc = chunks.size() - c0 < (size_t)kAppendChunks ? chunks.size() - c0 : (size_t)kAppendChunks;
    AppendArgs args;
    memset(&args, 0, sizeof(args));
    size_t most16 = 1;     // the largest chunk of the launch (copied plus cleared 16-byte pieces) sizes the block columns
    for (size_t i = 0; i < nc; ++i) {
      const AppendChunk& ch = chunks[c0 + i];
      args.c[i] = ch;
      const size_t rows = (size_t)(ch.zero_to > ch.tok + ch.n ? ch.zero_to - ch.tok : ch.n);
      if (rows * row16 > most16) most16 = rows * row16;
    }
    const unsigned bx = (unsigned)(most16 / 256 > 32 ? 32 : (most16 + 255) / 256);
    hipLaunchKernelGGL(append_rows_kernel, dim3(bx, (unsigned)nc), dim3(256), 0, st, (uint4*)pool->k_dev, (uint4*)pool->v_dev,
                       (const uint4*)k_rows_dev, (const uint4*)v_rows_dev, pool->fill_dev, args, row16, slot16);
  }
  TL_HIP(hipGetLastError());
  return TL_OK;
}

tl_status tl_pool_append(tl_pool* pool, int32_t has_tail, uint64_t tail_id, const uint64_t* new_ids, int32_t n_new,
                         const void* k_rows_dev, const void* v_rows_dev, int32_t n_rows, int32_t* new_slots_out,
                         void* stream) {
  if (!pool || n_rows < 0 || n_new < 0 || (n_new > 0 && !new_ids)) TL_FAIL(TL_EINVAL, "tl_pool_append: bad argument");
  const int32_t tail_flag = has_tail ? 1 : 0;
  const int32_t new_ptr[2] = {0, n_new}, row_ptr[2] = {0, n_rows};
  return tl_pool_append_batch(pool, 1, &tail_flag, &tail_id, new_ptr, new_ids, row_ptr, k_rows_dev, v_rows_dev,
                              new_slots_out, stream);
}

tl_status tl_pool_adopt(tl_pool* pool, const uint64_t* ids, const int32_t* slots, const int32_t* fills, int32_t n,
                        void* stream) {
  (void)stream;
  if (!pool || n < 0 || (n > 0 && (!ids || !slots || !fills))) TL_FAIL(TL_EINVAL, "tl_pool_adopt: bad argument");
  // validate everything first so that a failure registers nothing
  std::unordered_map<uint64_t, int> seen_id;
  std::unordered_map<int32_t, int> seen_slot;
  for (int32_t i = 0; i < n; ++i) {
    if (slots[i] < 0 || slots[i] >= pool->n_slots) TL_FAIL(TL_EINVAL, "tl_pool_adopt: slot %d out of range", slots[i]);
    if (fills[i] < 1 || fills[i] > pool->seg_len) TL_FAIL(TL_EINVAL, "tl_pool_adopt: fill %d outside 1..%d", fills[i], pool->seg_len);
    if (pool->fill[slots[i]] != 0) TL_FAIL(TL_EINVAL, "tl_pool_adopt: slot %d is taken", slots[i]);
    if (pool->slot_of.count(ids[i])) TL_FAIL(TL_EINVAL, "tl_pool_adopt: id %llu already resident", (unsigned long long)ids[i]);
    if (!seen_id.emplace(ids[i], i).second) TL_FAIL(TL_EINVAL, "tl_pool_adopt: id %llu listed twice", (unsigned long long)ids[i]);
    if (!seen_slot.emplace(slots[i], i).second) TL_FAIL(TL_EINVAL, "tl_pool_adopt: slot %d listed twice", slots[i]);
  }
  for (int32_t i = 0; i < n; ++i) occupy(pool, slots[i], ids[i], fills[i]);
  pool->fill_dirty = true;
  return TL_OK;
}

tl_status tl_pool_release(tl_pool* pool, uint64_t segment_id) {
  if (!pool) TL_FAIL(TL_EINVAL, "tl_pool_release: null pool");
  auto it = pool->slot_of.find(segment_id);
  if (it == pool->slot_of.end()) TL_FAIL(TL_ENOTFOUND, "tl_pool_release: id %llu not resident", (unsigned long long)segment_id);
  if (pool->refcnt[it->second] <= 0) TL_FAIL(TL_EINVAL, "tl_pool_release: id %llu has no references", (unsigned long long)segment_id);
  pool->refcnt[it->second]--;
  return TL_OK;
}

tl_status tl_pool_evict_lru(tl_pool* pool, uint64_t* evicted_id) {
  if (!pool) TL_FAIL(TL_EINVAL, "tl_pool_evict_lru: null pool");
  int32_t best = -1;
  for (int32_t s = 0; s < pool->n_slots; ++s)
    if (pool->fill[s] != 0 && pool->refcnt[s] == 0 && (best < 0 || pool->stamp[s] < pool->stamp[best])) best = s;
  if (best < 0) TL_FAIL(TL_ENOTFOUND, "tl_pool_evict_lru: no segment with zero references");
  if (evicted_id) *evicted_id = pool->id_of[best];
  pool->slot_of.erase(pool->id_of[best]);
  pool->tree.remove_slot(best);          // a prefix that has lost a segment is no prefix: its nodes go, with what hangs below
  pool->fill[best] = 0;
  pool->n_used--;
  pool->generation++;
  if (best < pool->free_hint) pool->free_hint = best;
  pool->fill_dirty = true;
  return TL_OK;
}

tl_status tl_pool_hot_segments(const tl_pool* pool, int32_t max_n, uint64_t* ids_out, int64_t* loads_out, int32_t* depths_out,
                               int32_t* n_out) {
  if (!pool || max_n < 0 || !n_out || (max_n > 0 && !ids_out)) TL_FAIL(TL_EINVAL, "tl_pool_hot_segments: bad argument");
  try {
    std::vector<int32_t> nodes;
    pool->tree.hottest(max_n, nodes);
    for (size_t i = 0; i < nodes.size(); ++i) {
      const TreeNode& x = pool->tree.at(nodes[i]);
      ids_out[i] = x.id;
      if (loads_out) loads_out[i] = x.load;
      if (depths_out) depths_out[i] = x.depth;
    }
    *n_out = (int32_t)nodes.size();
  } catch (const std::bad_alloc&) {
    TL_FAIL(TL_ENOMEM, "tl_pool_hot_segments: host allocation failed");
  }
  return TL_OK;
}

tl_status tl_pool_prefix_tree(const tl_pool* pool, int32_t max_nodes, uint64_t* ids_out, int32_t* parents_out, int64_t* loads_out,
                              int32_t* n_out, int32_t* n_total_out) {
  if (!pool || max_nodes < 0 || !n_out || (max_nodes > 0 && (!ids_out || !parents_out)))
    TL_FAIL(TL_EINVAL, "tl_pool_prefix_tree: bad argument");
  try {
    std::vector<int32_t> nodes;
    pool->tree.level_order(max_nodes, nodes);
    std::unordered_map<int32_t, int32_t> pos;       // node -> position in the output
    for (size_t i = 0; i < nodes.size(); ++i) {
      const TreeNode& x = pool->tree.at(nodes[i]);
      pos.emplace(nodes[i], (int32_t)i);
      ids_out[i] = x.id;
      parents_out[i] = x.parent == 0 ? -1 : pos.at(x.parent);      // a parent always comes earlier in level order
      if (loads_out) loads_out[i] = x.load;
    }
    *n_out = (int32_t)nodes.size();
    if (n_total_out) *n_total_out = pool->tree.size();
  } catch (const std::bad_alloc&) {
    TL_FAIL(TL_ENOMEM, "tl_pool_prefix_tree: host allocation failed");
  }
  return TL_OK;
}

tl_status tl_pool_lookup(const tl_pool* pool, const uint64_t* ids, int32_t n, int32_t* slots_out) {
  if (!pool || n < 0 || (n > 0 && (!ids || !slots_out))) TL_FAIL(TL_EINVAL, "tl_pool_lookup: bad argument");
  for (int32_t i = 0; i < n; ++i) {
    auto it = pool->slot_of.find(ids[i]);
    slots_out[i] = it == pool->slot_of.end() ? -1 : it->second;
  }
  return TL_OK;
}

tl_status tl_pool_fills(const tl_pool* pool, const int32_t* slots, int32_t n, int32_t* fills_out) {
  if (!pool || n < 0 || (n > 0 && (!slots || !fills_out))) TL_FAIL(TL_EINVAL, "tl_pool_fills: bad argument");
  for (int32_t i = 0; i < n; ++i) {
    if (slots[i] < 0 || slots[i] >= pool->n_slots) TL_FAIL(TL_EINVAL, "tl_pool_fills: slot %d out of range", slots[i]);
    fills_out[i] = pool->fill[slots[i]];
  }
  return TL_OK;
}

tl_status tl_pool_used(const tl_pool* pool, int32_t* n_used) {
  if (!pool || !n_used) TL_FAIL(TL_EINVAL, "tl_pool_used: bad argument");
  *n_used = pool->n_used;
  return TL_OK;
}

tl_status tl_pool_gather(tl_pool* pool, const int32_t* slots, int32_t n, void* k_out_dev, void* v_out_dev, void* stream) {
  if (!pool || n < 0 || (n > 0 && (!slots || !k_out_dev || !v_out_dev))) TL_FAIL(TL_EINVAL, "tl_pool_gather: bad argument");
  if (n == 0) return TL_OK;
  for (int32_t i = 0; i < n; ++i)
    if (slots[i] < 0 || slots[i] >= pool->n_slots) TL_FAIL(TL_EINVAL, "tl_pool_gather: slot %d out of range", slots[i]);
  hipStream_t st = (hipStream_t)stream;
  const size_t slot16 = (size_t)pool->seg_len * pool->kv_heads * pool->head_dim * 2 / 16;
  for (int32_t first = 0; first < n; first += kGatherPerLaunch) {
    const int32_t m = n - first < kGatherPerLaunch ? n - first : kGatherPerLaunch;
    GatherSlots gs;
    for (int32_t i = 0; i < kGatherPerLaunch; ++i) gs.slot[i] = i < m ? slots[first + i] : 0;
    const dim3 grid((unsigned)(slot16 / 256 > 64 ? 64 : (slot16 + 255) / 256), (unsigned)m);
    hipLaunchKernelGGL(gather_slots_kernel, grid, dim3(256), 0, st, (uint4*)k_out_dev, (const uint4*)pool->k_dev, gs, first, slot16);
    hipLaunchKernelGGL(gather_slots_kernel, grid, dim3(256), 0, st, (uint4*)v_out_dev, (const uint4*)pool->v_dev, gs, first, slot16);
  }
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) TL_FAIL(TL_EHIP, "tl_pool_gather: %s", hipGetErrorString(e));
  return TL_OK;
}

}  // extern "C"
