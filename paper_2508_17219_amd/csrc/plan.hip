// Host-side plan builder (paper Section 3.2: plans are generated per batch before the data
// plane runs; Section 4.3: segments near the root of the prefix tree are hot, so requests
// that share a run of segments are batched against it).
//
// Every request's list is walked down the pool's prefix tree (nodes are made as needed and stay
// for later batches; each node on the way takes the request's new tokens as load).  A maximal
// chain of tree nodes that the same set of requests passes through becomes one work item whose
// query rows are all new tokens of those requests.  Items with few rows per kv head are cut into
// split-K chunks.
#include <algorithm>
#include <cstring>
#include <new>
#include <queue>
#include <unordered_set>

#include "tl_internal.h"

using namespace tl;

namespace {

struct RawItem {
  std::vector<int32_t> reqs;   // ascending
  int32_t src_req;             // request whose list supplies the run
  int32_t begin, end;          // list positions [begin, end)
};


}  // namespace

extern "C" {

tl_status tl_plan_create(tl_plan** out, const tl_pool* pool, int32_t q_heads, int32_t n_req,
                         const int32_t* req_row_ptr, const int32_t* req_seg_ptr, const uint64_t* seg_ids,
                         int32_t flags, int32_t split_segments, int32_t compute_units) {
  if (!out) TL_FAIL(TL_EINVAL, "tl_plan_create: null out");
  *out = nullptr;
  if (!pool || n_req < 0 || !req_row_ptr || !req_seg_ptr) TL_FAIL(TL_EINVAL, "tl_plan_create: bad argument");
  if (q_heads <= 0 || q_heads % pool->kv_heads) TL_FAIL(TL_EINVAL, "tl_plan_create: q_heads must be a multiple of kv_heads");
  const int G = q_heads / pool->kv_heads;
  if (G > 32) TL_FAIL(TL_EINVAL, "tl_plan_create: q_heads/kv_heads must be at most 32");
  if (split_segments < 0) TL_FAIL(TL_EINVAL, "tl_plan_create: negative split_segments");
  if (compute_units > 4096) TL_FAIL(TL_EINVAL, "tl_plan_create: compute_units above 4096");
  if ((flags & (TL_PLAN_FUSE_ROWS | TL_PLAN_FUSE_TAILS)) && !(flags & TL_PLAN_SELF_BLOCK))
    TL_FAIL(TL_EINVAL, "tl_plan_create: TL_PLAN_FUSE_ROWS and TL_PLAN_FUSE_TAILS need TL_PLAN_SELF_BLOCK");
  if ((flags & TL_PLAN_FUSE_TAILS) && (flags & TL_PLAN_NO_SHARING))
    TL_FAIL(TL_EINVAL, "tl_plan_create: TL_PLAN_FUSE_TAILS has nothing to do under TL_PLAN_NO_SHARING");
  if (req_row_ptr[0] != 0 || req_seg_ptr[0] != 0) TL_FAIL(TL_EINVAL, "tl_plan_create: offsets must start at 0");
  for (int32_t r = 0; r < n_req; ++r)
    if (req_row_ptr[r + 1] < req_row_ptr[r] || req_seg_ptr[r + 1] < req_seg_ptr[r])
      TL_FAIL(TL_EINVAL, "tl_plan_create: offsets of request %d decrease", r);
  const int32_t T = req_row_ptr[n_req];
  const int32_t n_entries = req_seg_ptr[n_req];
  if (n_entries > 0 && !seg_ids) TL_FAIL(TL_EINVAL, "tl_plan_create: null seg_ids");

  tl_plan* p = new (std::nothrow) tl_plan();
  if (!p) TL_FAIL(TL_ENOMEM, "tl_plan_create: host allocation failed");
  tl_status rc = TL_OK;
  try {
    p->pool = pool;
    p->q_heads = q_heads;
    p->kv_heads = pool->kv_heads;
    p->group = G;
    p->n_req = n_req;
    p->n_tokens = T;
    p->flags = flags;
    p->blob_dev = nullptr;
    p->pool_generation = pool->generation;
    p->pool_n_slots = pool->n_slots;

    // ---- a0: segment id -> slot ------------------------------------------------------
    std::vector<int32_t> slots(n_entries);
    for (int32_t i = 0; i < n_entries; ++i) {
      auto it = pool->slot_of.find(seg_ids[i]);
      if (it == pool->slot_of.end()) {
        set_error("tl_plan_create: segment id %llu (list entry %d) is not resident", (unsigned long long)seg_ids[i], i);
        delete p;
        return TL_ENOTFOUND;
      }
      slots[i] = it->second;
    }
    const uint64_t now = ++pool->clock;
    for (int32_t s : slots) pool->stamp[s] = now;

    auto len_of = [&](int32_t r) { return req_seg_ptr[r + 1] - req_seg_ptr[r]; };
    auto slot_at = [&](int32_t r, int32_t pos) { return slots[req_seg_ptr[r] + pos]; };
    auto ntok_of = [&](int32_t r) { return req_row_ptr[r + 1] - req_row_ptr[r]; };

    // ---- group requests along shared runs ----------------------------------------------
    // With TL_PLAN_FUSE_ROWS a request is set aside for the one-pass kernel if sharing a run of slots
    // with other requests gains it nothing: it has no slot in common with another request of the
    // batch, or it has enough rows of its own (the work is then bound by the matrix unit, not by KV
    // traffic) -- either way it would only lose a partial per row, and a merge, on the other path.
    // Requests with a token's worth of rows (decode) always take split-K units.
    const int tok_tile = kRowTile / G;
    const int64_t n_cu = compute_units < 0 ? kComputeUnits : compute_units;
    const int32_t min_chunk_slots = std::max(1, 2048 / pool->seg_len);
    std::vector<char> fused(n_req, 0);
    // A one-pass row tile cannot be cut along its KV: when the whole batch is fewer row-tile
    // workgroups than the GPU has CUs (one long prompt, say), requests whose slot lists are long
    // enough to be cut (see below) stay on the three-step path
    bool small_batch = false;
    {
      int64_t wgs = 0;
      for (int32_t r = 0; r < n_req; ++r)
        if (ntok_of(r) > 0) wgs += (int64_t)((ntok_of(r) + tok_tile - 1) / tok_tile) * pool->kv_heads;
      small_batch = wgs < n_cu;
    }
    if (flags & TL_PLAN_FUSE_ROWS) {
      std::vector<int32_t> users(pool->n_slots, 0), last_user(pool->n_slots, -1);
      for (int32_t r = 0; r < n_req; ++r) {
        if (ntok_of(r) == 0) continue;
        for (int32_t pos = 0; pos < len_of(r); ++pos) {
          const int32_t sl = slot_at(r, pos);
          if (last_user[sl] != r) {
            last_user[sl] = r;
            users[sl]++;
          }
        }
      }
      for (int32_t r = 0; r < n_req; ++r) {
        const int64_t rows = (int64_t)ntok_of(r) * G;
        if (rows <= kUnitRows) continue;
        if (small_batch && len_of(r) > min_chunk_slots) continue;
        bool shares = false;
        for (int32_t pos = 0; pos < len_of(r) && !shares; ++pos) shares = users[slot_at(r, pos)] > 1;
        fused[r] = rows >= kFuseRows || !shares;
      }
    }
    // ---- walk the prefix tree ---------------------------------------------------------------------
    // every request with a list, in order, front to back; `grouped` requests are those the planner
    // may put together (new tokens, not set aside for the one-pass kernel)
    PrefixTree& tree = pool->tree;
    // Lists that follow no tree (the same segments in ever new orders) would add nodes batch after batch:
    // beyond kTreeNodesPerSlot nodes per slot the tree, a record of loads, starts over.
    if ((int64_t)tree.size() > (int64_t)kTreeNodesPerSlot * pool->n_slots) tree.reset(pool->n_slots);
    tree.begin_batch();
    std::vector<int32_t> path(n_entries);          // tree node of every list entry
    auto is_live = [&](int32_t r) { return ntok_of(r) > 0 && len_of(r) > 0 && !fused[r]; };
    for (int32_t r = 0; r < n_req; ++r) {
      const bool grouped = is_live(r);
      int32_t node = 0;
      for (int32_t i = req_seg_ptr[r]; i < req_seg_ptr[r + 1]; ++i) {
        node = tree.child(node, seg_ids[i], slots[i]);
        tree.visit(node, ntok_of(r), grouped, r);
        path[i] = node;
      }
    }
    // the batch's part of the tree, copied for tl_plan_hot_slots (which must not need the pool)
    {
      const std::vector<int32_t>& bn = tree.batch_nodes();
      const size_t nb = bn.size();
      p->bt_slot.resize(nb);
      p->bt_load.resize(nb);
      p->bt_first_child.resize(nb);
      p->bt_next_sib.resize(nb);
      auto idx = [&](int32_t n) { return n < 0 ? -1 : tree.at(n).batch_index; };
      for (size_t i = 0; i < nb; ++i) {
        const TreeNode& x = tree.at(bn[i]);
        p->bt_slot[i] = x.slot;
        p->bt_load[i] = x.batch_load;
        p->bt_first_child[i] = idx(x.batch_first_child);
        p->bt_next_sib[i] = idx(x.batch_next_sib);
      }
      for (int32_t c = tree.at(0).batch_first_child; c >= 0; c = tree.at(c).batch_next_sib) p->bt_roots.push_back(idx(c));
    }

    // ---- work items from tree nodes -----------------------------------------------------------------
    std::vector<RawItem> raw;
    std::vector<int32_t> live;
    for (int32_t r = 0; r < n_req; ++r)
      if (is_live(r)) live.push_back(r);
    if (flags & TL_PLAN_NO_SHARING) {
      for (int32_t r : live) raw.push_back(RawItem{{r}, r, 0, len_of(r)});
    } else {
      // A run starts at a node and goes down while one child carries all of the node's grouped
      // requests (then nobody has ended and nobody has turned off).  Runs come out parent level
      // first, siblings in order of their first request, then each sibling's subtree in turn.
      std::vector<int32_t> item_of(tree.batch_nodes().size(), -1);   // run that starts at a visited node
      std::vector<int32_t> stack(1, 0), kids, next;
      while (!stack.empty()) {
        const int32_t f = stack.back();
        stack.pop_back();
        kids.clear();
        for (int32_t c = tree.at(f).batch_first_child; c >= 0; c = tree.at(c).batch_next_sib)
          if (tree.at(c).batch_cnt > 0) kids.push_back(c);
        std::sort(kids.begin(), kids.end(),
                  [&](int32_t a, int32_t b) { return tree.at(a).batch_first_req < tree.at(b).batch_first_req; });
        next.clear();
        for (int32_t c : kids) {
          const int32_t cnt = tree.at(c).batch_cnt;
          int32_t last = c;
          for (;;) {
            int32_t all = -1;
            for (int32_t d = tree.at(last).batch_first_child; d >= 0; d = tree.at(d).batch_next_sib)
              if (tree.at(d).batch_cnt == cnt) { all = d; break; }
            if (all < 0) break;
            last = all;
          }
          item_of[tree.at(c).batch_index] = (int32_t)raw.size();
          raw.push_back(RawItem{{}, tree.at(c).batch_first_req, tree.at(c).depth, tree.at(last).depth + 1});
          next.push_back(last);
        }
        for (auto it = next.rbegin(); it != next.rend(); ++it) stack.push_back(*it);
      }
      // who passes through each run's first node, in request order
      for (int32_t r : live)
        for (int32_t i = req_seg_ptr[r]; i < req_seg_ptr[r + 1]; ++i) {
          const int32_t it = item_of[tree.at(path[i]).batch_index];
          if (it >= 0) raw[it].reqs.push_back(r);
        }
    }

    // The kv tokens of a slot list as tiles of kKvTile rows.  A slot listed several times (lists are
    // multisets: Section 3.1 has no order or uniqueness among the segments a request attends to) is
    // walked once; its tiles carry log2 of the multiplicity, which the kernel adds to the exponent
    // (m equal keys weigh m exp(s) in numerator and denominator alike).  Returns the pairs computed.
    const bool dedupe = !(flags & TL_PLAN_WALK_REPEATS);
    std::vector<int32_t> mult_of(dedupe ? pool->n_slots : 0, 0);
    auto emit_tiles = [&](auto slot_of_pos, int32_t n_pos) -> int64_t {
      int64_t kv_tokens = 0;
      if (dedupe)
        for (int32_t pos = 0; pos < n_pos; ++pos) mult_of[slot_of_pos(pos)]++;
      for (int32_t pos = 0; pos < n_pos; ++pos) {
        const int32_t sl = slot_of_pos(pos), f = pool->fill[sl];
        int32_t m = 1;
        if (dedupe) {
          m = mult_of[sl];
          if (m == 0) continue;        // a later occurrence of a slot already emitted
          mult_of[sl] = 0;
        }
        const float lm = log2f((float)m);
        if (m > 1) p->any_repeat = true;
        kv_tokens += f;
        for (int32_t off = 0; off < f; off += kKvTile) {
          if (off + kKvTile <= f) {
            p->tile_base.push_back(sl * pool->seg_len + off);
            p->tile_lm.push_back(lm);
          } else {
            p->part_tile.push_back(sl * pool->seg_len + off);
            p->part_tile.push_back(f - off);
            p->part_lm.push_back(lm);
          }
        }
      }
      return kv_tokens;
    };

    // ---- one-pass tails ---------------------------------------------------------------------
    // TL_PLAN_FUSE_TAILS: a request with more than a token's worth of rows takes the one-pass kernel
    // for the end of its list that nobody shares (the run whose only request it is; possibly empty)
    // and its own new tokens.  The shared runs above stay work items, read once for all their
    // requesters' rows; their partial rows for this request are listed as `priors`, which the
    // one-pass kernel's epilogue merges in, so the request needs no causal tile and no tl_merge.
    std::vector<char> tailed(n_req, 0);
    std::vector<int32_t> tail_begin(n_req, 0), tail_end(n_req, 0);
    std::vector<std::vector<int32_t>> priors(n_req);     // per request: partial row of its first token in every shared item
    std::vector<char> is_tail_item(raw.size(), 0);
    if (flags & TL_PLAN_FUSE_TAILS) {
      for (int32_t r = 0; r < n_req; ++r) {
        if (fused[r] || (int64_t)ntok_of(r) * G <= kUnitRows) continue;
        tailed[r] = 1;
        tail_begin[r] = tail_end[r] = len_of(r);
      }
      for (size_t i = 0; i < raw.size(); ++i) {
        const RawItem& it = raw[i];
        if (it.reqs.size() != 1 || !tailed[it.reqs[0]]) continue;
        const int32_t r = it.reqs[0];
        if (small_batch && it.end - it.begin > min_chunk_slots) {    // long enough to be cut along its KV instead
          tailed[r] = 0;
          continue;
        }
        is_tail_item[i] = 1;
        tail_begin[r] = it.begin;
        tail_end[r] = it.end;
      }
    }

    // ---- final items, work lists ----------------------------------------------------------
    // An item goes to split-K units if it has a token's worth of rows, or if it is a run shared by
    // decode-type requests only (each with a token's worth of rows) that together would not fill
    // one row tile: such a run has too little arithmetic for a row tile to matter and, as a handful
    // of workgroups in a launch of its own, would only add its latency to the step.  Its tokens are
    // then dealt to units of kUnitRows rows, which re-read the run through L2.
    const int32_t tok_unit = std::max(1, kUnitRows / G);
    auto unit_item = [&](const RawItem& it, int64_t n_tok) -> bool {
      if (n_tok * G <= kUnitRows) return true;
      if (n_tok * G > kRowTile) return false;
      for (int32_t r : it.reqs)
        if ((int64_t)ntok_of(r) * G > kUnitRows) return false;
      return true;
    };
    int split = split_segments;
    if (split == 0) {
      // Split-K chunk, in slots.  Measured on decode batches of 1 to 1024 requests: long chunks stream
      // best (2 slots 5.6 TB/s, 8 slots 6.0, 32 slots 6.1, and fewer partials to merge), as long as
      // there are about as many units as CUs or more; equal-sized units that overflow one round of CUs
      // by a little leave a thin second round that cannot fill the memory system.  So: the longest
      // chunk (at most 32 slots, at least 512 tokens) that still gives three quarters of a unit per
      // CU, halved if the count then lands between one and one and a half rounds.
      std::vector<std::pair<int64_t, int64_t>> runs;     // (list entries, token groups) of every unit item
      for (size_t i = 0; i < raw.size(); ++i) {
        const RawItem& it = raw[i];
        if (is_tail_item[i]) continue;
        int64_t n_tok = 0;
        for (int32_t r : it.reqs) n_tok += ntok_of(r);
        if (unit_item(it, n_tok)) runs.emplace_back(it.end - it.begin, (n_tok + tok_unit - 1) / tok_unit);
      }
      auto units_with = [&](int sp) {
        int64_t u = 0;
        for (const auto& r : runs) u += (r.first + sp - 1) / sp * r.second;
        return u;
      };
      const int lo = std::max(1, 512 / pool->seg_len);
      const int64_t cus = n_cu > 0 ? n_cu : kComputeUnits;
      split = 32;
      while (split > lo && 4 * units_with(split) < 3 * cus) --split;
      const int64_t u = units_with(split);
      if (u > cus && 2 * u < 3 * cus && split >= 2 * lo) split /= 2;
    }
    // Row-tile items of a small batch: when all row tiles together are fewer workgroups than the
    // GPU has CUs, long slot lists are cut into chunks (each a work item with partial rows of its
    // own, merged like any other) until there are about two workgroups per CU; a chunk keeps at
    // least 2048 tokens so that its start-up stays small against its work.
    int tile_chunks = 1;
    {
      int64_t wgs = 0;
      for (size_t i = 0; i < raw.size(); ++i) {
        const RawItem& it = raw[i];
        if (is_tail_item[i]) continue;
        int64_t n_tok = 0;
        for (int32_t r : it.reqs) n_tok += ntok_of(r);
        if (!unit_item(it, n_tok)) wgs += ((n_tok + tok_tile - 1) / tok_tile) * pool->kv_heads;
      }
      if (wgs > 0 && wgs < n_cu) tile_chunks = (int)std::min<int64_t>(16, (2 * n_cu + wgs - 1) / wgs);
    }
    int32_t row_cursor = 0;
    p->item_tok_ptr.push_back(0);
    p->item_slot_ptr.push_back(0);
    int64_t prefix_pairs = 0, tile_pairs = 0;
    int32_t n_fused_tokens = 0;
    int64_t item_pairs = 0;
    for (size_t ri = 0; ri < raw.size(); ++ri) {
      const RawItem& it = raw[ri];
      if (is_tail_item[ri]) continue;
      int32_t n_tok = 0;
      for (int32_t r : it.reqs) n_tok += ntok_of(r);
      const bool few_rows = unit_item(it, n_tok);
      // The run's slots, each with the number of times the run lists it.  Split-K units walk a slot
      // that is listed m times once, with weight m, like the row tiles (reading 8 of the paper's
      // silence on repeated segments: a list is a multiset); row-tile items dedupe in emit_tiles,
      // so for them every list position stays an entry of its own here.
      std::vector<std::pair<int32_t, int32_t>> run_slots;
      {
        const int32_t n_pos = it.end - it.begin;
        if (few_rows && dedupe) {
          for (int32_t pos = it.begin; pos < it.end; ++pos) mult_of[slot_at(it.src_req, pos)]++;
          for (int32_t pos = it.begin; pos < it.end; ++pos) {
            const int32_t sl = slot_at(it.src_req, pos);
            if (mult_of[sl] == 0) continue;
            run_slots.emplace_back(sl, mult_of[sl]);
            mult_of[sl] = 0;
          }
        } else {
          run_slots.reserve(n_pos);
          for (int32_t pos = it.begin; pos < it.end; ++pos) run_slots.emplace_back(slot_at(it.src_req, pos), 1);
        }
      }
      const int32_t run = (int32_t)run_slots.size();
      const int32_t step = few_rows ? split
                           : tile_chunks > 1 ? std::max(min_chunk_slots, (run + tile_chunks - 1) / tile_chunks)
                                             : run;
      for (int32_t c0 = 0; c0 < run; c0 += step) {
        const int32_t c1 = std::min(run, c0 + step);
        const int32_t tok_base = (int32_t)p->item_tokens.size();
        for (int32_t r : it.reqs)
          for (int32_t t = req_row_ptr[r]; t < req_row_ptr[r + 1]; ++t) p->item_tokens.push_back(t);
        const int32_t slot_base = (int32_t)p->item_slots.size();
        const int32_t unit_base = (int32_t)p->unit_slots.size();
        for (int32_t u = c0; u < c1; ++u) {
          const int32_t sl = run_slots[u].first, m = run_slots[u].second;
          for (int32_t k = 0; k < m; ++k) p->item_slots.push_back(sl);       // the item's list keeps every occurrence
          prefix_pairs += (int64_t)m * n_tok * pool->fill[sl];
          item_pairs += (int64_t)m * n_tok * pool->fill[sl];
          if (few_rows) {
            p->unit_slots.push_back(sl);
            p->unit_lm.push_back(log2f((float)m));
            if (m > 1) p->any_unit_repeat = true;
          }
        }
        {
          int32_t first = row_cursor;             // partial row of each tailed requester's first token in this item
          for (int32_t r : it.reqs) {
            if (tailed[r]) priors[r].push_back(first);
            first += ntok_of(r);
          }
        }
        p->item_row_base.push_back(row_cursor);
        p->item_tok_ptr.push_back((int32_t)p->item_tokens.size());
        p->item_slot_ptr.push_back((int32_t)p->item_slots.size());
        if (few_rows) {
          for (int32_t t0 = 0; t0 < n_tok; t0 += tok_unit)
            p->units.push_back(Work{tok_base + t0, std::min(tok_unit, n_tok - t0), row_cursor + t0, unit_base, c1 - c0, 0, 0, 0, 0, 0, 0});
        } else {
          // the item's kv tokens as tiles of kKvTile rows (shared by all its row tiles)
          const int32_t full_off = (int32_t)p->tile_base.size();
          const int32_t part_off = (int32_t)p->part_tile.size() / 2;
          tile_pairs += (int64_t)n_tok * emit_tiles([&](int32_t pos) { return p->item_slots[slot_base + pos]; },
                                                    (int32_t)p->item_slots.size() - slot_base);
          const int32_t n_full = (int32_t)p->tile_base.size() - full_off;
          const int32_t n_part = (int32_t)p->part_tile.size() / 2 - part_off;
          // row tiles never straddle two requests' token ranges unless ranges are short:
          // tokens are simply taken tok_tile at a time in item order (Q rows are gathered).
          for (int32_t t0 = 0; t0 < n_tok; t0 += tok_tile)
            p->tiles.push_back(Work{tok_base + t0, std::min(tok_tile, n_tok - t0), row_cursor + t0, slot_base, (int32_t)p->item_slots.size() - slot_base,
                                    full_off, n_full, part_off, n_part, 0, 0});
        }
        if ((int64_t)row_cursor + n_tok + T > INT32_MAX) {      // partial rows are numbered in 32 bits
          set_error("tl_plan_create: more than 2^31 partial rows");
          delete p;
          return TL_EINVAL;
        }
        row_cursor += n_tok;
      }
    }
    // the token array doubles as the tile token list
    p->tok = p->item_tokens;

    const int32_t n_items = (int32_t)p->item_row_base.size();
    int32_t self_base = -1;
    int64_t self_pairs = 0;
    if (flags & TL_PLAN_SELF_BLOCK) {
      self_base = row_cursor;
      const int32_t ident_base = (int32_t)p->tok.size();
      for (int32_t t = 0; t < T; ++t) p->tok.push_back(t);
      for (int32_t r = 0; r < n_req; ++r) {
        const int32_t a = req_row_ptr[r], b = req_row_ptr[r + 1];
        const int64_t lq = b - a;
        self_pairs += lq * (lq + 1) / 2;
        int32_t full_off = 0, n_full = 0, part_off = 0, n_part = 0;
        int32_t prior_off = 0, n_prior = 0;
        if (fused[r] || tailed[r]) {
          // the request's whole slot list (one-pass rows) or the private end of it (one-pass tail) as
          // tiles of kKvTile rows
          const int32_t p0 = fused[r] ? 0 : tail_begin[r], p1 = fused[r] ? len_of(r) : tail_end[r];
          full_off = (int32_t)p->tile_base.size();
          part_off = (int32_t)p->part_tile.size() / 2;
          for (int32_t pos = p0; pos < p1; ++pos) prefix_pairs += lq * pool->fill[slot_at(r, pos)];
          tile_pairs += lq * emit_tiles([&](int32_t pos) { return slot_at(r, p0 + pos); }, p1 - p0);
          n_full = (int32_t)p->tile_base.size() - full_off;
          n_part = (int32_t)p->part_tile.size() / 2 - part_off;
          n_fused_tokens += (int32_t)lq;
          prior_off = (int32_t)p->prior_rows.size();
          n_prior = (int32_t)priors[r].size();
          p->prior_rows.insert(p->prior_rows.end(), priors[r].begin(), priors[r].end());
          fused[r] = 1;                   // from here on the two kinds are the same thing
        }
        if (!fused[r] && lq == 1) {      // a single new token sees itself only: no row tile for it
          p->single_tok.push_back(a);
          continue;
        }
        for (int32_t t0 = a; t0 < b; t0 += tok_tile) {
          const int32_t n = std::min(tok_tile, b - t0);
          if (fused[r])
            p->ftiles.push_back(Work{ident_base + t0, n, t0, a, t0 + n - a, full_off, n_full, part_off, n_part, prior_off, n_prior});
          else
            p->ctiles.push_back(Work{ident_base + t0, n, self_base + t0, a, t0 + n - a, 0, 0, 0, 0, 0, 0});
        }
      }
      row_cursor += T;
    }

    // longest first, so that the tail of the launch is made of short work
    auto by_len = [&](const Work& x, const Work& y) {
      return (x.n_full + x.n_part ? x.n_full + x.n_part : x.kv_len) > (y.n_full + y.n_part ? y.n_full + y.n_part : y.kv_len);
    };
    std::stable_sort(p->tiles.begin(), p->tiles.end(), by_len);
    std::stable_sort(p->units.begin(), p->units.end(), by_len);
    std::stable_sort(p->ctiles.begin(), p->ctiles.end(), by_len);
    // one-pass rows: by the request's pool length only, so that the row tiles of a request stay
    // next to each other in the launch order, run at the same time and share its KV through L2
    std::stable_sort(p->ftiles.begin(), p->ftiles.end(),
                     [](const Work& x, const Work& y) { return x.n_full + x.n_part > y.n_full + y.n_part; });

    // ---- merge lists --------------------------------------------------------------------------
    // (tokens of one-pass requests are in no merge list: a one-pass tail's partial rows in the shared
    // items are read by the one-pass kernel itself)
    std::vector<char> tok_fused(T, 0);
    for (int32_t r = 0; r < n_req; ++r)
      if (fused[r])
        for (int32_t t = req_row_ptr[r]; t < req_row_ptr[r + 1]; ++t) tok_fused[t] = 1;
    p->merge_ptr.assign(T + 1, 0);
    for (int32_t i = 0; i < n_items; ++i)
      for (int32_t j = p->item_tok_ptr[i]; j < p->item_tok_ptr[i + 1]; ++j)
        if (!tok_fused[p->item_tokens[j]]) p->merge_ptr[p->item_tokens[j] + 1]++;
    for (int32_t t = 0; t < T; ++t)
      if (!tok_fused[t]) p->merge_tok.push_back(t);
    if (self_base >= 0)
      for (int32_t t = 0; t < T; ++t)
        if (!tok_fused[t]) p->merge_ptr[t + 1]++;
    for (int32_t t = 0; t < T; ++t) p->merge_ptr[t + 1] += p->merge_ptr[t];
    // tokens with long lists (split-K) last: tl_merge gives them the sliced kernel
    {
      auto is_short = [&](int32_t t) { return p->merge_ptr[t + 1] - p->merge_ptr[t] < kLongMergeList; };
      auto mid = std::stable_partition(p->merge_tok.begin(), p->merge_tok.end(), is_short);
      p->n_merge_short = (int32_t)(mid - p->merge_tok.begin());
    }
    p->merge_rows.assign(p->merge_ptr[T], 0);
    {
      std::vector<int32_t> cur(p->merge_ptr.begin(), p->merge_ptr.end() - 1);
      for (int32_t i = 0; i < n_items; ++i)
        for (int32_t j = p->item_tok_ptr[i]; j < p->item_tok_ptr[i + 1]; ++j)
          if (!tok_fused[p->item_tokens[j]]) p->merge_rows[cur[p->item_tokens[j]]++] = p->item_row_base[i] + (j - p->item_tok_ptr[i]);
      if (self_base >= 0)
        for (int32_t t = 0; t < T; ++t)
          if (!tok_fused[t]) p->merge_rows[cur[t]++] = self_base + t;
    }
    // the short lists once more as fixed records, so that the merge kernel gets a token's whole list with
    // one load instead of three dependent ones
    static_assert(kLongMergeList <= kMergeFixInts, "a short list and its token fit one record");
    p->merge_fix.assign((size_t)p->n_merge_short * kMergeFixInts, -1);
    for (int32_t i = 0; i < p->n_merge_short; ++i) {
      const int32_t t = p->merge_tok[i];
      int32_t* rec = &p->merge_fix[(size_t)i * kMergeFixInts];
      rec[0] = t;
      for (int32_t j = p->merge_ptr[t]; j < p->merge_ptr[t + 1]; ++j) rec[1 + j - p->merge_ptr[t]] = p->merge_rows[j];
    }

    int64_t uniq_tok = 0;
    {
      std::vector<char> seen(pool->n_slots, 0);
      for (int32_t s : slots)
        if (!seen[s]) {
          seen[s] = 1;
          uniq_tok += pool->fill[s];
        }
    }

    tl_plan_info& inf = p->info;
    memset(&inf, 0, sizeof(inf));
    inf.n_req = n_req;
    inf.n_tokens = T;
    inf.q_heads = q_heads;
    inf.kv_heads = pool->kv_heads;
    inf.n_items = n_items;
    inf.n_partial_rows = row_cursor;
    inf.self_row_base = self_base;
    inf.n_tiles = (int32_t)p->tiles.size();
    inf.n_units = (int32_t)p->units.size();
    inf.n_causal_tiles = (int32_t)p->ctiles.size();
    inf.n_list_entries = n_entries;
    inf.n_merge_entries = (int32_t)p->merge_rows.size();
    inf.prefix_pairs = prefix_pairs;
    inf.self_pairs = self_pairs;
    inf.unique_kv_tokens = uniq_tok;
    inf.n_fused_tiles = (int32_t)p->ftiles.size();
    inf.n_fused_tokens = n_fused_tokens;
    inf.n_single_tokens = (int32_t)p->single_tok.size();
    inf.tile_pairs = tile_pairs;
    inf.item_pairs = item_pairs;
    inf.n_prior_rows = (int32_t)p->prior_rows.size();

    // ---- one block with everything the kernels read ---------------------------------------------
    {
      size_t total = 0;
      auto reserve = [&](size_t bytes) {
        const size_t at = total;
        total += (bytes + 255) & ~(size_t)255;
        return at;
      };
      auto& o = p->off;
      o.tiles = reserve(sizeof(Work) * p->tiles.size());
      o.units = reserve(sizeof(Work) * p->units.size());
      o.ctiles = reserve(sizeof(Work) * p->ctiles.size());
      o.ftiles = reserve(sizeof(Work) * p->ftiles.size());
      o.tok = reserve(sizeof(int32_t) * p->tok.size());
      o.slots = reserve(sizeof(int32_t) * p->unit_slots.size());
      o.unit_lm = reserve(sizeof(float) * p->unit_lm.size());
      o.merge_ptr = reserve(sizeof(int32_t) * p->merge_ptr.size());
      o.merge_rows = reserve(sizeof(int32_t) * p->merge_rows.size());
      o.tile_base = reserve(sizeof(int32_t) * p->tile_base.size());
      o.part_tile = reserve(sizeof(int32_t) * p->part_tile.size());
      o.merge_tok = reserve(sizeof(int32_t) * p->merge_tok.size());
      o.single_tok = reserve(sizeof(int32_t) * p->single_tok.size());
      o.tile_lm = reserve(sizeof(float) * p->tile_lm.size());
      o.part_lm = reserve(sizeof(float) * p->part_lm.size());
      o.prior_rows = reserve(sizeof(int32_t) * p->prior_rows.size());
      o.merge_fix = reserve(sizeof(int32_t) * p->merge_fix.size());
      p->blob_host.assign(total + 256, 0);
      auto fill = [&](size_t at, const void* src, size_t bytes) {
        if (bytes) memcpy(p->blob_host.data() + at, src, bytes);
      };
      fill(o.tiles, p->tiles.data(), sizeof(Work) * p->tiles.size());
      fill(o.units, p->units.data(), sizeof(Work) * p->units.size());
      fill(o.ctiles, p->ctiles.data(), sizeof(Work) * p->ctiles.size());
      fill(o.ftiles, p->ftiles.data(), sizeof(Work) * p->ftiles.size());
      fill(o.tok, p->tok.data(), sizeof(int32_t) * p->tok.size());
      fill(o.slots, p->unit_slots.data(), sizeof(int32_t) * p->unit_slots.size());
      fill(o.unit_lm, p->unit_lm.data(), sizeof(float) * p->unit_lm.size());
      fill(o.merge_ptr, p->merge_ptr.data(), sizeof(int32_t) * p->merge_ptr.size());
      fill(o.merge_rows, p->merge_rows.data(), sizeof(int32_t) * p->merge_rows.size());
      fill(o.tile_base, p->tile_base.data(), sizeof(int32_t) * p->tile_base.size());
      fill(o.part_tile, p->part_tile.data(), sizeof(int32_t) * p->part_tile.size());
      fill(o.merge_tok, p->merge_tok.data(), sizeof(int32_t) * p->merge_tok.size());
      fill(o.single_tok, p->single_tok.data(), sizeof(int32_t) * p->single_tok.size());
      fill(o.tile_lm, p->tile_lm.data(), sizeof(float) * p->tile_lm.size());
      fill(o.part_lm, p->part_lm.data(), sizeof(float) * p->part_lm.size());
      fill(o.prior_rows, p->prior_rows.data(), sizeof(int32_t) * p->prior_rows.size());
      fill(o.merge_fix, p->merge_fix.data(), sizeof(int32_t) * p->merge_fix.size());
    }
  } catch (const std::bad_alloc&) {
    rc = TL_ENOMEM;
    set_error("tl_plan_create: host allocation failed");
  }
  if (rc != TL_OK) {
    delete p;
    return rc;
  }
  *out = p;
  return TL_OK;
}

tl_status tl_plan_destroy(tl_plan* plan) {
  if (!plan) return TL_OK;
  if (plan->blob_dev) (void)hipFree(plan->blob_dev);
  delete plan;
  return TL_OK;
}

tl_status tl_plan_get_info(const tl_plan* plan, tl_plan_info* info) {
  if (!plan || !info) TL_FAIL(TL_EINVAL, "tl_plan_get_info: bad argument");
  *info = plan->info;
  return TL_OK;
}

tl_status tl_plan_hot_slots(const tl_plan* plan, int32_t max_n, int32_t* slots_out, int64_t* loads_out, int32_t* n_out) {
  if (!plan || max_n < 0 || !n_out || (max_n > 0 && !slots_out)) TL_FAIL(TL_EINVAL, "tl_plan_hot_slots: bad argument");
  // Best-first search from the root over the nodes this batch walked: a node enters the frontier when
  // its parent leaves it and is never more loaded than its parent, so nodes leave in order of
  // decreasing load (equal loads: first visited first) and only the children of what is returned
  // are ever looked at.
  int32_t n = 0;
  try {
    auto later = [&](int32_t a, int32_t b) { return plan->bt_load[a] != plan->bt_load[b] ? plan->bt_load[a] < plan->bt_load[b] : a > b; };
    std::priority_queue<int32_t, std::vector<int32_t>, decltype(later)> frontier(later);
    for (int32_t c : plan->bt_roots) frontier.push(c);
    while (n < max_n && !frontier.empty()) {
      const int32_t x = frontier.top();
      frontier.pop();
      slots_out[n] = plan->bt_slot[x];
      if (loads_out) loads_out[n] = plan->bt_load[x];
      ++n;
      for (int32_t c = plan->bt_first_child[x]; c >= 0; c = plan->bt_next_sib[c]) frontier.push(c);
    }
  } catch (const std::bad_alloc&) {
    TL_FAIL(TL_ENOMEM, "tl_plan_hot_slots: host allocation failed");
  }
  *n_out = n;
  return TL_OK;
}

tl_status tl_plan_export_sizes(const tl_plan* plan, int32_t* n_item_tokens, int32_t* n_item_slots) {
  if (!plan) TL_FAIL(TL_EINVAL, "tl_plan_export_sizes: null plan");
  if (n_item_tokens) *n_item_tokens = (int32_t)plan->item_tokens.size();
  if (n_item_slots) *n_item_slots = (int32_t)plan->item_slots.size();
  return TL_OK;
}

tl_status tl_plan_export(const tl_plan* plan, int32_t* item_row_base, int32_t* item_tok_ptr, int32_t* item_tokens,
                         int32_t* item_slot_ptr, int32_t* item_slots, int32_t* merge_ptr, int32_t* merge_rows) {
  if (!plan) TL_FAIL(TL_EINVAL, "tl_plan_export: null plan");
  auto cp = [](int32_t* dst, const std::vector<int32_t>& src) {
    if (dst && !src.empty()) memcpy(dst, src.data(), sizeof(int32_t) * src.size());
  };
  cp(item_row_base, plan->item_row_base);
  cp(item_tok_ptr, plan->item_tok_ptr);
  cp(item_tokens, plan->item_tokens);
  cp(item_slot_ptr, plan->item_slot_ptr);
  cp(item_slots, plan->item_slots);
  cp(merge_ptr, plan->merge_ptr);
  cp(merge_rows, plan->merge_rows);
  return TL_OK;
}

}  // extern "C"

namespace tl {

tl_status plan_device_ready(tl_plan* p, hipStream_t stream) {
  if (p->blob_dev) return TL_OK;
  void* blob = nullptr;
  TL_HIP(hipMalloc(&blob, p->blob_host.size()));
  // on the caller's stream, in order with the kernels that read it; the host block belongs to the
  // plan, which the caller keeps alive until the stream work of its calls has completed
  hipError_t e = hipMemcpyAsync(blob, p->blob_host.data(), p->blob_host.size(), hipMemcpyHostToDevice, stream);
  if (e != hipSuccess) {
    (void)hipFree(blob);
    TL_FAIL(TL_EHIP, "plan upload failed: %s", hipGetErrorString(e));
  }
  p->blob_dev = blob;
  return TL_OK;
}

tl_status plan_is_current(const tl_plan* plan, const tl_pool* pool, const char* who) {
  if (plan->pool != pool) TL_FAIL(TL_EINVAL, "%s: plan was built for another pool", who);
  if (plan->pool_generation != pool->generation)
    TL_FAIL(TL_EINVAL, "%s: the pool has changed since the plan was built (put, append, adopt or evict): build a new plan", who);
  return TL_OK;
}

}  // namespace tl
