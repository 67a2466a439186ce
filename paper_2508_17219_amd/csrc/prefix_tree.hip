// Prefix tree of the segment pool: see prefix_tree.h.  Host code only.
#include "prefix_tree.h"

#include <queue>

namespace tl {

PrefixTree::PrefixTree() { reset(0); }

void PrefixTree::reset(int32_t n_slots) {
  nodes_.clear();
  free_.clear();
  child_of_.clear();
  batch_nodes_.clear();
  slot_head_.assign(n_slots, -1);
  epoch_ = 1;
  created_ = 0;
  live_ = 0;
  TreeNode root{};
  root.slot = -1;
  root.parent = -1;
  root.depth = -1;
  root.first_child = root.last_child = root.next_sib = root.prev_sib = -1;
  root.next_same_slot = root.prev_same_slot = -1;
  root.batch_first_child = root.batch_last_child = root.batch_next_sib = -1;
  nodes_.push_back(root);
}

int32_t PrefixTree::child(int32_t parent, uint64_t id, int32_t slot) {
  // most nodes sit on a chain with one child: look at the parent's own links before the table
  const int32_t fc = nodes_[parent].first_child;
  if (fc >= 0) {
    if (nodes_[fc].id == id) return fc;
    const int32_t lc = nodes_[parent].last_child;
    if (nodes_[lc].id == id) return lc;
  }
  auto it = child_of_.find(Key{parent, id});
  if (it != child_of_.end()) return it->second;
  int32_t n;
  if (!free_.empty()) {
    n = free_.back();
    free_.pop_back();
  } else {
    n = (int32_t)nodes_.size();
    nodes_.emplace_back();
  }
  TreeNode& x = nodes_[n];
  x = TreeNode{};
  x.id = id;
  x.slot = slot;
  x.parent = parent;
  x.depth = nodes_[parent].depth + 1;
  x.first_child = x.last_child = x.next_sib = -1;
  x.created = ++created_;
  x.batch_first_child = x.batch_last_child = x.batch_next_sib = -1;
  // last among its parent's children
  x.prev_sib = nodes_[parent].last_child;
  if (x.prev_sib >= 0) nodes_[x.prev_sib].next_sib = n; else nodes_[parent].first_child = n;
  nodes_[parent].last_child = n;
  // first among its slot's nodes
  x.prev_same_slot = -1;
  x.next_same_slot = slot_head_[slot];
  if (x.next_same_slot >= 0) nodes_[x.next_same_slot].prev_same_slot = n;
  slot_head_[slot] = n;
  child_of_.emplace(Key{parent, id}, n);
  ++live_;
  return n;
}

// takes node n (whose children are gone already) out of every list it is on
void PrefixTree::unlink(int32_t n) {
  TreeNode& x = nodes_[n];
  if (x.prev_sib >= 0) nodes_[x.prev_sib].next_sib = x.next_sib; else nodes_[x.parent].first_child = x.next_sib;
  if (x.next_sib >= 0) nodes_[x.next_sib].prev_sib = x.prev_sib; else nodes_[x.parent].last_child = x.prev_sib;
  if (x.prev_same_slot >= 0) nodes_[x.prev_same_slot].next_same_slot = x.next_same_slot; else slot_head_[x.slot] = x.next_same_slot;
  if (x.next_same_slot >= 0) nodes_[x.next_same_slot].prev_same_slot = x.prev_same_slot;
  child_of_.erase(Key{x.parent, x.id});
  x.epoch = 0;
  free_.push_back(n);
  --live_;
}

void PrefixTree::remove_slot(int32_t slot) {
  std::vector<int32_t> stack, order;
  while (slot_head_[slot] >= 0) {
    // the subtree under the slot's first node, children before parents
    stack.assign(1, slot_head_[slot]);
    order.clear();
    while (!stack.empty()) {
      const int32_t n = stack.back();
      stack.pop_back();
      order.push_back(n);
      for (int32_t c = nodes_[n].first_child; c >= 0; c = nodes_[c].next_sib) stack.push_back(c);
    }
    for (auto it = order.rbegin(); it != order.rend(); ++it) unlink(*it);
  }
  // per-batch child lists may name removed nodes: they are rebuilt by the next batch
  ++epoch_;
  batch_nodes_.clear();
}

void PrefixTree::begin_batch() {
  ++epoch_;
  batch_nodes_.clear();
  nodes_[0].epoch = epoch_;
  nodes_[0].batch_first_child = nodes_[0].batch_last_child = -1;
}

bool PrefixTree::visit(int32_t n, int64_t ntok, bool grouped, int32_t req) {
  TreeNode& x = nodes_[n];
  x.load += ntok;
  const bool first = x.epoch != epoch_;
  if (first) {
    x.epoch = epoch_;
    x.batch_load = 0;
    x.batch_cnt = 0;
    x.batch_first_req = -1;
    x.batch_seq = x.batch_index = (int32_t)batch_nodes_.size();
    x.batch_first_child = x.batch_last_child = x.batch_next_sib = -1;
    batch_nodes_.push_back(n);
    TreeNode& p = nodes_[x.parent];
    if (p.batch_last_child >= 0) nodes_[p.batch_last_child].batch_next_sib = n; else p.batch_first_child = n;
    p.batch_last_child = n;
  }
  x.batch_load += ntok;
  if (grouped) {
    if (x.batch_cnt == 0) x.batch_first_req = req;
    x.batch_cnt++;
  }
  return first;
}

void PrefixTree::hottest(int32_t max_n, std::vector<int32_t>& out) const {
  out.clear();
  // best-first from the root: a node enters the frontier when its parent leaves it, and no node is
  // more loaded than its parent, so nodes leave in order of decreasing load (older first among equals)
  auto later = [&](int32_t a, int32_t b) {
    const TreeNode &x = nodes_[a], &y = nodes_[b];
    return x.load != y.load ? x.load < y.load : x.created > y.created;
  };
  std::priority_queue<int32_t, std::vector<int32_t>, decltype(later)> frontier(later);
  for (int32_t c = nodes_[0].first_child; c >= 0; c = nodes_[c].next_sib) frontier.push(c);
  while ((int32_t)out.size() < max_n && !frontier.empty()) {
    const int32_t n = frontier.top();
    frontier.pop();
    out.push_back(n);
    for (int32_t c = nodes_[n].first_child; c >= 0; c = nodes_[c].next_sib) frontier.push(c);
  }
}

void PrefixTree::level_order(int32_t max_n, std::vector<int32_t>& out) const {
  out.clear();
  size_t head = 0;
  for (int32_t c = nodes_[0].first_child; c >= 0 && (int32_t)out.size() < max_n; c = nodes_[c].next_sib) out.push_back(c);
  while (head < out.size() && (int32_t)out.size() < max_n) {
    const int32_t n = out[head++];
    for (int32_t c = nodes_[n].first_child; c >= 0 && (int32_t)out.size() < max_n; c = nodes_[c].next_sib) out.push_back(c);
  }
}

}  // namespace tl
