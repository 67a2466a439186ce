// The pool's prefix tree (paper Section 3.1: a global prefix tree indexes the cache segments and
// is what `get_prefix_tree` hands to the scheduler; Section 4.3: a segment is accessed only when
// its prefix is, so load concentrates near the root and heavy hitters are found from the root
// without walking the whole tree).  Host-side, owned by a tl_pool, alive across batches.
//
// A node is a segment at one position: (parent node, segment id).  The same id under two
// different prefixes is two nodes that name the same slot.  Every request list that is walked
// from the root adds the request's new tokens to the load of each node on its way, so a node
// is never more loaded than its parent; that is what lets the most loaded nodes be found by a
// best-first search that expands only what it returns.
#pragma once

#include <cstdint>
#include <unordered_map>
#include <vector>

namespace tl {

struct TreeNode {
  uint64_t id;        // segment id
  int32_t slot;       // the segment's pool slot
  int32_t parent;     // node index; 0 = the root
  int32_t depth;      // 0 for children of the root
  int32_t first_child, last_child, next_sib, prev_sib;   // children in order of creation
  int32_t next_same_slot, prev_same_slot;                // all nodes of one slot (for eviction)
  uint64_t created;   // creation order (ties of equal loads)
  int64_t load;       // cumulative: new tokens of every request walked through this node
  // marks of the batch being planned (valid while epoch == the tree's)
  uint64_t epoch;
  int64_t batch_load;   // new tokens of this batch's requests through the node
  int32_t batch_cnt;    // grouped requests of this batch through the node
  int32_t batch_seq;    // order of first visit in this batch
  int32_t batch_first_child, batch_last_child, batch_next_sib;   // children visited in this batch, in that order
  int32_t batch_first_req;                                       // first grouped request through the node
  int32_t batch_index;                                           // position in the batch's list of visited nodes
};

class PrefixTree {
 public:
  PrefixTree();
  void reset(int32_t n_slots);
  // child of `parent` with this id, created (naming `slot`) if absent
  int32_t child(int32_t parent, uint64_t id, int32_t slot);
  // removes every node that names `slot`, with its subtree
  void remove_slot(int32_t slot);
  // starts a new batch: all per-batch marks become invalid
  void begin_batch();
  // marks node n as visited by a request of `ntok` new tokens; `grouped` requests also count for the
  // planner's grouping, `req` is the request's index.  Returns true on the node's first visit in this batch.
  bool visit(int32_t n, int64_t ntok, bool grouped, int32_t req);
  // up to max_n nodes by decreasing cumulative load (equal loads: older first); best-first from the root
  void hottest(int32_t max_n, std::vector<int32_t>& out) const;
  // level order from the root, at most max_n nodes
  void level_order(int32_t max_n, std::vector<int32_t>& out) const;

  const TreeNode& at(int32_t n) const { return nodes_[n]; }
  TreeNode& at(int32_t n) { return nodes_[n]; }
  int32_t size() const { return live_; }     // nodes alive, the root not counted
  uint64_t epoch() const { return epoch_; }
  const std::vector<int32_t>& batch_nodes() const { return batch_nodes_; }   // visited in this batch, in order of first visit

 private:
  struct Key {
    int32_t parent;
    uint64_t id;
    bool operator==(const Key& o) const { return parent == o.parent && id == o.id; }
  };
  struct KeyHash {
    size_t operator()(const Key& k) const {
      uint64_t z = k.id + 0x9E3779B97F4A7C15ull * (uint64_t)(uint32_t)(k.parent + 1);
      z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
      z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
      return (size_t)(z ^ (z >> 31));
    }
  };
  void unlink(int32_t n);
  std::vector<TreeNode> nodes_;       // [0] is the root
  std::vector<int32_t> free_;
  std::unordered_map<Key, int32_t, KeyHash> child_of_;
  std::vector<int32_t> slot_head_;    // first node of every slot, -1 = none
  std::vector<int32_t> batch_nodes_;
  uint64_t epoch_, created_;
  int32_t live_;
};

}  // namespace tl
