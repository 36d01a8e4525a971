// Hierarchical pCtx pool (Sec. 4.3 of the paper): a bounded, pre-created set of
// CU allocations organised as a binary tree of nodes plus one remainder pCtx
// per non-root node.  Nothing is created or merged at run time; the tree only
// organises alternatives, remainder links and lease constraints.
//
// This file is pure host logic (no HIP): the backend attaches a stream to each
// entry, the dispatcher drives the state machine.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

namespace vte {

enum PctxKind { kNode = 0, kRemainder = 1 };
enum PctxState { kIdle = 0, kLeased = 1, kDraining = 2, kReserved = 3 };

struct Pctx {
  int id = -1;
  int kind = kNode;
  int width = 0;
  int level = 0;
  int parent = -1;          // node: parent node; remainder: the node it complements
  int child[2] = {-1, -1};
  int remainder = -1;       // node: pCtx covering every other CU (-1 for the root)
  int leaf_lo = 0, leaf_hi = 0;  // node: leaves [lo,hi)
  std::vector<uint32_t> mask;    // one bit per CU
  int pipe = 0;                  // dispatch pipe its queue is meant to land on (see assign_pipes)
  // ---- dynamic state (guarded by the runtime lock) ----
  int state = kIdle;
  bool gate_open = true;
  int outstanding = 0;
  int holder = -1;          // vstream whose ops hold the current lease (-1: explicit launches)
  int reserved_for = -1;    // vstream id that holds / awaits a reservation
  bool reservation_pending = false;  // reservation waits for overlapping work to drain
  // hierarchy bookkeeping for conflict checks by traversal
  int active_self = 0;      // 1 while this pCtx holds a resource commitment
  int active_below = 0;     // node: number of active node-descendants
  void* stream = nullptr;   // backend object
};

class Pool {
 public:
  // total_cus CUs, minimum unit leaf_cus; leaves = largest power of two not above
  // total/leaf.  CUs beyond leaves*leaf belong to remainders only.
  // remainders: 0 none, 1 one per non-root node, 2 one per tree level (for the first node of the level)
  bool build(int total_cus, int leaf_cus, int remainders, std::string* err);

  int size() const { return static_cast<int>(p_.size()); }
  Pctx& at(int id) { return p_[id]; }
  const Pctx& at(int id) const { return p_[id]; }
  int total_cus() const { return total_; }
  int mask_words() const { return words_; }
  int root() const { return root_; }

  // Static overlap of two pCtxs, decided from the hierarchy alone:
  //   node/node           : one is an ancestor of (or equal to) the other;
  //   remainder(n)/node m : unless m lies inside n's subtree (m == n included);
  //   remainder/remainder : always, unless the two nodes together cover the device.
  bool overlaps(int a, int b) const;

  // "Active" = holds a resource commitment (leased, draining, reserved or with a
  // pending reservation).  True if `id` overlaps an active pCtx other than itself.
  // If `ignore_reserved_for` >= 0, reservations held by that vstream do not count.
  bool conflicts_with_active(int id, int ignore_reserved_for = -1) const;
  // Active pCtxs overlapping `id` (excluding itself), appended to *out.
  void active_overlapping(int id, std::vector<int>* out) const;

  void set_active(int id, bool on);  // keeps active_below / remainder counters in step
  bool is_active(int id) const { return p_[id].active_self != 0; }

  bool is_ancestor_or_self(int anc, int node) const;  // both NODE ids

  // The command processor dispatches from a fixed number of pipes, and queues on
  // the same pipe dispatch one kernel at a time: two disjoint pCtxs whose queues
  // share a pipe do not overlap in time however many CUs are free.  Gives every
  // pCtx a pipe in [0,pipes) so that disjoint pCtxs share one as little as
  // possible: a node and the remainder that complements it weigh most, then
  // pairs by the width of the narrower one.  Pipe labels are ordered by how many
  // pCtxs use them, most first.
  void assign_pipes(int pipes);
  // Order in which to create the backend queues so that the k-th queue created
  // (they are dealt to pipes round-robin) belongs to a pCtx of pipe k % pipes;
  // -1 entries are placeholder queues that keep the rotation in step.
  std::vector<int> creation_order() const;
  int pipes() const { return pipes_; }

 private:
  int add_node(int lo, int hi, int parent, int level, int leaf_cus);
  std::vector<Pctx> p_;
  int total_ = 0, leaf_ = 0, leaves_ = 0, words_ = 0, root_ = -1, pipes_ = 1;
  int active_nodes_ = 0;       // number of active NODE pCtxs
  int active_remainders_ = 0;  // number of active REMAINDER pCtxs
  std::vector<int> active_rem_ids_;
};

}  // namespace vte
