// Hierarchical pCtx pool: construction and lease-conflict rules (Sec. 4.3).
#include "pool.h"

#include <algorithm>

namespace vte {

int Pool::add_node(int lo, int hi, int parent, int level, int leaf_cus) {
  const int id = static_cast<int>(p_.size());
  p_.emplace_back();
  {
    Pctx& n = p_[id];
    n.id = id;
    n.kind = kNode;
    n.level = level;
    n.parent = parent;
    n.leaf_lo = lo;
    n.leaf_hi = hi;
    n.width = (hi - lo) * leaf_cus;
    n.mask.assign(words_, 0u);
    for (int cu = lo * leaf_cus; cu < hi * leaf_cus; ++cu) n.mask[cu >> 5] |= 1u << (cu & 31);
  }
  if (hi - lo > 1) {
    const int mid = lo + (hi - lo) / 2;
    const int c0 = add_node(lo, mid, id, level + 1, leaf_cus);
    const int c1 = add_node(mid, hi, id, level + 1, leaf_cus);
    p_[id].child[0] = c0;
    p_[id].child[1] = c1;
  }
  return id;
}

bool Pool::build(int total_cus, int leaf_cus, int remainders, std::string* err) {
  p_.clear();
  active_nodes_ = active_remainders_ = 0;
  active_rem_ids_.clear();
  if (total_cus <= 0 || leaf_cus <= 0 || leaf_cus > total_cus) {
    if (err) *err = "pool: need 0 < leaf_cus <= total_cus";
    return false;
  }
  int leaves = 1;
  while (leaves * 2 * leaf_cus <= total_cus) leaves *= 2;
  total_ = total_cus;
  leaf_ = leaf_cus;
  leaves_ = leaves;
  words_ = (total_cus + 31) / 32;
  root_ = add_node(0, leaves, -1, 0, leaf_cus);
  if (remainders == 0) return true;
  const int nodes = size();
  std::vector<char> level_done(64, 0);
  for (int id = 0; id < nodes; ++id) {
    if (id == root_) continue;  // nothing would be left (or less than a leaf)
    // a child of the root is complemented by its sibling when the tree covers
    // the whole device: link instead of creating a duplicate allocation
    if (p_[id].parent == root_ && leaves_ * leaf_ == total_) {
      const Pctx& par = p_[root_];
      p_[id].remainder = (par.child[0] == id) ? par.child[1] : par.child[0];
      continue;
    }
    if (remainders == 2) {  // bounded variant: only the first node of every level gets one
      if (level_done[p_[id].level]) continue;
      level_done[p_[id].level] = 1;
    }
    const int rem_width = total_ - p_[id].width;
    const int rid = size();
    p_.emplace_back();
    Pctx& r = p_[rid];
    r.id = rid;
    r.kind = kRemainder;
    r.parent = id;
    r.level = p_[id].level;
    r.width = rem_width;
    r.mask.assign(words_, 0u);
    for (int cu = 0; cu < total_; ++cu) {
      const bool in_node = (p_[id].mask[cu >> 5] >> (cu & 31)) & 1u;
      if (!in_node) r.mask[cu >> 5] |= 1u << (cu & 31);
    }
    p_[id].remainder = rid;
  }
  return true;
}

void Pool::assign_pipes(int pipes) {
  pipes_ = std::max(1, pipes);
  const int n = size();
  std::vector<int> order(n), color(n, -1);
  for (int i = 0; i < n; ++i) order[i] = i;
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return p_[a].width > p_[b].width; });
  auto weight = [&](int a, int b) {
    int w = std::min(p_[a].width, p_[b].width);
    if (p_[a].remainder == b || p_[b].remainder == a) w *= 4;  // a node and its complement are the pair meant to run together
    return w;
  };
  auto pick = [&](int x) {
    int best = 0;
    long best_cost = -1;
    int best_used = 0;
    for (int c = 0; c < pipes_; ++c) {
      long cost = 0;
      int used = 0;
      for (int q = 0; q < n; ++q) {
        if (q == x || color[q] != c) continue;
        ++used;
        if (!overlaps(x, q)) cost += weight(x, q);
      }
      if (best_cost < 0 || cost < best_cost || (cost == best_cost && used < best_used)) { best = c; best_cost = cost; best_used = used; }
    }
    return best;
  };
  for (int x : order) color[x] = pick(x);
  for (int pass = 0; pass < 8; ++pass) {  // local improvement until nothing moves
    bool moved = false;
    for (int x : order) {
      const int c = pick(x);
      if (c != color[x]) { color[x] = c; moved = true; }
    }
    if (!moved) break;
  }
  // relabel: most used pipe first, so the creation order needs no (or few) placeholders
  std::vector<int> count(pipes_, 0), label(pipes_), rank(pipes_);
  for (int i = 0; i < n; ++i) ++count[color[i]];
  for (int c = 0; c < pipes_; ++c) label[c] = c;
  std::stable_sort(label.begin(), label.end(), [&](int a, int b) { return count[a] > count[b]; });
  for (int r = 0; r < pipes_; ++r) rank[label[r]] = r;
  for (int i = 0; i < n; ++i) p_[i].pipe = rank[color[i]];
}

std::vector<int> Pool::creation_order() const {
  std::vector<std::vector<int>> by_pipe(pipes_);
  for (int i = 0; i < size(); ++i) by_pipe[p_[i].pipe].push_back(i);
  std::vector<size_t> next(pipes_, 0);
  std::vector<int> out;
  int left = size();
  for (int k = 0; left > 0; ++k) {
    const int c = k % pipes_;
    if (next[c] < by_pipe[c].size()) { out.push_back(by_pipe[c][next[c]++]); --left; }
    else out.push_back(-1);
  }
  return out;
}

bool Pool::is_ancestor_or_self(int anc, int node) const {
  for (int n = node; n >= 0; n = p_[n].parent)
    if (n == anc) return true;
  return false;
}

bool Pool::overlaps(int a, int b) const {
  if (a == b) return true;
  const Pctx& A = p_[a];
  const Pctx& B = p_[b];
  if (A.kind == kNode && B.kind == kNode)
    return is_ancestor_or_self(a, b) || is_ancestor_or_self(b, a);
  if (A.kind == kRemainder && B.kind == kNode) return !is_ancestor_or_self(A.parent, b);
  if (A.kind == kNode && B.kind == kRemainder) return !is_ancestor_or_self(B.parent, a);
  // two remainders miss each other only if their nodes jointly cover every CU,
  // i.e. the nodes are the two children of a root that spans the device; such
  // remainders are links to nodes and never appear here
  return true;
}

void Pool::set_active(int id, bool on) {
  Pctx& x = p_[id];
  const int want = on ? 1 : 0;
  if (x.active_self == want) return;
  x.active_self = want;
  const int d = on ? 1 : -1;
  if (x.kind == kNode) {
    active_nodes_ += d;
    for (int n = x.parent; n >= 0; n = p_[n].parent) p_[n].active_below += d;
  } else {
    active_remainders_ += d;
    if (on) active_rem_ids_.push_back(id);
    else active_rem_ids_.erase(std::remove(active_rem_ids_.begin(), active_rem_ids_.end(), id), active_rem_ids_.end());
  }
}

namespace {
// Active nodes in the subtree of `n` (n included), skipping the subtree of `skip`.
void collect_active(const std::vector<Pctx>& p, int n, int skip, std::vector<int>* out) {
  if (n < 0 || n == skip) return;
  if (p[n].active_self) out->push_back(n);
  if (p[n].active_below == 0) return;
  collect_active(p, p[n].child[0], skip, out);
  collect_active(p, p[n].child[1], skip, out);
}
}  // namespace

void Pool::active_overlapping(int id, std::vector<int>* out) const {
  const Pctx& x = p_[id];
  if (x.kind == kNode) {
    for (int n = x.parent; n >= 0; n = p_[n].parent)  // ancestors
      if (p_[n].active_self) out->push_back(n);
    if (x.active_below) {                               // descendants
      collect_active(p_, x.child[0], -1, out);
      collect_active(p_, x.child[1], -1, out);
    }
    // an active remainder of node m overlaps unless this node lies inside m
    for (int r : active_rem_ids_)
      if (!is_ancestor_or_self(p_[r].parent, id)) out->push_back(r);
  } else {
    // every active node outside the complemented node's subtree, and every other
    // active remainder
    if (active_nodes_ > p_[x.parent].active_self + p_[x.parent].active_below)
      collect_active(p_, root_, x.parent, out);
    for (int r : active_rem_ids_)
      if (r != id) out->push_back(r);
  }
}

bool Pool::conflicts_with_active(int id, int ignore_reserved_for) const {
  if (active_nodes_ + active_remainders_ == 0) return false;
  static thread_local std::vector<int> ov;  // asked for every pCtx in every dispatch round: no allocation per call
  ov.clear();
  active_overlapping(id, &ov);
  for (int o : ov) {
    const Pctx& q = p_[o];
    const bool only_reservation = (q.state == kReserved || (q.state == kIdle && q.reservation_pending));
    if (ignore_reserved_for >= 0 && only_reservation && q.reserved_for == ignore_reserved_for) continue;
    return true;
  }
  return false;
}

}  // namespace vte
