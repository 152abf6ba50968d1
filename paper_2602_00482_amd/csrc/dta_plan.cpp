// Host side, integer only: the paper's backward DFS order of the leaves and its
// leaf-order schedule with chunked pops (section 3.2; pseudocode appendix,
// algorithms "Backward DFS Order" and "Dynamic Tree Attention Backward"),
// expanded into the segment calls of this library.  See include/dta.h.
#include <algorithm>
#include <cstdint>
#include <memory>
#include <new>
#include <tuple>
#include <vector>

#include "dta_internal.h"

struct dta_plan {
  std::vector<int32_t> leaf_order;
  std::vector<dta_plan_op_t> ops;
  std::vector<int64_t> call_ptr;   // [n_ops + 1] calls of op i
  std::vector<dta_plan_call_t> calls;
  int64_t n_fwd = 0, n_nograd = 0, n_chunks = 0, max_stack = 0;
};

extern "C" {

int dta_tree_plan(const dta_tree_t* tree, int64_t block, dta_plan_t** out) {
  if (!out) return DTA_ERR_INVALID_ARG;
  *out = nullptr;
  if (!tree) return DTA_ERR_INVALID_ARG;
  try {
    const int32_t n = tree->n_nodes;
    const auto& parent = tree->parent;
    std::vector<std::vector<int32_t>> kids((size_t)n);
    std::vector<int32_t> roots;
    for (int32_t u = 0; u < n; ++u) (parent[(size_t)u] < 0 ? roots : kids[(size_t)parent[(size_t)u]]).push_back(u);
    auto end_depth = [&](int32_t u) { return tree->node_start_depth[(size_t)u] + tree->seg_len[(size_t)u]; };

    // ---- backward DFS order: tails bottom-up (dfs_order is a preorder, so its
    // reverse visits children before parents), children sorted leaf first, then
    // by tail, ties by node id
    std::vector<int64_t> tail((size_t)n, 0);
    auto key = [&](int32_t u) { return std::make_tuple(kids[(size_t)u].empty() ? 0 : 1, tail[(size_t)u], u); };
    auto by_key = [&](int32_t a, int32_t b) { return key(a) < key(b); };
    for (auto it = tree->dfs_order.rbegin(); it != tree->dfs_order.rend(); ++it) {
      const int32_t v = *it;
      if (kids[(size_t)v].empty()) {
        tail[(size_t)v] = end_depth(v);
      } else {
        std::sort(kids[(size_t)v].begin(), kids[(size_t)v].end(), by_key);
        tail[(size_t)v] = tail[(size_t)kids[(size_t)v][0]];
      }
    }
    std::sort(roots.begin(), roots.end(), by_key);
    std::unique_ptr<dta_plan> owner(new dta_plan());
    dta_plan* p = owner.get();
    {
      std::vector<int32_t> stack(roots.rbegin(), roots.rend());
      while (!stack.empty()) {
        const int32_t u = stack.back();
        stack.pop_back();
        if (kids[(size_t)u].empty()) p->leaf_order.push_back(u);
        for (auto k = kids[(size_t)u].rbegin(); k != kids[(size_t)u].rend(); ++k) stack.push_back(*k);
      }
      std::reverse(p->leaf_order.begin(), p->leaf_order.end());
    }

    // ---- per leaf of that order: its depth and how many tokens of its root path
    // it shares with the leaf before and after it (the depth of the deepest common node)
    std::vector<int32_t> path_a, path_b;
    auto node_path = [&](int32_t u, std::vector<int32_t>& path) {
      path.clear();
      for (; u >= 0; u = parent[(size_t)u]) path.push_back(u);
      std::reverse(path.begin(), path.end());
    };
    auto shared_depth = [&](int32_t a, int32_t b) {
      node_path(a, path_a);
      node_path(b, path_b);
      int64_t d = 0;
      for (size_t i = 0; i < std::min(path_a.size(), path_b.size()) && path_a[i] == path_b[i]; ++i)
        d = end_depth(path_a[i]);
      return d;
    };
    struct LeafRec { int32_t leaf; int64_t depth, with_prev, with_next; };
    const size_t NL = p->leaf_order.size();
    std::vector<LeafRec> recs(NL);
    for (size_t i = 0; i < NL; ++i) {
      const int32_t s = p->leaf_order[i];
      recs[i] = LeafRec{s, end_depth(s), 0, 0};
      if (i > 0) recs[i].with_prev = recs[i - 1].with_next = shared_depth(p->leaf_order[i - 1], s);
    }

    // One splitter serves every release of the stack: depths (lo, hi] are cut at
    // evenly spaced boundaries at most `block` apart, cuts[0] = lo ... cuts[m] = hi.
    std::vector<int64_t> cuts;
    auto split = [&](int64_t lo, int64_t hi) {
      cuts.clear();
      const int64_t len = hi - lo;
      const int64_t m = (block <= 0 || len <= block) ? 1 : (len + block - 1) / block;
      for (int64_t j = 0; j <= m; ++j) cuts.push_back(lo + len * j / m);
    };
    auto emit = [&](int32_t op, int32_t leaf, int64_t lo, int64_t hi) {
      p->ops.push_back(dta_plan_op_t{op, leaf, lo, hi});
    };
    // releases depths (lo, hi] of `leaf`'s path, deepest chunk first; each chunk is
    // forwarded again (its activations are gone) and then back-propagated
    auto release = [&](int32_t leaf, int64_t lo, int64_t hi) {
      if (hi <= lo) return;
      split(lo, hi);
      for (size_t j = cuts.size() - 1; j > 0; --j) {
        emit(DTA_OP_REFWD, leaf, cuts[j - 1], cuts[j]);
        emit(DTA_OP_BWD, leaf, cuts[j - 1], cuts[j]);
        ++p->n_chunks;
      }
    };
    for (size_t i = 0; i < NL; ++i) {
      const LeafRec& r = recs[i];
      // what the stack holds beyond the part shared with this leaf goes first
      if (i > 0) release(recs[i - 1].leaf, r.with_prev, recs[i - 1].depth);
      emit(DTA_OP_FWD, r.leaf, r.with_prev, r.depth);
      ++p->n_fwd;
      p->max_stack = std::max(p->max_stack, r.depth);
      // The next release of this leaf's path, (with_next, depth], starts with its
      // deepest chunk; the keys/values below that chunk's start must be on the
      // stack without gradient state by then, which is the anchor forward (needed
      // only where this leaf's own forward started above that point).
      split(r.with_next, r.depth);
      const int64_t anchor = cuts[cuts.size() - 2];
      if (r.with_prev < anchor) {
        emit(DTA_OP_FWD_NOGRAD, r.leaf, r.with_prev, anchor);
        ++p->n_nograd;
      }
    }
    if (NL) release(recs[NL - 1].leaf, 0, recs[NL - 1].depth);

    // ---- every operation as segment calls: one per node the range touches;
    // forwards root side first, backwards leaf side first
    p->call_ptr.push_back(0);
    for (const dta_plan_op_t& op : p->ops) {
      node_path(op.leaf, path_a);
      const size_t first = p->calls.size();
      for (int32_t u : path_a) {
        const int64_t sd = tree->node_start_depth[(size_t)u];
        const int64_t a = std::max(op.lo, sd), b = std::min(op.hi, sd + tree->seg_len[(size_t)u]);
        if (a < b)
          p->calls.push_back(dta_plan_call_t{op.op, u, tree->node_offset[(size_t)u] + (a - sd),
                                             tree->node_offset[(size_t)u] + (b - sd)});
      }
      if (op.op == DTA_OP_BWD) std::reverse(p->calls.begin() + (ptrdiff_t)first, p->calls.end());
      p->call_ptr.push_back((int64_t)p->calls.size());
    }
    *out = owner.release();
  } catch (const std::bad_alloc&) {
    return DTA_ERR_ALLOC;
  }
  return DTA_OK;
}

int dta_plan_view(const dta_plan_t* plan, dta_plan_view_t* out) {
  if (!plan || !out) return DTA_ERR_INVALID_ARG;
  out->n_leaves = (int32_t)plan->leaf_order.size();
  out->leaf_order = plan->leaf_order.data();
  out->n_ops = (int64_t)plan->ops.size();
  out->ops = plan->ops.data();
  out->call_ptr = plan->call_ptr.data();
  out->n_calls = (int64_t)plan->calls.size();
  out->calls = plan->calls.data();
  out->n_fwd = plan->n_fwd;
  out->n_fwd_nograd = plan->n_nograd;
  out->n_chunks = plan->n_chunks;
  out->max_stack_tokens = plan->max_stack;
  return DTA_OK;
}

void dta_plan_destroy(dta_plan_t* plan) { delete plan; }

}  // extern "C"
