// Host side, integer only: the paper's backward DFS order of the leaves and its
// leaf-order schedule with chunked pops (section 3.2; pseudocode appendix,
// algorithms "Backward DFS Order" and "Dynamic Tree Attention Backward"),
// expanded into the segment calls of this library.  See include/dta.h.
#include <algorithm>
#include <cstdint>
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
    auto* p = new dta_plan();
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

    // ---- the schedule over depth ranges of the current leaf's root path
    std::vector<int32_t> path_a, path_b;
    auto node_path = [&](int32_t u, std::vector<int32_t>& path) {
      path.clear();
      for (; u >= 0; u = parent[(size_t)u]) path.push_back(u);
      std::reverse(path.begin(), path.end());
    };
    auto lcp = [&](int32_t a, int32_t b) {
      node_path(a, path_a);
      node_path(b, path_b);
      int64_t l = 0;
      for (size_t i = 0; i < std::min(path_a.size(), path_b.size()) && path_a[i] == path_b[i]; ++i)
        l = end_depth(path_a[i]);
      return l;
    };
    auto emit = [&](int32_t op, int32_t leaf, int64_t lo, int64_t hi) {
      p->ops.push_back(dta_plan_op_t{op, leaf, lo, hi});
    };
    auto pop_by_chunk = [&](int32_t leaf, int64_t hi, int64_t lo) {
      const int64_t len = hi - lo;
      if (len <= 0) return;
      const int64_t m = (block <= 0 || block >= len) ? 1 : (len + block - 1) / block;
      for (int64_t j = m - 1; j >= 0; --j) {   // evenly spaced boundaries, last chunk first
        const int64_t a = lo + len * j / m, b = lo + len * (j + 1) / m;
        emit(DTA_OP_REFWD, leaf, a, b);
        emit(DTA_OP_BWD, leaf, a, b);
        ++p->n_chunks;
      }
    };
    int64_t l_backward = 0;
    const size_t NL = p->leaf_order.size();
    for (size_t i = 0; i < NL; ++i) {
      const int32_t s = p->leaf_order[i];
      const int64_t len = end_depth(s);
      int64_t l_lcp = 0;
      if (i > 0) {
        l_lcp = lcp(p->leaf_order[i - 1], s);
        pop_by_chunk(p->leaf_order[i - 1], l_backward, l_lcp);
      }
      emit(DTA_OP_FWD, s, l_lcp, len);
      ++p->n_fwd;
      p->max_stack = std::max(p->max_stack, len);
      l_backward = len;
      int64_t l_anchor = i + 1 < NL ? lcp(s, p->leaf_order[i + 1]) : 0;
      const int64_t p_pop = len - l_anchor;
      if (block > 0 && p_pop >= block) {
        const int64_t m = (p_pop + block - 1) / block;
        l_anchor = len - (p_pop + m - 1) / m;
      }
      if (l_lcp < l_anchor) {
        emit(DTA_OP_FWD_NOGRAD, s, l_lcp, l_anchor);
        ++p->n_nograd;
      }
    }
    if (NL) pop_by_chunk(p->leaf_order[NL - 1], l_backward, 0);

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
    *out = p;
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
