// Host side, integer only: from rollout token sequences to the prefix tree the
// attention calls work on, and the paper's load-balanced DFS-contiguous
// partitioning of the rollouts (section 4; pseudocode appendix, algorithm
// "Load-Balanced DFS-Contiguous Partitioning").  See include/dta.h.
#include <algorithm>
#include <cstdint>
#include <new>
#include <numeric>
#include <vector>

#include "dta.h"

struct dta_rollouts {
  int32_t n_seqs = 0;
  std::vector<int32_t> order;      // lexicographic order of the input sequences
  std::vector<int64_t> len;        // length of the i-th sequence of that order
  std::vector<int64_t> lcp;        // common prefix with its predecessor in that order
  std::vector<int32_t> parent, seg_len, tokens, seq_node;
};

namespace {

struct Node {
  int32_t parent;          // temporary id, -1 = root level
  int64_t start, end;      // token depths [start, end) on the path
  int32_t rep;             // a sorted-sequence index whose tokens spell the segment
  std::vector<int32_t> kids;
};

}  // namespace

extern "C" {

int dta_rollouts_build(const int32_t* tokens, const int64_t* seq_offsets, int32_t n_seqs,
                       dta_rollouts_t** out) {
  if (!out) return DTA_ERR_INVALID_ARG;
  *out = nullptr;
  if (!tokens || !seq_offsets || n_seqs < 1) return DTA_ERR_INVALID_ARG;
  if (seq_offsets[0] != 0) return DTA_ERR_INVALID_ARG;
  for (int32_t i = 0; i < n_seqs; ++i)
    if (seq_offsets[i + 1] <= seq_offsets[i]) return DTA_ERR_INVALID_ARG;   // empty or decreasing
  try {
    auto* r = new dta_rollouts();
    r->n_seqs = n_seqs;
    auto seq = [&](int32_t i) { return tokens + seq_offsets[i]; };
    auto length = [&](int32_t i) { return seq_offsets[i + 1] - seq_offsets[i]; };
    // lexicographic order: a proper prefix first, equal sequences in input order
    r->order.resize((size_t)n_seqs);
    std::iota(r->order.begin(), r->order.end(), 0);
    std::stable_sort(r->order.begin(), r->order.end(), [&](int32_t a, int32_t b) {
      return std::lexicographical_compare(seq(a), seq(a) + length(a), seq(b), seq(b) + length(b));
    });
    r->len.resize((size_t)n_seqs);
    r->lcp.assign((size_t)n_seqs, 0);
    for (int32_t i = 0; i < n_seqs; ++i) {
      r->len[(size_t)i] = length(r->order[(size_t)i]);
      if (i > 0) {
        const int32_t* a = seq(r->order[(size_t)i - 1]);
        const int32_t* b = seq(r->order[(size_t)i]);
        const int64_t n = std::min(r->len[(size_t)i - 1], r->len[(size_t)i]);
        int64_t l = 0;
        while (l < n && a[l] == b[l]) ++l;
        r->lcp[(size_t)i] = l;
      }
    }

    // Compressed trie by one pass over the sorted sequences: the stack is the
    // root-to-node path of the previous sequence; the next sequence leaves it
    // at depth lcp, where a node is split if the depth falls inside it.
    std::vector<Node> nodes;
    std::vector<int32_t> roots, stack, end_node((size_t)n_seqs);
    for (int32_t i = 0; i < n_seqs; ++i) {
      const int64_t l = r->lcp[(size_t)i], n = r->len[(size_t)i];
      while (!stack.empty() && nodes[(size_t)stack.back()].start >= l) stack.pop_back();
      if (!stack.empty() && nodes[(size_t)stack.back()].end > l) {
        // split: a new upper node [start, l) takes the old node's place; the old
        // node keeps its id (so sequences that end at it stay right), its
        // children, and becomes the lower part [l, end)
        const int32_t x = stack.back();
        Node top{nodes[(size_t)x].parent, nodes[(size_t)x].start, l, nodes[(size_t)x].rep, {x}};
        const int32_t t = (int32_t)nodes.size();
        std::vector<int32_t>& sibs = top.parent < 0 ? roots : nodes[(size_t)top.parent].kids;
        *std::find(sibs.begin(), sibs.end(), x) = t;
        nodes.push_back(top);
        nodes[(size_t)x].parent = t;
        nodes[(size_t)x].start = l;
        stack.back() = t;
      }
      if (n > l) {
        const int32_t par = stack.empty() ? -1 : stack.back();
        const int32_t u = (int32_t)nodes.size();
        nodes.push_back(Node{par, l, n, i, {}});
        (par < 0 ? roots : nodes[(size_t)par].kids).push_back(u);
        stack.push_back(u);
      }
      end_node[(size_t)i] = stack.back();   // n == l: the same sequence again
    }

    // canonical numbering: DFS preorder, children in creation order (ascending
    // first token, because the sequences came sorted)
    const size_t M = nodes.size();
    std::vector<int32_t> new_id(M, -1);
    r->parent.reserve(M);
    r->seg_len.reserve(M);
    std::vector<int32_t> work(roots.rbegin(), roots.rend());
    int64_t total = 0;
    while (!work.empty()) {
      const int32_t u = work.back();
      work.pop_back();
      const Node& nd = nodes[(size_t)u];
      new_id[(size_t)u] = (int32_t)r->parent.size();
      r->parent.push_back(nd.parent < 0 ? -1 : new_id[(size_t)nd.parent]);
      if (nd.end - nd.start > 0x7fffffff) { delete r; return DTA_ERR_BAD_TREE; }
      r->seg_len.push_back((int32_t)(nd.end - nd.start));
      total += nd.end - nd.start;
      if (total > 0x7fffffff) { delete r; return DTA_ERR_BAD_TREE; }   // token count overflow
      const int32_t* s = seq(r->order[(size_t)nd.rep]);
      r->tokens.insert(r->tokens.end(), s + nd.start, s + nd.end);
      for (auto k = nd.kids.rbegin(); k != nd.kids.rend(); ++k) work.push_back(*k);
    }
    r->seq_node.resize((size_t)n_seqs);
    for (int32_t i = 0; i < n_seqs; ++i)
      r->seq_node[(size_t)r->order[(size_t)i]] = new_id[(size_t)end_node[(size_t)i]];
    *out = r;
  } catch (const std::bad_alloc&) {
    return DTA_ERR_ALLOC;
  }
  return DTA_OK;
}

int dta_rollouts_view(const dta_rollouts_t* r, dta_rollouts_view_t* out) {
  if (!r || !out) return DTA_ERR_INVALID_ARG;
  out->n_seqs = r->n_seqs;
  out->n_nodes = (int32_t)r->parent.size();
  out->n_tokens = (int64_t)r->tokens.size();
  out->parent = r->parent.data();
  out->seg_len = r->seg_len.data();
  out->tokens = r->tokens.data();
  out->seq_node = r->seq_node.data();
  out->order = r->order.data();
  out->lcp = r->lcp.data();
  return DTA_OK;
}

int dta_rollouts_partition(const dta_rollouts_t* r, int32_t k, int32_t* group_begin,
                           int64_t* group_cost) {
  if (!r || !group_begin || !group_cost) return DTA_ERR_INVALID_ARG;
  const int32_t N = r->n_seqs;
  if (k < 1 || k > N) return DTA_ERR_INVALID_ARG;
  const std::vector<int64_t>& len = r->len;
  const std::vector<int64_t>& lcp = r->lcp;
  try {
    std::vector<int32_t> cuts;   // first index of every group
    // greedy scan: can the order be cut into at most k groups of cost <= tau?
    auto feasible = [&](int64_t tau) {
      cuts.clear();
      cuts.push_back(0);
      int64_t c = len[0];
      for (int32_t i = 1; i < N; ++i) {
        const int64_t delta = len[(size_t)i] - lcp[(size_t)i];   // new tree tokens added by pi_i
        if (c + delta > tau) {
          cuts.push_back(i);
          c = len[(size_t)i];
        } else {
          c += delta;
        }
      }
      return (int32_t)cuts.size() <= k;
    };
    int64_t L = *std::max_element(len.begin(), len.end());
    int64_t R = len[0];
    for (int32_t i = 1; i < N; ++i) R += len[(size_t)i] - lcp[(size_t)i];
    while (L < R) {
      const int64_t tau = (L + R) / 2;
      if (feasible(tau)) R = tau;
      else L = tau + 1;
    }
    feasible(L);
    // split non-singleton groups (the first one, after its first element) until there are k
    while ((int32_t)cuts.size() < k) {
      size_t j = 0;
      while ((j + 1 < cuts.size() ? cuts[j + 1] : N) - cuts[j] < 2) ++j;
      cuts.insert(cuts.begin() + (ptrdiff_t)j + 1, cuts[j] + 1);
    }
    for (int32_t g = 0; g < k; ++g) {
      const int32_t a = cuts[(size_t)g], b = g + 1 < k ? cuts[(size_t)g + 1] : N;
      group_begin[g] = a;
      int64_t c = len[(size_t)a];
      for (int32_t i = a + 1; i < b; ++i) c += len[(size_t)i] - lcp[(size_t)i];
      group_cost[g] = c;
    }
    group_begin[k] = N;
  } catch (const std::bad_alloc&) {
    return DTA_ERR_ALLOC;
  }
  return DTA_OK;
}

void dta_rollouts_destroy(dta_rollouts_t* r) { delete r; }

}  // extern "C"
