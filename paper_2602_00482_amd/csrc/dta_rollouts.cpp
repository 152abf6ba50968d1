// Host side, integer only: from rollout token sequences to the prefix tree the
// attention calls work on, and the paper's load-balanced DFS-contiguous
// partitioning of the rollouts (section 4; pseudocode appendix, algorithm
// "Load-Balanced DFS-Contiguous Partitioning").  See include/dta.h.
#include <algorithm>
#include <cstdint>
#include <memory>
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
    std::unique_ptr<dta_rollouts> owner(new dta_rollouts());
    dta_rollouts* r = owner.get();
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
      if (nd.end - nd.start > 0x7fffffff) return DTA_ERR_BAD_TREE;
      r->seg_len.push_back((int32_t)(nd.end - nd.start));
      total += nd.end - nd.start;
      if (total > 0x7fffffff) return DTA_ERR_BAD_TREE;   // token count overflow
      const int32_t* s = seq(r->order[(size_t)nd.rep]);
      r->tokens.insert(r->tokens.end(), s + nd.start, s + nd.end);
      for (auto k = nd.kids.rbegin(); k != nd.kids.rend(); ++k) work.push_back(*k);
    }
    r->seq_node.resize((size_t)n_seqs);
    for (int32_t i = 0; i < n_seqs; ++i)
      r->seq_node[(size_t)r->order[(size_t)i]] = new_id[(size_t)end_node[(size_t)i]];
    *out = owner.release();
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
  try {
    // grown[i] = tree tokens of the first i sequences of the order taken together
    // (a sequence adds what it does not share with its predecessor).  A group
    // [a, b) rebuilt on its own needs the shared part of its first sequence as
    // well: cost(a, b) = lcp[a] + grown[b] - grown[a].
    std::vector<int64_t> grown((size_t)N + 1, 0);
    for (int32_t i = 0; i < N; ++i)
      grown[(size_t)i + 1] = grown[(size_t)i] + (r->len[(size_t)i] - r->lcp[(size_t)i]);
    auto cost = [&](int32_t a, int32_t b) {
      return r->lcp[(size_t)a] + grown[(size_t)b] - grown[(size_t)a];
    };
    // Filling groups greedily under a cost bound: a group that starts at a runs up
    // to the last b with cost(a, b) <= bound, found by bisection in the
    // non-decreasing `grown`.  Returns the number of groups, at most `limit` + 1.
    std::vector<int32_t> starts;
    auto fill = [&](int64_t bound, int32_t limit) {
      starts.clear();
      for (int32_t a = 0; a < N && (int32_t)starts.size() <= limit;) {
        starts.push_back(a);
        const int64_t reach = bound - r->lcp[(size_t)a] + grown[(size_t)a];
        const int32_t b = (int32_t)(std::upper_bound(grown.begin() + a + 1, grown.end(), reach) - grown.begin()) - 1;
        a = std::max(b, a + 1);   // the bound is never below the longest sequence, so b > a
      }
      return (int32_t)starts.size();
    };
    // smallest bound that k groups can meet: between the longest sequence (every
    // group holds at least one whole sequence) and the whole tree
    int64_t lo = *std::max_element(r->len.begin(), r->len.end()), hi = grown[(size_t)N];
    while (lo < hi) {
      const int64_t mid = lo + (hi - lo) / 2;
      if (fill(mid, k) <= k) hi = mid;
      else lo = mid + 1;
    }
    int32_t spare = k - fill(lo, k);
    // fewer groups than asked for: single sequences are taken off the front of
    // the first groups that have more than one (this is the paper's "split any
    // non-singleton interval", always applied to the first one after its first
    // sequence)
    int32_t g = 0;
    for (size_t j = 0; j < starts.size(); ++j) {
      const int32_t a = starts[j], b = j + 1 < starts.size() ? starts[j + 1] : N;
      const int32_t peel = std::min(spare, b - a - 1);
      for (int32_t t = 0; t < peel; ++t) group_begin[g++] = a + t;
      group_begin[g++] = a + peel;
      spare -= peel;
    }
    group_begin[k] = N;
    for (g = 0; g < k; ++g) group_cost[g] = cost(group_begin[g], group_begin[g + 1]);
  } catch (const std::bad_alloc&) {
    return DTA_ERR_ALLOC;
  }
  return DTA_OK;
}

void dta_rollouts_destroy(dta_rollouts_t* r) { delete r; }

}  // extern "C"
