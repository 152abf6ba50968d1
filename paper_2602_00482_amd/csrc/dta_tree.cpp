// Host side of the library: tree metadata (dta_tree_build and friends) and the
// DFS tile schedule.  Integer work only; nothing here touches the GPU.
//
// The tree is the rollout prefix tree of paper section 3 (problem formulation):
// nodes are token segments, root-to-leaf paths are rollouts, and path length is
// counted in tokens.  Nodes are packed in DFS preorder (any DFS order is valid,
// section 4); in that order the tokens that can see key k form the contiguous
// range [k, kend[k]) where kend[k] is the end of the subtree of k's node, which
// is what the kernels use as their visibility mask.
#include <algorithm>
#include <cstring>
#include <limits>
#include <new>
#include <numeric>

#include "dta_internal.h"

namespace {

int build_impl(const int32_t* parent, const int32_t* seg_len, int32_t n, dta_tree* t) {
  t->n_nodes = n;
  t->parent.assign(parent, parent + n);
  t->seg_len.assign(seg_len, seg_len + n);

  int64_t total = 0;
  for (int32_t i = 0; i < n; ++i) {
    if (parent[i] < -1 || parent[i] >= n || parent[i] == i) return DTA_ERR_BAD_TREE;
    if (seg_len[i] < 1) return DTA_ERR_BAD_TREE;
    total += seg_len[i];
  }
  // leave room so that tile-padded indices still fit in int32
  if (total > (int64_t)std::numeric_limits<int32_t>::max() - 4096) return DTA_ERR_BAD_TREE;

  // children in CSR form; filling in ascending i keeps each list ascending
  std::vector<int32_t> child_ptr(n + 1, 0), child(n > 0 ? n : 1), roots;
  for (int32_t i = 0; i < n; ++i) {
    if (parent[i] >= 0) child_ptr[parent[i] + 1]++;
    else roots.push_back(i);
  }
  for (int32_t i = 0; i < n; ++i) child_ptr[i + 1] += child_ptr[i];
  {
    std::vector<int32_t> fill(child_ptr.begin(), child_ptr.end() - 1);
    for (int32_t i = 0; i < n; ++i)
      if (parent[i] >= 0) child[fill[parent[i]]++] = i;
  }

  // iterative preorder; nodes on a parent cycle are never reached from a root
  t->dfs_order.clear();
  t->dfs_order.reserve(n);
  {
    std::vector<int32_t> stack;
    for (auto it = roots.rbegin(); it != roots.rend(); ++it) stack.push_back(*it);
    while (!stack.empty()) {
      int32_t u = stack.back();
      stack.pop_back();
      t->dfs_order.push_back(u);
      for (int32_t c = child_ptr[u + 1] - 1; c >= child_ptr[u]; --c) stack.push_back(child[c]);
    }
  }
  if ((int32_t)t->dfs_order.size() != n) return DTA_ERR_BAD_TREE;

  t->node_offset.assign(n, 0);
  t->node_start_depth.assign(n, 0);
  t->subtree_tokens.assign(n, 0);
  std::vector<int32_t> depth_nodes(n, 1);
  int64_t pos = 0;
  for (int32_t r = 0; r < n; ++r) {
    int32_t u = t->dfs_order[r];
    t->node_offset[u] = pos;
    pos += seg_len[u];
    int32_t p = parent[u];
    if (p >= 0) {
      t->node_start_depth[u] = t->node_start_depth[p] + seg_len[p];
      depth_nodes[u] = depth_nodes[p] + 1;
    }
  }
  for (int32_t r = n - 1; r >= 0; --r) {
    int32_t u = t->dfs_order[r];
    t->subtree_tokens[u] += seg_len[u];
    if (parent[u] >= 0) t->subtree_tokens[parent[u]] += t->subtree_tokens[u];
  }

  // per-node ancestor key intervals, root first, merged when contiguous
  t->anc_ptr.assign(n + 1, 0);
  t->anc_seg_off.clear();
  t->anc_seg_len.clear();
  {
    std::vector<int32_t> path;
    for (int32_t u = 0; u < n; ++u) {
      path.clear();
      for (int32_t a = parent[u]; a >= 0; a = parent[a]) path.push_back(a);
      size_t first = t->anc_seg_off.size();
      for (auto it = path.rbegin(); it != path.rend(); ++it) {
        int64_t off = t->node_offset[*it], len = seg_len[*it];
        if (t->anc_seg_off.size() > first &&
            t->anc_seg_off.back() + t->anc_seg_len.back() == off) {
          t->anc_seg_len.back() += len;
        } else {
          t->anc_seg_off.push_back(off);
          t->anc_seg_len.push_back(len);
        }
      }
      t->anc_ptr[u + 1] = (int64_t)t->anc_seg_off.size();
    }
  }

  t->token_kend.resize((size_t)total);
  t->token_node.resize((size_t)total);
  for (int32_t u = 0; u < n; ++u) {
    int64_t off = t->node_offset[u];
    int32_t kend = (int32_t)(off + t->subtree_tokens[u]);
    for (int32_t j = 0; j < seg_len[u]; ++j) {
      t->token_kend[(size_t)(off + j)] = kend;
      t->token_node[(size_t)(off + j)] = u;
    }
  }

  dta_tree_info_t& inf = t->info;
  std::memset(&inf, 0, sizeof(inf));
  inf.n_nodes = n;
  inf.n_tokens = total;
  inf.n_roots = (int64_t)roots.size();
  for (int32_t u = 0; u < n; ++u) {
    int64_t len = seg_len[u], sd = t->node_start_depth[u], end = sd + len;
    bool leaf = child_ptr[u + 1] == child_ptr[u];
    inf.unique_pairs += len * sd + len * (len + 1) / 2;
    inf.rollout_tokens_full += end;
    inf.dense_pairs_full += end * (end + 1) / 2;
    if (leaf) {
      inf.n_leaves++;
      inf.rollout_tokens += end;
      inf.dense_pairs += end * (end + 1) / 2;
    }
    inf.max_path_tokens = std::max(inf.max_path_tokens, end);
    inf.max_depth_nodes = std::max<int64_t>(inf.max_depth_nodes, depth_nodes[u]);
  }
  return DTA_OK;
}

}  // namespace

namespace dta {

namespace {
// Work items are launched longest first (the hardware hands out blocks in index
// order), but only by power-of-two cost class: inside a class the DFS order is
// kept, so blocks that run at the same time stream neighbouring rows.
int64_t order_key(int64_t cost) {
  int64_t b = 0;
  while ((cost >> b) > 1) ++b;
  return b;
}
}  // namespace

// Both work lists cut the packed token order into fixed runs of bm (bn) tokens,
// whatever the node boundaries.  A tile pays for all of its padded rows anyway,
// and the keys (queries) a run of consecutive DFS tokens needs are the union of
// nested / adjacent intervals, never more than the sum over separate per-node
// tiles, so cutting at node boundaries could only add work.  What a mixed tile
// must not do is let a row see a key outside its own root path: the kernels
// mask with kend[] wherever a key interval is not visible to every row.
namespace {
// adds the chunks a query tile streams, for both chunk sizes of the forward kernel
void count_chunks(Schedule& s, const QTile& qt) {
  auto add = [&](int64_t len) {
    s.fwd_chunks64 += (len + 63) / 64;
    s.fwd_chunks128 += (len + 127) / 128;
  };
  for (int32_t i = qt.seg_begin; i < qt.seg_end; ++i) add(s.segs[(size_t)i].end - s.segs[(size_t)i].start);
  add(qt.t1 - qt.t0);
}
}  // namespace

namespace {
// copies each tile's first key interval into its record
void fill_first_intervals(Schedule& s) {
  for (QTile& t : s.q_tiles)
    t.first = t.seg_begin < t.seg_end ? s.segs[(size_t)t.seg_begin] : KeySeg{t.t0, t.t0, 0, 0};
}
}  // namespace

size_t partial_bytes(const Schedule& s) {
  return (size_t)s.n_slots * (size_t)s.hkv * 2u * (size_t)s.kv_keys * 128u * sizeof(float);
}

Schedule& get_schedule(dta_tree* tree, int bm, int bn, int hkv, int group) {
  const uint64_t key = schedule_key(bm, bn, hkv, group);
  auto it = tree->schedules.find(key);
  if (it != tree->schedules.end()) return it->second;
  // built aside and moved into the map when complete: an allocation failure half
  // way must not leave a partial schedule behind that a later call would use
  Schedule s;
  s.bm = bm;
  s.bn = bn;
  s.hkv = hkv;
  s.group = group;
  const int64_t T = tree->info.n_tokens;
  const auto& parent = tree->parent;

  // ---- query tiles (forward and dQ)
  std::vector<int64_t> cost;
  std::vector<int32_t> path;
  for (int64_t t0 = 0; t0 < T; t0 += bm) {
    int64_t t1 = std::min<int64_t>(T, t0 + bm);
    QTile qt;
    qt.t0 = (int32_t)t0;
    qt.t1 = (int32_t)t1;
    qt.seg_begin = (int32_t)s.segs.size();
    int32_t u0 = tree->token_node[(size_t)t0];
    path.clear();
    for (int32_t a = parent[u0]; a >= 0; a = parent[a]) path.push_back(a);
    int64_t keys = t1 - t0;
    auto add = [&](int64_t start, int64_t end, int64_t kend) {
      int32_t full = kend >= t1 ? 1 : 0;
      if ((int32_t)s.segs.size() > qt.seg_begin && s.segs.back().end == start &&
          s.segs.back().full == full) {
        s.segs.back().end = (int32_t)end;
      } else {
        s.segs.push_back(KeySeg{(int32_t)start, (int32_t)end, full, 0});
      }
      keys += end - start;
    };
    for (auto a = path.rbegin(); a != path.rend(); ++a) {
      int64_t off = tree->node_offset[*a];
      add(off, off + tree->seg_len[*a], off + tree->subtree_tokens[*a]);
    }
    int64_t off0 = tree->node_offset[u0];
    if (t0 > off0) add(off0, t0, off0 + tree->subtree_tokens[u0]);
    qt.seg_end = (int32_t)s.segs.size();
    s.q_tiles.push_back(qt);
    cost.push_back(keys);
    s.fwd_tile_pairs += keys * bm;
    count_chunks(s, qt);
  }
  {
    std::vector<size_t> order(s.q_tiles.size());
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(),
                     [&](size_t a, size_t b) { return order_key(cost[a]) > order_key(cost[b]); });
    std::vector<QTile> sorted;
    sorted.reserve(order.size());
    for (size_t i : order) sorted.push_back(s.q_tiles[i]);
    s.q_tiles.swap(sorted);
  }
  fill_first_intervals(s);

  // ---- key tiles (dK/dV): runs of at most bn consecutive packed keys.  A block
  // walks the union of the query ranges of its keys, [k0, max kend), so a run that
  // mixes keys of small nodes with disjoint or much shorter ranges (leaves of a
  // forest of short segments) keeps its four waves waiting for each other.  The
  // cuts are therefore chosen, by dynamic programming over the packed order, to
  // minimise the summed block time  sum over tiles of (fixed cost + walk steps):
  // a tile either ends at a node boundary or is bn keys long.  On trees of long
  // segments this reproduces the plain cut every bn keys.
  auto cut_key_tiles = [&](int keys) {
    cost.clear();
    s.kv_tiles.clear();
    s.bwd_tile_pairs = 0;
    s.kv_keys = keys;
    constexpr int64_t kChunkRows = 64, kFixedSteps = 7;   // a block's prologue and epilogue cost about 7 walk steps
    const int64_t INF = std::numeric_limits<int64_t>::max() / 4;
    std::vector<int64_t> best((size_t)T + 1, INF);
    std::vector<int32_t> from((size_t)T + 1, -1);
    best[0] = 0;
    const std::vector<int32_t>& order = tree->dfs_order;
    size_t rank_of_q = 0;   // DFS rank of the node that holds position q
    for (int64_t q = 0; q < T; ++q) {
      while (tree->node_offset[(size_t)order[rank_of_q]] + tree->seg_len[(size_t)order[rank_of_q]] <= q) ++rank_of_q;
      const int64_t base = best[(size_t)q];
      if (base == INF) continue;
      int64_t mx = 0;
      const int64_t limit = std::min<int64_t>(T, q + keys);
      for (size_t r = rank_of_q; r < order.size(); ++r) {
        const int32_t u = order[r];
        const int64_t off = tree->node_offset[(size_t)u];
        if (off >= limit) break;
        mx = std::max(mx, off + tree->subtree_tokens[(size_t)u]);
        // the tile ends with this node, or after bn keys inside it
        const int64_t p = std::min(limit, off + tree->seg_len[(size_t)u]);
        const int64_t c = base + kFixedSteps + (mx - q + kChunkRows - 1) / kChunkRows * group;
        if (c < best[(size_t)p]) {   // (on ties the earlier start, visited first, stays)
          best[(size_t)p] = c;
          from[(size_t)p] = (int32_t)q;
        }
      }
    }
    std::vector<int64_t> cuts;
    for (int64_t p = T; p > 0; p = from[(size_t)p]) cuts.push_back(p);
    cuts.push_back(0);
    std::reverse(cuts.begin(), cuts.end());
    for (size_t i = 0; i + 1 < cuts.size(); ++i) {
      const int64_t k0 = cuts[i], k1 = cuts[i + 1];
      int32_t mx = 0, mn = std::numeric_limits<int32_t>::max();
      for (int64_t k = k0; k < k1; ++k) {
        mx = std::max(mx, tree->token_kend[(size_t)k]);
        mn = std::min(mn, tree->token_kend[(size_t)k]);
      }
      s.kv_tiles.push_back(KvTile{(int32_t)k0, (int32_t)k1, mx, mn, (int32_t)k0, {0, 0, 0}});
      cost.push_back(mx - k0);
      s.bwd_tile_pairs += (int64_t)(mx - k0) * keys;
    }
    std::vector<size_t> by_cost(s.kv_tiles.size());
    std::iota(by_cost.begin(), by_cost.end(), 0);
    std::stable_sort(by_cost.begin(), by_cost.end(),
                     [&](size_t a, size_t b) { return order_key(cost[a]) > order_key(cost[b]); });
    std::vector<KvTile> sorted;
    sorted.reserve(by_cost.size());
    for (size_t i : by_cost) sorted.push_back(s.kv_tiles[i]);
    s.kv_tiles.swap(sorted);
  };
  cut_key_tiles(bn);

  // ---- dK/dV launch items: cut the longest walks so that no block becomes the
  // critical path.  The chip holds `resident` blocks of this kernel (512 of four
  // waves, 256 of eight); a piece of a cut walk is at most 2/3 of the work one of
  // those slots gets on average, and only walks longer than that are cut.  Finer pieces balance no better and cost
  // more (every item pays its prologue, the masked steps of its diagonal and,
  // when cut, fp32 partial sums): with pieces of 1/4 of a slot's share the dK/dV
  // launch of the 16-response tree (configuration 2) was 5 % slower, coarser
  // ones (a whole share) let a single piece decide the end of the launch.
  // A launch with at least 8 rounds of items runs as resident blocks that draw
  // the items from queues and take over work from slower XCDs (see the kernel);
  // what they can take over is whole items, so where the items are long the
  // walks are cut four times finer (1/6 of a share): measured on the deep tree with its 128
  // root tiles of 17 344 steps per kv head, 3 % faster than uncut walks handed
  // out block by block, while the same queues over uncut walks are 2.5 % slower.
  auto cut_items = [&](int64_t target_items) {
    constexpr int kChunkRows = 64;
    s.kv_items.clear();
    s.kv_reduce.clear();
    s.n_slots = 0;
    s.kv_item_iters = 0;
    auto iters_of = [&](const KvTile& t) {
      return (int64_t)((t.q_end - t.k0 + kChunkRows - 1) / kChunkRows) * group;
    };
    int64_t total = 0;
    for (const KvTile& t : s.kv_tiles) total += iters_of(t);
    const int64_t target = std::max<int64_t>(32, (total * hkv + target_items - 1) / target_items);
    std::vector<int64_t> icost;
    for (const KvTile& t : s.kv_tiles) {
      const int64_t iters = iters_of(t);
      int64_t nparts = 1;
      if (iters > target) nparts = (iters + target - 1) / target;
      if (nparts > 1) s.kv_reduce.push_back(KvReduce{t.k0, t.k1, (int32_t)s.n_slots, (int32_t)nparts});
      for (int64_t p = 0; p < nparts; ++p) {
        KvItem it{t.k0, t.k1, t.q_end, t.q_full_end, (int32_t)(iters * p / nparts),
                  (int32_t)(iters * (p + 1) / nparts), nparts > 1 ? (int32_t)(s.n_slots + p) : -1,
                  t.q_begin};
        s.kv_items.push_back(it);
        icost.push_back(it.it_end - it.it_begin);
        s.kv_item_iters += it.it_end - it.it_begin;
      }
      if (nparts > 1) s.n_slots += nparts;
    }
    std::vector<size_t> order(s.kv_items.size());
    std::iota(order.begin(), order.end(), 0);
    // same cost class: parts that cover the same slice of the walk next to each
    // other (they stream the same query rows), then DFS order
    std::stable_sort(order.begin(), order.end(), [&](size_t a, size_t b) {
      const int64_t ka = order_key(icost[a]), kb = order_key(icost[b]);
      if (ka != kb) return ka > kb;
      return s.kv_items[a].it_begin < s.kv_items[b].it_begin;
    });
    std::vector<KvItem> sorted;
    sorted.reserve(order.size());
    for (size_t i : order) sorted.push_back(s.kv_items[i]);
    s.kv_items.swap(sorted);
  };
  // items for a launch shape that keeps `resident` blocks on the chip
  auto cut_for = [&](int64_t resident) {
    cut_items(resident * 3 / 2);
    s.kv_queues = (int64_t)s.kv_items.size() * hkv >= 8 * resident;
    // (forests of short items, under 384 steps on average, have nothing to gain from
    // finer pieces and would only pay for more partial sums)
    if (s.kv_queues && s.kv_item_iters > 384 * (int64_t)s.kv_items.size()) cut_items(resident * 6);
  };
  cut_for(2 * (int64_t)kNumCUs);
  constexpr int64_t kWideMinIters = 256;
  if (bn == 128 && wide_key_tiles && s.kv_item_iters > kWideMinIters * (int64_t)s.kv_tiles.size()) {
    // Long walks (256 steps per 128-key tile and more): tiles of 256 keys for the
    // eight-wave form of the kernel, one block per CU.  Every streamed 64-row
    // chunk then meets twice the keys, which halves the copies L2 -> LDS per
    // product; the steps of a walk, and so the piece lengths in steps, stay what
    // they are with 128 keys.  Measured on MI355X (dK/dV launch): the deep tree
    // -3.8 %, the multi-turn forest (374 steps per tile) -2 %, 16 long answers
    // -1.3 %; forests of short segments (130 steps per tile and fewer) take the
    // same time either way (+-0.5 %) with more of the block's waves idle, so
    // they stay on the two-blocks-per-CU form.
    cut_key_tiles(256);
    cut_for((int64_t)kNumCUs);
  }
  return tree->schedules.emplace(key, std::move(s)).first->second;
}

Schedule& get_segment_schedule(dta_tree* tree, int bm, int bn, int hkv, int group,
                               int64_t t_begin, int64_t t_end) {
  const std::array<uint64_t, 3> key = {schedule_key(bm, bn, hkv, group), (uint64_t)t_begin,
                                       (uint64_t)t_end};
  auto it = tree->segment_schedules.find(key);
  if (it != tree->segment_schedules.end()) {
    it->second.last_used = ++tree->use_counter;
    return it->second;
  }
  Schedule s;   // built aside, see get_schedule
  s.last_used = ++tree->use_counter;
  s.bm = bm;
  s.bn = bn;
  s.kv_keys = bn;
  s.hkv = hkv;
  s.group = group;

  // The keys the rows see: the segments of the ancestors (root first), then the
  // node's own tokens before t_begin; every row sees all of them.  Adjacent
  // pieces are merged.
  const int32_t u0 = tree->token_node[(size_t)t_begin];
  std::vector<int32_t> path;
  for (int32_t a = tree->parent[u0]; a >= 0; a = tree->parent[a]) path.push_back(a);
  std::vector<KeySeg> prefix;
  auto add = [&](int64_t start, int64_t end) {
    if (start >= end) return;
    if (!prefix.empty() && prefix.back().end == start) prefix.back().end = (int32_t)end;
    else prefix.push_back(KeySeg{(int32_t)start, (int32_t)end, 1, 0});
  };
  for (auto a = path.rbegin(); a != path.rend(); ++a) {
    const int64_t off = tree->node_offset[*a];
    add(off, off + tree->seg_len[*a]);
  }
  add(tree->node_offset[u0], t_begin);
  int64_t prefix_keys = 0;
  for (const KeySeg& ks : prefix) prefix_keys += ks.end - ks.start;

  // ---- query tiles over the rows; a tile also sees the rows before it
  for (int64_t t0 = t_begin; t0 < t_end; t0 += bm) {
    const int64_t t1 = std::min<int64_t>(t_end, t0 + bm);
    QTile qt;
    qt.t0 = (int32_t)t0;
    qt.t1 = (int32_t)t1;
    qt.seg_begin = (int32_t)s.segs.size();
    for (const KeySeg& ks : prefix) s.segs.push_back(ks);
    if (t0 > t_begin) {
      if (!prefix.empty() && s.segs.back().end == t_begin) s.segs.back().end = (int32_t)t0;
      else s.segs.push_back(KeySeg{(int32_t)t_begin, (int32_t)t0, 1, 0});
    }
    qt.seg_end = (int32_t)s.segs.size();
    s.q_tiles.push_back(qt);
    s.fwd_tile_pairs += (prefix_keys + (t1 - t_begin)) * bm;
    count_chunks(s, qt);
  }
  std::reverse(s.q_tiles.begin(), s.q_tiles.end());   // the last tile sees the most keys
  fill_first_intervals(s);

  // ---- key tiles: the prefix pieces (walk = all rows, no mask beyond padding),
  // then the rows themselves (causal)
  auto add_tiles = [&](int64_t start, int64_t end, bool own) {
    for (int64_t k0 = start; k0 < end; k0 += bn) {
      const int64_t k1 = std::min<int64_t>(end, k0 + bn);
      const int64_t qb = own ? k0 : t_begin;
      s.kv_tiles.push_back(KvTile{(int32_t)k0, (int32_t)k1, (int32_t)t_end, (int32_t)t_end,
                                  (int32_t)qb, {0, 0, 0}});
      s.bwd_tile_pairs += (t_end - qb) * bn;
    }
  };
  add_tiles(t_begin, t_end, true);
  for (const KeySeg& ks : prefix) add_tiles(ks.start, ks.end, false);
  constexpr int kChunkRows = 64;
  for (const KvTile& t : s.kv_tiles) {
    const int64_t iters = (int64_t)((t.q_end - t.q_begin + kChunkRows - 1) / kChunkRows) * group;
    s.kv_items.push_back(KvItem{t.k0, t.k1, t.q_end, t.q_full_end, 0, (int32_t)iters, -1, t.q_begin});
    s.kv_item_iters += iters;
  }
  // keep the cache bounded: drop the least recently used schedule; its device
  // block may still be read by a launch in flight, so it is only set aside here
  // (whoever uploads into it next orders that copy behind the tree's launches)
  if (tree->segment_schedules.size() >= max_segment_schedules(tree->n_nodes)) {
    auto lru = tree->segment_schedules.begin();
    for (auto e = tree->segment_schedules.begin(); e != tree->segment_schedules.end(); ++e)
      if (e->second.last_used < lru->second.last_used) lru = e;
    if (lru->second.d_blob)
      tree->retired.push_back(dta_tree::RetiredBlock{lru->second.d_blob, lru->second.d_blob_cap, lru->second.device});
    tree->segment_schedules.erase(lru);
  }
  return tree->segment_schedules.emplace(key, std::move(s)).first->second;
}

int validate_params(const dta_attn_params_t* p) {
  if (!p) return DTA_ERR_INVALID_ARG;
  if (p->n_q_heads < 1 || p->n_kv_heads < 1) return DTA_ERR_INVALID_ARG;
  // finite and nonzero (the bf16 backward divides by it)
  if (!(p->softmax_scale == p->softmax_scale) || p->softmax_scale == 0.f ||
      p->softmax_scale - p->softmax_scale != 0.f)
    return DTA_ERR_INVALID_ARG;
  if (p->n_q_heads % p->n_kv_heads != 0) return DTA_ERR_UNSUPPORTED;
  if (p->dtype == DTA_F32) {
    if (p->head_dim != 64 && p->head_dim != 128) return DTA_ERR_UNSUPPORTED;
  } else if (p->dtype == DTA_BF16) {
    if (p->head_dim != 64 && p->head_dim != 128) return DTA_ERR_UNSUPPORTED;
  } else {
    return DTA_ERR_UNSUPPORTED;
  }
  return DTA_OK;
}

int choose_tiles(const dta_attn_params_t* p, TileChoice* out) {
  int st = validate_params(p);
  if (st != DTA_OK) return st;
  int G = p->n_q_heads / p->n_kv_heads;
  if (p->dtype == DTA_F32) {
    out->bm = 64;
    out->bn = 64;
    out->hb = 1;
    out->hblocks = G;
  } else {
    // eight waves per block: hb q heads of the group x (8/hb) 32-row query blocks
    int hb = (G % 8 == 0) ? 8 : (G % 4 == 0) ? 4 : (G % 2 == 0) ? 2 : 1;
    out->hb = hb;
    out->hblocks = G / hb;
    out->bm = 32 * (8 / hb);
    out->bn = 128;
  }
  return DTA_OK;
}

}  // namespace dta

extern "C" {

int dta_tree_build(const int32_t* parent, const int32_t* seg_len, int32_t n_nodes,
                   uint32_t flags, dta_tree_t** out) {
  if (out) *out = nullptr;
  if (!parent || !seg_len || !out || n_nodes < 1 || flags != 0) return DTA_ERR_INVALID_ARG;
  dta_tree* t = new (std::nothrow) dta_tree();
  if (!t) return DTA_ERR_ALLOC;
  int st;
  try {
    st = build_impl(parent, seg_len, n_nodes, t);
  } catch (const std::bad_alloc&) {
    st = DTA_ERR_ALLOC;
  }
  if (st != DTA_OK) {
    delete t;
    return st;
  }
  *out = t;
  return DTA_OK;
}

int dta_tree_info(const dta_tree_t* tree, dta_tree_info_t* out) {
  if (!tree || !out) return DTA_ERR_INVALID_ARG;
  *out = tree->info;
  return DTA_OK;
}

int dta_tree_layout(const dta_tree_t* tree, dta_tree_layout_t* out) {
  if (!tree || !out) return DTA_ERR_INVALID_ARG;
  out->dfs_order = tree->dfs_order.data();
  out->node_offset = tree->node_offset.data();
  out->node_start_depth = tree->node_start_depth.data();
  out->subtree_tokens = tree->subtree_tokens.data();
  out->anc_ptr = tree->anc_ptr.data();
  out->anc_seg_off = tree->anc_seg_off.data();
  out->anc_seg_len = tree->anc_seg_len.data();
  out->token_kend = tree->token_kend.data();
  return DTA_OK;
}

int dta_tree_schedule_info(dta_tree_t* tree, const dta_attn_params_t* params,
                           dta_schedule_info_t* out) {
  if (!tree || !out) return DTA_ERR_INVALID_ARG;
  dta::TileChoice tc;
  int st = dta::choose_tiles(params, &tc);
  if (st != DTA_OK) return st;
  try {
    std::lock_guard<std::mutex> lock(tree->mu);
    dta::Schedule& s = dta::get_schedule(tree, tc.bm, tc.bn, params->n_kv_heads,
                                         params->n_q_heads / params->n_kv_heads);
    out->fwd_q_tile_tokens = tc.bm;
    out->fwd_work_items = (int64_t)s.q_tiles.size();
    out->fwd_tile_pairs = s.fwd_tile_pairs;
    out->bwd_kv_tile_tokens = s.kv_keys;
    out->bwd_work_items = (int64_t)s.kv_items.size();
    out->bwd_tile_pairs = s.bwd_tile_pairs;
    out->metadata_bytes =
        (int64_t)(tree->token_kend.size() * sizeof(int32_t) + s.q_tiles.size() * sizeof(dta::QTile) +
                  s.segs.size() * sizeof(dta::KeySeg) + s.kv_tiles.size() * sizeof(dta::KvTile) +
                  s.kv_items.size() * sizeof(dta::KvItem) + s.kv_reduce.size() * sizeof(dta::KvReduce));
  } catch (const std::bad_alloc&) {
    return DTA_ERR_ALLOC;
  }
  return DTA_OK;
}

const char* dta_status_string(int status) {
  switch (status) {
    case DTA_OK: return "DTA_OK";
    case DTA_ERR_INVALID_ARG: return "DTA_ERR_INVALID_ARG";
    case DTA_ERR_BAD_TREE: return "DTA_ERR_BAD_TREE";
    case DTA_ERR_UNSUPPORTED: return "DTA_ERR_UNSUPPORTED";
    case DTA_ERR_ALLOC: return "DTA_ERR_ALLOC";
    case DTA_ERR_HIP: return "DTA_ERR_HIP";
    case DTA_ERR_WORKSPACE: return "DTA_ERR_WORKSPACE";
    default: return "DTA_ERR_UNKNOWN";
  }
}

}  // extern "C"
