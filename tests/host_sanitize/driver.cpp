// Test driver for the pure-host sources of the library (tree metadata and tile
// schedule, leaf-order plan, rollout prefix tree and partitioning), meant to be
// built with -fsanitize=address,undefined and run by tests/test_host_sanitize.py.
// Reads cases from stdin, calls the C ABI, prints what it got as text; the
// Python side compares the text with the regular library's answers.  Input:
//   tree <n> parent[n] seg_len[n] <n_cfg> {Hq Hkv d dtype}... <n_blocks> block...
//   seqs <n_seqs> {len tok...}... <n_k> k...
#include <cstdint>
#include <cstdio>
#include <iostream>
#include <string>
#include <vector>

#include "dta_internal.h"

// The attention entry points (and with them the real dta_tree_destroy, which
// also returns device blocks) need the HIP runtime; this build has no device
// copies, so destroying a tree is deleting it.
extern "C" void dta_tree_destroy(dta_tree_t* tree) { delete tree; }

template <typename T>
static void dump(const char* name, const T* p, int64_t n) {
  std::cout << name;
  for (int64_t i = 0; i < n; ++i) std::cout << ' ' << (long long)p[i];
  std::cout << '\n';
}

int main() {
  std::string kind;
  while (std::cin >> kind) {
    if (kind == "tree") {
      int n;
      std::cin >> n;
      std::vector<int32_t> parent(n > 0 ? n : 0), seg(n > 0 ? n : 0);
      for (auto& x : parent) std::cin >> x;
      for (auto& x : seg) std::cin >> x;
      dta_tree_t* tree = nullptr;
      const int st = dta_tree_build(parent.data(), seg.data(), n, 0, &tree);
      std::cout << "build " << st << '\n';
      int n_cfg;
      std::cin >> n_cfg;
      std::vector<dta_attn_params_t> cfgs(n_cfg);
      for (auto& c : cfgs) {
        std::cin >> c.n_q_heads >> c.n_kv_heads >> c.head_dim >> c.dtype;
        c.softmax_scale = 0.125f;
      }
      int n_blocks;
      std::cin >> n_blocks;
      std::vector<long long> blocks(n_blocks);
      for (auto& b : blocks) std::cin >> b;
      if (st != DTA_OK) continue;
      dta_tree_info_t info;
      dta_tree_info(tree, &info);
      dump("info", &info.n_nodes, sizeof(info) / sizeof(int64_t));
      dta_tree_layout_t lay;
      dta_tree_layout(tree, &lay);
      dump("dfs_order", lay.dfs_order, n);
      dump("node_offset", lay.node_offset, n);
      dump("subtree_tokens", lay.subtree_tokens, n);
      dump("anc_ptr", lay.anc_ptr, n + 1);
      dump("anc_seg_off", lay.anc_seg_off, lay.anc_ptr[n]);
      dump("anc_seg_len", lay.anc_seg_len, lay.anc_ptr[n]);
      dump("token_kend", lay.token_kend, info.n_tokens);
      for (const auto& c : cfgs) {
        dta_schedule_info_t si;
        const int s2 = dta_tree_schedule_info(tree, &c, &si);
        std::cout << "schedule " << s2;
        if (s2 == DTA_OK) dump("", &si.fwd_q_tile_tokens, sizeof(si) / sizeof(int64_t));
        else std::cout << '\n';
        // the segment schedules of every node, first and last row ranges included
        if (s2 == DTA_OK) {
          dta::TileChoice tc;
          dta::choose_tiles(&c, &tc);
          int64_t items = 0;
          for (int u = 0; u < n; ++u) {
            const int64_t a = lay.node_offset[u], b = a + seg[u];
            items += (int64_t)dta::get_segment_schedule(tree, tc.bm, tc.bn, c.n_kv_heads,
                                                        c.n_q_heads / c.n_kv_heads, a, b).kv_items.size();
            items += (int64_t)dta::get_segment_schedule(tree, tc.bm, tc.bn, c.n_kv_heads,
                                                        c.n_q_heads / c.n_kv_heads, b - 1, b).q_tiles.size();
          }
          std::cout << "segment_items " << (long long)items << '\n';
        }
      }
      for (long long b : blocks) {
        dta_plan_t* plan = nullptr;
        const int s3 = dta_tree_plan(tree, b, &plan);
        std::cout << "plan " << s3 << '\n';
        if (s3 != DTA_OK) continue;
        dta_plan_view_t v;
        dta_plan_view(plan, &v);
        dump("leaf_order", v.leaf_order, v.n_leaves);
        std::cout << "ops";
        for (int64_t i = 0; i < v.n_ops; ++i)
          std::cout << ' ' << v.ops[i].op << ' ' << v.ops[i].leaf << ' ' << (long long)v.ops[i].lo << ' '
                    << (long long)v.ops[i].hi;
        std::cout << "\ncalls";
        for (int64_t i = 0; i < v.n_calls; ++i)
          std::cout << ' ' << v.calls[i].op << ' ' << v.calls[i].node << ' ' << (long long)v.calls[i].t_begin << ' '
                    << (long long)v.calls[i].t_end;
        std::cout << '\n';
        dump("call_ptr", v.call_ptr, v.n_ops + 1);
        dta_plan_destroy(plan);
      }
      dta_tree_destroy(tree);
    } else if (kind == "seqs") {
      int n;
      std::cin >> n;
      std::vector<int32_t> toks;
      std::vector<int64_t> offs{0};
      for (int i = 0; i < n; ++i) {
        int len;
        std::cin >> len;
        for (int j = 0; j < len; ++j) {
          int t;
          std::cin >> t;
          toks.push_back(t);
        }
        offs.push_back((int64_t)toks.size());
      }
      int nk;
      std::cin >> nk;
      std::vector<int> ks(nk);
      for (auto& k : ks) std::cin >> k;
      dta_rollouts_t* r = nullptr;
      const int st = dta_rollouts_build(toks.data(), offs.data(), n, &r);
      std::cout << "rollouts " << st << '\n';
      if (st != DTA_OK) continue;
      dta_rollouts_view_t v;
      dta_rollouts_view(r, &v);
      dump("parent", v.parent, v.n_nodes);
      dump("seg_len", v.seg_len, v.n_nodes);
      dump("tokens", v.tokens, v.n_tokens);
      dump("seq_node", v.seq_node, v.n_seqs);
      dump("order", v.order, v.n_seqs);
      dump("lcp", v.lcp, v.n_seqs);
      for (int k : ks) {
        std::vector<int32_t> gb(k > 0 ? k + 1 : 1);
        std::vector<int64_t> gc(k > 0 ? k : 1);
        const int s2 = dta_rollouts_partition(r, k, gb.data(), gc.data());
        std::cout << "partition " << s2 << '\n';
        if (s2 != DTA_OK) continue;
        dump("group_begin", gb.data(), k + 1);
        dump("group_cost", gc.data(), k);
      }
      dta_rollouts_destroy(r);
    }
  }
  return 0;
}
