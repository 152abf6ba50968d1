// Internal declarations shared by the host tree builder, the C-ABI entry points
// and the kernel launchers.  Not part of the public interface.
#pragma once

#include <cstddef>
#include <cstdint>
#include <array>
#include <map>
#include <mutex>
#include <vector>

#include "dta.h"

namespace dta {

// A key interval [start, end) in packed token coordinates.  full != 0 means
// every query row of the tile sees every key of the interval (no mask needed).
struct KeySeg {
  int32_t start, end;
  int32_t full;
  int32_t pad;
};

// One forward / dQ work item: BM consecutive packed query tokens [t0, t1).  The
// keys they can see are the key intervals segs[seg_begin, seg_end) that lie
// before t0 (pieces of t0's root path) followed by the tile's own range, which
// always needs the visibility mask  k <= t < kend[k].
// The first interval is repeated inside the tile record (first.start == first.end
// when there is none), so that a block can start its first K/V copy after one
// dependent read instead of two.
struct QTile {
  int32_t t0, t1;
  int32_t seg_begin, seg_end;
  KeySeg first;
};

// One dK/dV work item: BN consecutive packed keys [k0, k1).  The queries the
// item walks are [q_begin, q_end): for a whole-tree launch q_begin = k0 and
// these are exactly the rows that see at least one of the keys; a segment
// launch narrows the walk to the segment's rows.  Rows in
// [max(k1, q_begin), q_full_end) see all of the keys, every other row needs the
// visibility mask.
struct KvTile {
  int32_t k0, k1;
  int32_t q_end;
  int32_t q_full_end;
  int32_t q_begin;
  int32_t pad[3];
};

// One launch unit of the bf16 dK/dV kernel: key tile [k0, k1) and a slice
// [it_begin, it_end) of its flattened (q head of the group, 64-row query chunk)
// iteration space.  A tile whose walk is much longer than the average is cut
// into several items so that no block becomes the critical path; such items
// write fp32 partial sums to workspace slot `slot` (>= 0) and a reduce launch
// adds them in a fixed order.  slot < 0: the item covers the whole tile and
// writes dK/dV directly.
struct KvItem {
  int32_t k0, k1;
  int32_t q_end, q_full_end;
  int32_t it_begin, it_end;
  int32_t slot;
  int32_t q_begin;   // first row of the walk (see KvTile)
};

// A split key tile: its partial sums live in slots [first_slot, first_slot + nparts).
struct KvReduce {
  int32_t k0, k1;
  int32_t first_slot, nparts;
};

// Tile schedule for one (BM, BN) choice: host vectors, and device copies made on
// first use.  Work items are stored longest first so that the hardware block
// dispatcher, which hands out blocks in index order, balances the CUs.
struct Schedule {
  int bm = 0, bn = 0;
  int kv_keys = 0;   // keys per dK/dV tile in this schedule: bn, or 2*bn where the walks are long
  std::vector<QTile> q_tiles;
  std::vector<KeySeg> segs;
  std::vector<KvTile> kv_tiles;
  int hkv = 0, group = 0;          // head configuration the item split was made for
  std::vector<KvItem> kv_items;
  std::vector<KvReduce> kv_reduce;
  int64_t n_slots = 0;
  int64_t kv_item_iters = 0;       // sum over kv_items of (it_end - it_begin)
  bool kv_queues = false;          // the dK/dV launch runs as resident blocks drawing items from queues
  int64_t fwd_tile_pairs = 0, bwd_tile_pairs = 0;
  // chunks the query tiles stream when every key interval is cut into pieces of 64 / 128 keys
  int64_t fwd_chunks64 = 0, fwd_chunks128 = 0;
  // device copies: one allocation (d_blob, owned, released with the tree) that
  // the typed pointers below point into
  uint64_t last_used = 0;   // segment schedules: the tree's use counter at the latest call
  int device = -1;
  void* d_blob = nullptr;
  size_t d_blob_cap = 0;
  QTile* d_q_tiles = nullptr;
  KeySeg* d_segs = nullptr;
  KvTile* d_kv_tiles = nullptr;
  KvItem* d_kv_items = nullptr;
  KvReduce* d_kv_reduce = nullptr;
};

}  // namespace dta

struct dta_tree {
  int32_t n_nodes = 0;
  std::vector<int32_t> parent, seg_len;
  std::vector<int32_t> dfs_order;
  std::vector<int64_t> node_offset, node_start_depth, subtree_tokens;
  std::vector<int64_t> anc_ptr, anc_seg_off, anc_seg_len;
  std::vector<int32_t> token_kend;   // [T]
  std::vector<int32_t> token_node;   // [T] node id owning each packed token
  dta_tree_info_t info{};
  // schedules keyed by (bm, bn, kv heads, group size)
  std::map<uint64_t, dta::Schedule> schedules;
  // schedules of segment calls, keyed by (tile configuration, t_begin, t_end): at most
  // dta::max_segment_schedules(n_nodes) of them; beyond that the least recently used one is dropped
  // and its device block waits in `retired` for the next schedule that fits into it
  std::map<std::array<uint64_t, 3>, dta::Schedule> segment_schedules;
  uint64_t use_counter = 0;
  struct RetiredBlock { void* ptr; size_t cap; int device; };
  std::vector<RetiredBlock> retired;
  int32_t* d_token_kend = nullptr;
  size_t d_kend_cap = 0;
  int kend_device = -1;
  void* last_use = nullptr;   // hipEvent_t recorded after every launch that reads the device copies
  bool used = false;          // last_use has been recorded at least once
  std::mutex mu;
};

namespace dta {

// Segment schedules a tree keeps: an executor walks a tree's segments over and over, one
// schedule per distinct row range.  The push / pop order has one range per node and chunked
// pops a few more, so the bound grows with the tree: max(1024, 4 x nodes + 64).
inline size_t max_segment_schedules(int32_t n_nodes) {
  const size_t by_nodes = 4 * (size_t)n_nodes + 64;
  return by_nodes > 1024 ? by_nodes : 1024;
}

// Resident blocks of a launch whose blocks draw work items from queues: the
// 256 CUs of an MI355X times the blocks of that kernel that fit on a CU.
constexpr int kNumCUs = 256;
// Key tiles of 256 keys (eight-wave dK/dV blocks) for schedules of long walks.
constexpr bool wide_key_tiles = true;

// Key of a whole-tree schedule in dta_tree::schedules.
inline uint64_t schedule_key(int bm, int bn, int hkv, int group) {
  return ((uint64_t)bm << 48) | ((uint64_t)bn << 32) | ((uint64_t)hkv << 16) | (uint64_t)group;
}
// Host: build (or fetch) the schedule for tile sizes (bm, bn).
Schedule& get_schedule(dta_tree* tree, int bm, int bn, int hkv, int group);
// Same for a segment call on rows [t_begin, t_end), which must lie inside one
// node's segment (checked by the caller): query tiles over the rows, key tiles
// over the root path up to t_end, no split items.
Schedule& get_segment_schedule(dta_tree* tree, int bm, int bn, int hkv, int group,
                               int64_t t_begin, int64_t t_end);
// Bytes of fp32 partial dK/dV sums the split items of a schedule need.
size_t partial_bytes(const Schedule& s);

// Tile sizes the kernels use for a head configuration.
struct TileChoice {
  int bm;       // query tokens per forward / dQ work item
  int bn;       // keys per dK/dV work item
  int hb;       // q heads of one kv group handled by one forward block
  int hblocks;  // blocks per (tile, kv head) = group size / hb
};
int choose_tiles(const dta_attn_params_t* p, TileChoice* out);
int validate_params(const dta_attn_params_t* p);

struct LaunchArgs {
  const dta_tree* tree;
  const Schedule* sched;
  const int32_t* d_kend;
  dta_attn_params_t p;
  TileChoice tc;
  const void *q, *k, *v, *o, *d_o;
  const float* lse_in;
  void *o_out, *dq, *dk, *dv;
  float* lse_out;
  float* delta;  // workspace: D[t,h] = dO.O
  float* lse2;   // workspace (bf16 path): -lse / softmax_scale, written with delta (there: -D)
  int* tickets;    // workspace (bf16 path): 2 x n_kv_heads work-queue counters
  float* partial;  // workspace: fp32 partial dK/dV of split key tiles
  // segment calls: rows [row_begin, row_end) only, and dK/dV are ADDED to these
  // fp32 [T,Hkv,d] accumulators instead of written to dk/dv (null otherwise)
  int64_t row_begin, row_end;
  float *dk_acc, *dv_acc;
  uint32_t stages;  // backward stages to launch (DTA_BWD_*)
  void* stream;
};

// HIP keeps the last error of earlier, unrelated runtime calls of this thread
// (the caller's framework may have left one behind).  clear_hip_error() drops it
// before a launch; launch_status() turns the launch's own result into a DTA
// status and names a failure on stderr.
void clear_hip_error();
int launch_status(const char* what);

// The backward entry points share this: argument checks, metadata residency and
// launch.  allocate_ok = false refuses (DTA_ERR_INVALID_ARG) instead of building
// or uploading anything that is not resident yet.
int bwd_entry(dta_tree* tree, const dta_attn_params_t* params, const void* q, const void* k,
              const void* v, const void* o, const float* lse, const void* d_o, void* dq, void* dk,
              void* dv, void* workspace, size_t workspace_bytes, void* hip_stream,
              uint32_t stage_mask, bool allocate_ok);
// Backward workspace bytes for a tree whose schedule may still have to be built.
size_t bwd_workspace_need(dta_tree* tree, const dta_attn_params_t* params);
// Device address and size of the library-held scratch array on device `dev`,
// which must be the current device (resolved once per device, then cached).
int static_scratch(int dev, void** ptr, size_t* bytes);

// Kernel launchers (defined in the .hip files); return a DTA status.
int launch_fwd_f32(const LaunchArgs& a);
int launch_bwd_f32(const LaunchArgs& a);
int launch_fwd_bf16(const LaunchArgs& a);
int launch_bwd_bf16(const LaunchArgs& a);

}  // namespace dta
