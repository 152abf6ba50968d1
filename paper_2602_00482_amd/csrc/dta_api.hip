// C-ABI attention entry points: argument checks, device metadata upload and
// dispatch to the kernel launchers.  See include/dta.h for the contract.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>
#include <initializer_list>
#include <memory>
#include <mutex>
#include <vector>
#include <new>

#include "dta_internal.h"

namespace {

inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

size_t delta_bytes(const dta_tree* tree, const dta_attn_params_t* p) {
  return round_up((size_t)tree->info.n_tokens * (size_t)p->n_q_heads * sizeof(float), 256);
}

// ticket counters of the kernels that draw their work items from queues: one int per kv head
// for each of two kernels
size_t ticket_bytes(const dta_attn_params_t* p) {
  return round_up(2 * (size_t)p->n_kv_heads * sizeof(int), 256);
}

// delta plus, in bf16 mode, the rescaled lse, the ticket counters and the partial sums of split
// key tiles (building the host schedule if this head configuration has not been seen yet)
size_t bwd_workspace_bytes(dta_tree* tree, const dta::TileChoice& tc, const dta_attn_params_t* p) {
  size_t bytes = delta_bytes(tree, p);
  if (p->dtype == DTA_BF16) {
    bytes += delta_bytes(tree, p);   // lse in log2 units, same shape as delta
    bytes += ticket_bytes(p);
    try {
      std::lock_guard<std::mutex> lock(tree->mu);
      bytes += dta::partial_bytes(
          dta::get_schedule(tree, tc.bm, tc.bn, p->n_kv_heads, p->n_q_heads / p->n_kv_heads));
    } catch (const std::bad_alloc&) {
      return 0;
    }
  }
  return bytes;
}

// Device metadata lives in blocks from a small pool of the library's own and is
// filled on a stream of the library's own (non-blocking, default priority, one
// per device, kept until the process ends), so that preparing the next tree
// neither waits for kernels the caller still has in flight nor, on release, for
// the device to go idle.  A released block carries the event recorded after
// the last launch that reads it and is handed out again only once that event
// has completed; blocks are power-of-two sized and are not returned to the
// driver while the process lives (hipFree would wait for the device).
constexpr int kMaxDevices = 64;
std::mutex g_stream_mu;
hipStream_t g_stream[kMaxDevices];
bool g_stream_ok[kMaxDevices];

int upload_stream(int dev, hipStream_t* out) {
  if (dev < 0 || dev >= kMaxDevices) return DTA_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_stream_mu);
  if (!g_stream_ok[dev]) {
    if (hipStreamCreateWithFlags(&g_stream[dev], hipStreamNonBlocking) != hipSuccess) {
      fprintf(stderr, "dta: cannot create the metadata upload stream\n");
      (void)hipGetLastError();
      return DTA_ERR_HIP;
    }
    g_stream_ok[dev] = true;
  }
  *out = g_stream[dev];
  return DTA_OK;
}

struct EventHolder {
  hipEvent_t ev;
  bool done = false;   // the event has been seen complete (guarded by g_pool_mu)
  explicit EventHolder(hipEvent_t e) : ev(e) {}
  ~EventHolder() { (void)hipEventDestroy(ev); }
};

struct Block {
  void* ptr;
  size_t cap;
  std::shared_ptr<EventHolder> busy_until;   // null: free right away
};
std::mutex g_pool_mu;
// never destroyed: at process exit the HIP runtime may already be gone when
// static destructors run, and the blocks' events must not be touched then
std::vector<Block>* const g_pool = new std::vector<Block>[kMaxDevices];

size_t size_class(size_t bytes) {
  size_t c = 4096;
  while (c < bytes) c <<= 1;
  return c;
}

// A block of at least `bytes` on the current device `dev` that no launch reads
// any more; *cap receives its size.  Null on failure.
void* pool_alloc(int dev, size_t bytes, size_t* cap) {
  const size_t c = size_class(bytes);
  *cap = c;
  {
    std::lock_guard<std::mutex> lock(g_pool_mu);
    std::vector<Block>& pool = g_pool[dev];
    const EventHolder* not_ready = nullptr;   // all blocks of one tree share a holder: ask once
    for (size_t i = 0; i < pool.size(); ++i) {
      if (pool[i].cap != c) continue;
      EventHolder* h = pool[i].busy_until.get();
      if (h && !h->done) {
        if (h == not_ready) continue;
        if (hipEventQuery(h->ev) != hipSuccess) {
          (void)hipGetLastError();   // not ready yet: not an error
          not_ready = h;
          continue;
        }
        h->done = true;
      }
      void* p = pool[i].ptr;
      pool[i] = pool.back();
      pool.pop_back();
      return p;
    }
  }
  void* p = nullptr;
  if (hipMalloc(&p, c) != hipSuccess) {
    (void)hipGetLastError();
    return nullptr;
  }
  return p;
}

void pool_release(int dev, void* ptr, size_t cap, std::shared_ptr<EventHolder> busy_until) {
  if (!ptr) return;
  if (dev < 0 || dev >= kMaxDevices) {
    (void)hipFree(ptr);
    return;
  }
  std::lock_guard<std::mutex> lock(g_pool_mu);
  g_pool[dev].push_back(Block{ptr, cap, std::move(busy_until)});
}

struct Part {
  const void* src;
  size_t bytes;
  void** dst;
};

// One block holding every part (each 256-byte aligned), filled from the host
// and complete on return.
int upload_parts(int dev, hipStream_t st, std::initializer_list<Part> parts, void** blob,
                 size_t* cap, dta_tree* reuse_from = nullptr) {
  size_t total = 0;
  for (const Part& p : parts) total += round_up(p.bytes ? p.bytes : 1, 256);
  std::vector<char> staging;
  try {
    staging.resize(total);
  } catch (const std::bad_alloc&) {
    return DTA_ERR_ALLOC;
  }
  *blob = nullptr;
  if (reuse_from) {
    // a block this tree set aside when it dropped an old segment schedule: launches
    // in flight may still read it, so the copy is ordered behind the tree's latest launch
    auto& rl = reuse_from->retired;
    for (size_t i = 0; i < rl.size(); ++i) {
      if (rl[i].device != dev || rl[i].cap < total) continue;
      if (reuse_from->used &&
          hipStreamWaitEvent(st, (hipEvent_t)reuse_from->last_use, 0) != hipSuccess) {
        (void)hipGetLastError();
        break;
      }
      *blob = rl[i].ptr;
      *cap = rl[i].cap;
      rl[i] = rl.back();
      rl.pop_back();
      break;
    }
  }
  if (!*blob) *blob = pool_alloc(dev, total, cap);
  if (!*blob) return DTA_ERR_ALLOC;
  size_t off = 0;
  for (const Part& p : parts) {
    if (p.bytes) memcpy(staging.data() + off, p.src, p.bytes);
    *p.dst = (char*)*blob + off;
    off += round_up(p.bytes ? p.bytes : 1, 256);
  }
  hipError_t e = hipMemcpyAsync(*blob, staging.data(), total, hipMemcpyHostToDevice, st);
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  if (e != hipSuccess) {
    fprintf(stderr, "dta: metadata upload: %s\n", hipGetErrorString(e));
    (void)hipGetLastError();
    pool_release(dev, *blob, *cap, nullptr);
    *blob = nullptr;
    return DTA_ERR_HIP;
  }
  return DTA_OK;
}

// Used when a tree moves to another device: waits for the launches that still
// read the old copies (rare path), then returns the block to its pool.
void release_blob_blocking(dta_tree* tree, void* blob, size_t cap, int dev) {
  if (!blob) return;
  if (tree->used) (void)hipEventSynchronize((hipEvent_t)tree->last_use);
  pool_release(dev, blob, cap, nullptr);
}

template <typename T>
Part part_of(const std::vector<T>& v, T** dst) {
  return Part{v.data(), v.size() * sizeof(T), (void**)dst};
}

// Makes sure the schedule for (bm, bn) and kend[] are resident on the current
// device.  Takes the tree lock; blocking (on the upload only) on first use, a
// no-op afterwards.
int ensure_device(dta_tree* tree, const dta::TileChoice& tc, const dta_attn_params_t* p,
                  dta::Schedule** out, int64_t t_begin = -1, int64_t t_end = -1,
                  bool allocate_ok = true) {
  std::lock_guard<std::mutex> lock(tree->mu);
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) {
    fprintf(stderr, "dta: hipGetDevice failed (no usable GPU?)\n");
    (void)hipGetLastError();
    return DTA_ERR_HIP;
  }
  if (!allocate_ok) {
    // a caller that must not allocate: everything has to be resident already
    // (dta_tree_attn_prepare on this device); look, do not build
    const uint64_t key = dta::schedule_key(tc.bm, tc.bn, p->n_kv_heads, p->n_q_heads / p->n_kv_heads);
    auto it = tree->schedules.find(key);
    if (it == tree->schedules.end() || it->second.device != dev || tree->kend_device != dev ||
        !tree->last_use)
      return DTA_ERR_INVALID_ARG;
    *out = &it->second;
    return DTA_OK;
  }
  dta::Schedule* s;
  try {
    s = t_begin < 0
            ? &dta::get_schedule(tree, tc.bm, tc.bn, p->n_kv_heads, p->n_q_heads / p->n_kv_heads)
            : &dta::get_segment_schedule(tree, tc.bm, tc.bn, p->n_kv_heads,
                                         p->n_q_heads / p->n_kv_heads, t_begin, t_end);
  } catch (const std::bad_alloc&) {
    return DTA_ERR_ALLOC;
  }
  int st;
  if (tree->kend_device == dev && s->device == dev) {
    *out = s;
    return DTA_OK;
  }
  hipStream_t us;
  if ((st = upload_stream(dev, &us)) != DTA_OK) return st;
  if (!tree->last_use) {
    hipEvent_t ev;
    if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) {
      (void)hipGetLastError();
      return DTA_ERR_HIP;
    }
    tree->last_use = ev;
  }
  if (tree->kend_device != dev) {
    release_blob_blocking(tree, tree->d_token_kend, tree->d_kend_cap, tree->kend_device);
    tree->d_token_kend = nullptr;
    tree->kend_device = -1;
    void* blob = nullptr;
    if ((st = upload_parts(dev, us, {part_of(tree->token_kend, &tree->d_token_kend)}, &blob,
                           &tree->d_kend_cap)) != DTA_OK)
      return st;
    tree->kend_device = dev;
  }
  if (s->device != dev) {
    release_blob_blocking(tree, s->d_blob, s->d_blob_cap, s->device);
    s->d_blob = nullptr;
    s->device = -1;
    if ((st = upload_parts(dev, us,
                           {part_of(s->q_tiles, &s->d_q_tiles), part_of(s->segs, &s->d_segs),
                            part_of(s->kv_tiles, &s->d_kv_tiles),
                            part_of(s->kv_items, &s->d_kv_items),
                            part_of(s->kv_reduce, &s->d_kv_reduce)},
                           &s->d_blob, &s->d_blob_cap, t_begin < 0 ? nullptr : tree)) != DTA_OK)
      return st;
    s->device = dev;
  }
  *out = s;
  return DTA_OK;
}

// After a launch on `stream` that reads the tree's device copies.
int mark_use(dta_tree* tree, void* stream, int launch_result) {
  if (launch_result != DTA_OK) return launch_result;
  std::lock_guard<std::mutex> lock(tree->mu);
  if (hipEventRecord((hipEvent_t)tree->last_use, (hipStream_t)stream) != hipSuccess) {
    (void)hipGetLastError();
    return DTA_ERR_HIP;
  }
  tree->used = true;
  return DTA_OK;
}

inline bool misaligned(const void* p) { return ((uintptr_t)p & 15u) != 0; }

}  // namespace

namespace dta {

void clear_hip_error() { (void)hipGetLastError(); }

int launch_status(const char* what) {
  hipError_t e = hipGetLastError();
  if (e == hipSuccess) return DTA_OK;
  fprintf(stderr, "dta: %s: %s\n", what, hipGetErrorString(e));
  return DTA_ERR_HIP;
}

}  // namespace dta

extern "C" {

void dta_tree_destroy(dta_tree_t* tree) {
  if (!tree) return;
  // the device copies go back to the pool together with the event after the
  // tree's last launch; the pool hands them out again once it has completed
  std::shared_ptr<EventHolder> busy;
  if (tree->last_use) {
    busy = std::make_shared<EventHolder>((hipEvent_t)tree->last_use);
    if (!tree->used) busy.reset();   // never recorded: destroys the event, blocks are free at once
  }
  pool_release(tree->kend_device, tree->d_token_kend, tree->d_kend_cap, busy);
  for (auto& kv : tree->schedules)
    pool_release(kv.second.device, kv.second.d_blob, kv.second.d_blob_cap, busy);
  for (auto& kv : tree->segment_schedules)
    pool_release(kv.second.device, kv.second.d_blob, kv.second.d_blob_cap, busy);
  for (auto& rb : tree->retired) pool_release(rb.device, rb.ptr, rb.cap, busy);
  delete tree;
}

size_t dta_tree_attn_workspace_bytes(const dta_tree_t* tree, const dta_attn_params_t* params,
                                     int is_bwd) {
  dta::TileChoice tc;
  if (!tree || dta::choose_tiles(params, &tc) != DTA_OK) return 0;
  if (!is_bwd) return params->dtype == DTA_BF16 ? ticket_bytes(params) : 0;
  return bwd_workspace_bytes(const_cast<dta_tree*>(tree), tc, params);
}

int dta_tree_attn_prepare(dta_tree_t* tree, const dta_attn_params_t* params) {
  if (!tree) return DTA_ERR_INVALID_ARG;
  dta::TileChoice tc;
  int st = dta::choose_tiles(params, &tc);
  if (st != DTA_OK) return st;
  dta::Schedule* s = nullptr;
  if ((st = ensure_device(tree, tc, params, &s)) != DTA_OK) return st;
  // set-up for dta_tree_attn_bwd_noalloc: resolve this device's copy of the
  // library-held scratch array now, so that the call itself has nothing left to do
  int dev = -1;
  void* scratch = nullptr;
  size_t scratch_bytes = 0;
  if (hipGetDevice(&dev) != hipSuccess) return DTA_ERR_HIP;
  return dta::static_scratch(dev, &scratch, &scratch_bytes);
}

int dta_tree_attn_fwd(dta_tree_t* tree, const dta_attn_params_t* params, const void* q,
                      const void* k, const void* v, void* o, float* lse, void* workspace,
                      size_t workspace_bytes, void* hip_stream) {
  if (!tree || !params) return DTA_ERR_INVALID_ARG;
  dta::TileChoice tc;
  int st = dta::choose_tiles(params, &tc);
  if (st != DTA_OK) return st;
  if (!q || !k || !v || !o || !lse) return DTA_ERR_INVALID_ARG;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o) || misaligned(lse))
    return DTA_ERR_INVALID_ARG;
  dta::Schedule* s = nullptr;
  if ((st = ensure_device(tree, tc, params, &s)) != DTA_OK) return st;
  dta::LaunchArgs a{};
  a.tree = tree;
  a.sched = s;
  a.d_kend = tree->d_token_kend;
  a.p = *params;
  a.tc = tc;
  a.q = q;
  a.k = k;
  a.v = v;
  a.o_out = o;
  a.lse_out = lse;
  // optional: with room for the work-queue counters the bf16 forward may run as
  // resident blocks drawing items from queues
  if (params->dtype == DTA_BF16 && workspace && ((uintptr_t)workspace & 255u) == 0 &&
      workspace_bytes >= ticket_bytes(params))
    a.tickets = (int*)workspace;
  a.row_begin = 0;
  a.row_end = tree->info.n_tokens;
  a.stream = hip_stream;
  return mark_use(tree, hip_stream,
                  params->dtype == DTA_F32 ? dta::launch_fwd_f32(a) : dta::launch_fwd_bf16(a));
}

int dta_tree_attn_bwd_stages(dta_tree_t* tree, const dta_attn_params_t* params, const void* q,
                             const void* k, const void* v, const void* o, const float* lse,
                             const void* d_o, void* dq, void* dk, void* dv, void* workspace,
                             size_t workspace_bytes, void* hip_stream, uint32_t stage_mask) {
  return dta::bwd_entry(tree, params, q, k, v, o, lse, d_o, dq, dk, dv, workspace, workspace_bytes,
                        hip_stream, stage_mask, true);
}

}  // extern "C"

namespace dta {

size_t bwd_workspace_need(dta_tree* tree, const dta_attn_params_t* params) {
  TileChoice tc;
  if (!tree || choose_tiles(params, &tc) != DTA_OK) return 0;
  return bwd_workspace_bytes(tree, tc, params);
}

int bwd_entry(dta_tree* tree, const dta_attn_params_t* params, const void* q, const void* k,
              const void* v, const void* o, const float* lse, const void* d_o, void* dq, void* dk,
              void* dv, void* workspace, size_t workspace_bytes, void* hip_stream,
              uint32_t stage_mask, bool allocate_ok) {
  if (!tree || !params) return DTA_ERR_INVALID_ARG;
  if (stage_mask == 0 || (stage_mask & ~(uint32_t)DTA_BWD_ALL)) return DTA_ERR_INVALID_ARG;
  dta::TileChoice tc;
  int st = dta::choose_tiles(params, &tc);
  if (st != DTA_OK) return st;
  const bool want_dq = stage_mask & DTA_BWD_DQ, want_dkdv = stage_mask & DTA_BWD_DKDV;
  if (!q || !k || !v || !o || !lse || !d_o) return DTA_ERR_INVALID_ARG;
  if ((want_dq && !dq) || (want_dkdv && (!dk || !dv))) return DTA_ERR_INVALID_ARG;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o) || misaligned(lse) ||
      misaligned(d_o) || misaligned(dq) || misaligned(dk) || misaligned(dv))
    return DTA_ERR_INVALID_ARG;
  if (!workspace || workspace_bytes < bwd_workspace_bytes(tree, tc, params) ||
      ((uintptr_t)workspace & 255u))
    return DTA_ERR_WORKSPACE;
  dta::Schedule* s = nullptr;
  if ((st = ensure_device(tree, tc, params, &s, -1, -1, allocate_ok)) != DTA_OK) return st;
  dta::LaunchArgs a{};
  a.tree = tree;
  a.sched = s;
  a.d_kend = tree->d_token_kend;
  a.p = *params;
  a.tc = tc;
  a.q = q;
  a.k = k;
  a.v = v;
  a.o = o;
  a.d_o = d_o;
  a.lse_in = lse;
  a.dq = dq;
  a.dk = dk;
  a.dv = dv;
  a.delta = (float*)workspace;
  a.lse2 = (float*)((char*)workspace + delta_bytes(tree, params));
  a.tickets = (int*)((char*)workspace + 2 * delta_bytes(tree, params));
  a.partial = (float*)((char*)workspace + 2 * delta_bytes(tree, params) + ticket_bytes(params));
  a.stages = stage_mask;
  a.row_begin = 0;
  a.row_end = tree->info.n_tokens;
  a.stream = hip_stream;
  return mark_use(tree, hip_stream,
                  params->dtype == DTA_F32 ? dta::launch_bwd_f32(a) : dta::launch_bwd_bf16(a));
}

}  // namespace dta

extern "C" {

int dta_tree_attn_bwd(dta_tree_t* tree, const dta_attn_params_t* params, const void* q,
                      const void* k, const void* v, const void* o, const float* lse,
                      const void* d_o, void* dq, void* dk, void* dv, void* workspace,
                      size_t workspace_bytes, void* hip_stream) {
  return dta_tree_attn_bwd_stages(tree, params, q, k, v, o, lse, d_o, dq, dk, dv, workspace,
                                  workspace_bytes, hip_stream, DTA_BWD_ALL);
}

// rows [t_begin, t_end) must be non-empty and lie inside one node's segment
static int check_segment(const dta_tree* tree, int64_t t_begin, int64_t t_end) {
  if (t_begin < 0 || t_end <= t_begin || t_end > tree->info.n_tokens) return DTA_ERR_INVALID_ARG;
  if (tree->token_node[(size_t)t_begin] != tree->token_node[(size_t)(t_end - 1)])
    return DTA_ERR_INVALID_ARG;
  return DTA_OK;
}

int dta_tree_attn_fwd_segment(dta_tree_t* tree, const dta_attn_params_t* params, int64_t t_begin,
                              int64_t t_end, const void* q, const void* k, const void* v, void* o,
                              float* lse, void* workspace, size_t workspace_bytes,
                              void* hip_stream) {
  (void)workspace;
  (void)workspace_bytes;
  if (!tree || !params) return DTA_ERR_INVALID_ARG;
  dta::TileChoice tc;
  int st = dta::choose_tiles(params, &tc);
  if (st != DTA_OK) return st;
  if ((st = check_segment(tree, t_begin, t_end)) != DTA_OK) return st;
  if (!q || !k || !v || !o || !lse) return DTA_ERR_INVALID_ARG;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o) || misaligned(lse))
    return DTA_ERR_INVALID_ARG;
  dta::Schedule* s = nullptr;
  if ((st = ensure_device(tree, tc, params, &s, t_begin, t_end)) != DTA_OK) return st;
  dta::LaunchArgs a{};
  a.tree = tree;
  a.sched = s;
  a.d_kend = tree->d_token_kend;
  a.p = *params;
  a.tc = tc;
  a.q = q;
  a.k = k;
  a.v = v;
  a.o_out = o;
  a.lse_out = lse;
  a.row_begin = t_begin;
  a.row_end = t_end;
  a.stream = hip_stream;
  return mark_use(tree, hip_stream,
                  params->dtype == DTA_F32 ? dta::launch_fwd_f32(a) : dta::launch_fwd_bf16(a));
}

int dta_tree_attn_bwd_segment(dta_tree_t* tree, const dta_attn_params_t* params, int64_t t_begin,
                              int64_t t_end, const void* q, const void* k, const void* v,
                              const void* o, const float* lse, const void* d_o, void* dq,
                              float* dk_acc, float* dv_acc, void* workspace,
                              size_t workspace_bytes, void* hip_stream) {
  if (!tree || !params) return DTA_ERR_INVALID_ARG;
  dta::TileChoice tc;
  int st = dta::choose_tiles(params, &tc);
  if (st != DTA_OK) return st;
  if ((st = check_segment(tree, t_begin, t_end)) != DTA_OK) return st;
  if (!q || !k || !v || !o || !lse || !d_o || !dq || !dk_acc || !dv_acc) return DTA_ERR_INVALID_ARG;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o) || misaligned(lse) ||
      misaligned(d_o) || misaligned(dq) || misaligned(dk_acc) || misaligned(dv_acc))
    return DTA_ERR_INVALID_ARG;
  if (!workspace || workspace_bytes < bwd_workspace_bytes(tree, tc, params) ||
      ((uintptr_t)workspace & 255u))
    return DTA_ERR_WORKSPACE;
  dta::Schedule* s = nullptr;
  if ((st = ensure_device(tree, tc, params, &s, t_begin, t_end)) != DTA_OK) return st;
  dta::LaunchArgs a{};
  a.tree = tree;
  a.sched = s;
  a.d_kend = tree->d_token_kend;
  a.p = *params;
  a.tc = tc;
  a.q = q;
  a.k = k;
  a.v = v;
  a.o = o;
  a.d_o = d_o;
  a.lse_in = lse;
  a.dq = dq;
  a.dk_acc = dk_acc;
  a.dv_acc = dv_acc;
  a.delta = (float*)workspace;
  a.lse2 = (float*)((char*)workspace + delta_bytes(tree, params));
  a.tickets = (int*)((char*)workspace + 2 * delta_bytes(tree, params));
  a.partial = (float*)((char*)workspace + 2 * delta_bytes(tree, params) + ticket_bytes(params));
  a.stages = DTA_BWD_ALL;
  a.row_begin = t_begin;
  a.row_end = t_end;
  a.stream = hip_stream;
  return mark_use(tree, hip_stream,
                  params->dtype == DTA_F32 ? dta::launch_bwd_f32(a) : dta::launch_bwd_bf16(a));
}

}  // extern "C"
