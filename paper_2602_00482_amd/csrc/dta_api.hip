// C-ABI attention entry points: argument checks, device metadata upload and
// dispatch to the kernel launchers.  See include/dta.h for the contract.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <new>

#include "dta_internal.h"

namespace {

inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

size_t delta_bytes(const dta_tree* tree, const dta_attn_params_t* p) {
  return round_up((size_t)tree->info.n_tokens * (size_t)p->n_q_heads * sizeof(float), 256);
}

// delta plus, in bf16 mode, the rescaled lse and the partial sums of split key tiles (building the
// host schedule if this head configuration has not been seen yet)
size_t bwd_workspace_bytes(dta_tree* tree, const dta::TileChoice& tc, const dta_attn_params_t* p) {
  size_t bytes = delta_bytes(tree, p);
  if (p->dtype == DTA_BF16) {
    bytes += delta_bytes(tree, p);   // lse in log2 units, same shape as delta
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

template <typename T>
int upload(const std::vector<T>& host, T** dev) {
  if (*dev) {
    (void)hipFree(*dev);
    *dev = nullptr;
  }
  size_t bytes = host.size() * sizeof(T);
  if (bytes == 0) bytes = sizeof(T);
  if (hipMalloc((void**)dev, bytes) != hipSuccess) {
    *dev = nullptr;
    (void)hipGetLastError();
    return DTA_ERR_ALLOC;
  }
  if (!host.empty()) {
    hipError_t e = hipMemcpy(*dev, host.data(), host.size() * sizeof(T), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
      fprintf(stderr, "dta: metadata upload: %s\n", hipGetErrorString(e));
      (void)hipGetLastError();
      return DTA_ERR_HIP;
    }
  }
  return DTA_OK;
}

// Makes sure the schedule for (bm, bn) and kend[] are resident on the current
// device.  Takes the tree lock; blocking on first use, a no-op afterwards.
int ensure_device(dta_tree* tree, const dta::TileChoice& tc, const dta_attn_params_t* p,
                  dta::Schedule** out) {
  std::lock_guard<std::mutex> lock(tree->mu);
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) {
    fprintf(stderr, "dta: hipGetDevice failed (no usable GPU?)\n");
    (void)hipGetLastError();
    return DTA_ERR_HIP;
  }
  dta::Schedule* s;
  try {
    s = &dta::get_schedule(tree, tc.bm, tc.bn, p->n_kv_heads, p->n_q_heads / p->n_kv_heads);
  } catch (const std::bad_alloc&) {
    return DTA_ERR_ALLOC;
  }
  int st;
  if (tree->kend_device != dev) {
    if ((st = upload(tree->token_kend, &tree->d_token_kend)) != DTA_OK) return st;
    tree->kend_device = dev;
  }
  if (s->device != dev) {
    if ((st = upload(s->q_tiles, &s->d_q_tiles)) != DTA_OK) return st;
    if ((st = upload(s->segs, &s->d_segs)) != DTA_OK) return st;
    if ((st = upload(s->kv_tiles, &s->d_kv_tiles)) != DTA_OK) return st;
    if ((st = upload(s->kv_items, &s->d_kv_items)) != DTA_OK) return st;
    if ((st = upload(s->kv_reduce, &s->d_kv_reduce)) != DTA_OK) return st;
    s->device = dev;
  }
  *out = s;
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
  if (tree->d_token_kend) (void)hipFree(tree->d_token_kend);
  for (auto& kv : tree->schedules) {
    dta::Schedule& s = kv.second;
    if (s.d_q_tiles) (void)hipFree(s.d_q_tiles);
    if (s.d_segs) (void)hipFree(s.d_segs);
    if (s.d_kv_tiles) (void)hipFree(s.d_kv_tiles);
    if (s.d_kv_items) (void)hipFree(s.d_kv_items);
    if (s.d_kv_reduce) (void)hipFree(s.d_kv_reduce);
  }
  delete tree;
}

size_t dta_tree_attn_workspace_bytes(const dta_tree_t* tree, const dta_attn_params_t* params,
                                     int is_bwd) {
  dta::TileChoice tc;
  if (!tree || dta::choose_tiles(params, &tc) != DTA_OK) return 0;
  if (!is_bwd) return 0;
  return bwd_workspace_bytes(const_cast<dta_tree*>(tree), tc, params);
}

int dta_tree_attn_prepare(dta_tree_t* tree, const dta_attn_params_t* params) {
  if (!tree) return DTA_ERR_INVALID_ARG;
  dta::TileChoice tc;
  int st = dta::choose_tiles(params, &tc);
  if (st != DTA_OK) return st;
  dta::Schedule* s = nullptr;
  return ensure_device(tree, tc, params, &s);
}

int dta_tree_attn_fwd(dta_tree_t* tree, const dta_attn_params_t* params, const void* q,
                      const void* k, const void* v, void* o, float* lse, void* workspace,
                      size_t workspace_bytes, void* hip_stream) {
  (void)workspace;
  (void)workspace_bytes;
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
  a.stream = hip_stream;
  return params->dtype == DTA_F32 ? dta::launch_fwd_f32(a) : dta::launch_fwd_bf16(a);
}

int dta_tree_attn_bwd_stages(dta_tree_t* tree, const dta_attn_params_t* params, const void* q,
                             const void* k, const void* v, const void* o, const float* lse,
                             const void* d_o, void* dq, void* dk, void* dv, void* workspace,
                             size_t workspace_bytes, void* hip_stream, uint32_t stage_mask) {
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
  a.o = o;
  a.d_o = d_o;
  a.lse_in = lse;
  a.dq = dq;
  a.dk = dk;
  a.dv = dv;
  a.delta = (float*)workspace;
  a.lse2 = (float*)((char*)workspace + delta_bytes(tree, params));
  a.partial = (float*)((char*)workspace + 2 * delta_bytes(tree, params));
  a.stages = stage_mask;
  a.stream = hip_stream;
  return params->dtype == DTA_F32 ? dta::launch_bwd_f32(a) : dta::launch_bwd_bf16(a);
}

int dta_tree_attn_bwd(dta_tree_t* tree, const dta_attn_params_t* params, const void* q,
                      const void* k, const void* v, const void* o, const float* lse,
                      const void* d_o, void* dq, void* dk, void* dv, void* workspace,
                      size_t workspace_bytes, void* hip_stream) {
  return dta_tree_attn_bwd_stages(tree, params, q, k, v, o, lse, d_o, dq, dk, dv, workspace,
                                  workspace_bytes, hip_stream, DTA_BWD_ALL);
}

}  // extern "C"
