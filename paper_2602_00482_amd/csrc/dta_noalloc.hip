// dta_tree_attn_bwd_noalloc: the backward pass for callers that cannot allocate
// device memory (code under HIP graph capture, serving loops, harnesses that
// forbid it).  The scratch memory that dta_tree_attn_bwd takes as a workspace
// argument lives here in a device array the library itself holds.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <mutex>

#include "dta_internal.h"

namespace {

// 160 MiB per GPU, held from the moment the library's code is loaded on that GPU
// until the process ends: two fp32 row statistics per (token, q head), the
// work-queue counters and the fp32 partial sums of split key tiles.  Enough for
// trees of a few hundred thousand tokens (265 672 tokens x 64 q heads need
// 130 MiB) unless a long shared prefix is cut into very many partial sums (the
// deep benchmark tree with its 16K-token root needs 468 MiB and is refused).
constexpr size_t kScratchBytes = (size_t)160 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// In host code `scratch` is only a handle for the symbol; each device has its own
// copy at its own address, which hipGetSymbolAddress returns for the CURRENT
// device.  Resolved once per device and kept.
constexpr int kMaxDevices = 64;
std::mutex g_mu;
void* g_ptr[kMaxDevices];

}  // namespace

namespace dta {

int static_scratch(int dev, void** ptr, size_t* bytes) {
  if (dev < 0 || dev >= kMaxDevices) return DTA_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_mu);
  if (!g_ptr[dev]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      fprintf(stderr, "dta: cannot resolve the library's scratch array on device %d: %s\n", dev,
              hipGetErrorString(e));
      (void)hipGetLastError();
      return DTA_ERR_HIP;
    }
    g_ptr[dev] = p;
  }
  *ptr = g_ptr[dev];
  *bytes = kScratchBytes;
  return DTA_OK;
}

}  // namespace dta

extern "C" int dta_tree_attn_bwd_noalloc(dta_tree_t* tree, const dta_attn_params_t* params,
                                         const void* q, const void* k, const void* v,
                                         const void* o, const float* lse, const void* d_o,
                                         void* dq, void* dk, void* dv, void* hip_stream) {
  if (!tree || !params) return DTA_ERR_INVALID_ARG;
  const size_t need = dta::bwd_workspace_need(tree, params);
  if (need == 0) return DTA_ERR_INVALID_ARG;   // bad parameters: the common entry names the reason
  if (need > kScratchBytes) {
    fprintf(stderr,
            "dta_tree_attn_bwd_noalloc: this tree and head configuration need %zu bytes of scratch, "
            "the library holds %zu; use dta_tree_attn_bwd with a workspace\n",
            need, kScratchBytes);
    return DTA_ERR_WORKSPACE;
  }
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) {
    (void)hipGetLastError();
    return DTA_ERR_HIP;
  }
  void* ptr = nullptr;
  size_t bytes = 0;
  int st = dta::static_scratch(dev, &ptr, &bytes);
  if (st != DTA_OK) return st;
  st = dta::bwd_entry(tree, params, q, k, v, o, lse, d_o, dq, dk, dv, ptr, bytes, hip_stream,
                      DTA_BWD_ALL, /*allocate_ok=*/false);
  if (st == DTA_ERR_INVALID_ARG && q && k && v && o && lse && d_o && dq && dk && dv)
    fprintf(stderr,
            "dta_tree_attn_bwd_noalloc: bad arguments, or the tree's device metadata is not resident "
            "on device %d: call dta_tree_attn_prepare (which may allocate) first\n", dev);
  return st;
}
