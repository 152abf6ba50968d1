// fp32 tree attention for gfx950: forward, dQ and dK/dV kernels that keep every
// product, sum and exponential in fp32 (no matrix-core truncation), for callers
// that need ~1e-6 relative accuracy.  Four lanes share one query (or key) row,
// each holding a quarter of head_dim; keys (or queries) are streamed through LDS
// and every lane group walks them one by one.
//
// What is computed follows the attention inside the paper's FWD / BWD
// primitives (pseudocode appendix) for all segments of the tree at once: a
// query sees key k iff  k <= t < kend[k]  in packed DFS coordinates.
#include <hip/hip_runtime.h>

#include "dta_internal.h"

namespace dta {
namespace {

constexpr int kRows = 64;   // rows (queries or keys) per block
constexpr int kLanes = 4;   // lanes per row
constexpr int kChunk = 32;  // streamed rows per LDS fill

__device__ __forceinline__ float group_sum(float x) {
  x += __shfl_xor(x, 1);
  x += __shfl_xor(x, 2);
  return x;
}

// Copies `n` rows of D floats (row stride `stride` floats) into LDS, all 256 threads.
template <int D>
__device__ __forceinline__ void stage_rows(float (*dst)[D], const float* src, size_t stride, int n) {
  constexpr int V = D / 4;
  for (int i = threadIdx.x; i < n * V; i += blockDim.x) {
    int r = i / V, c = i % V;
    reinterpret_cast<float4*>(dst[r])[c] =
        *reinterpret_cast<const float4*>(src + (size_t)r * stride + 4 * c);
  }
}

template <int D>
__global__ __launch_bounds__(256) void fwd_f32_kernel(const QTile* __restrict__ tiles,
                                                      const KeySeg* __restrict__ segs,
                                                      const int32_t* __restrict__ kend,
                                                      const float* __restrict__ q,
                                                      const float* __restrict__ k,
                                                      const float* __restrict__ v,
                                                      float* __restrict__ o, float* __restrict__ lse,
                                                      int Hq, int Hkv, float scale) {
  constexpr int DS = D / kLanes;
  __shared__ float Ks[kChunk][D];
  __shared__ float Vs[kChunk][D];
  __shared__ int32_t kendS[kChunk];
  const QTile tile = tiles[blockIdx.x];
  const int h = blockIdx.y, g = h / (Hq / Hkv);
  const int r = threadIdx.x / kLanes, j = threadIdx.x % kLanes;
  const int t = tile.t0 + r;
  const bool valid = t < tile.t1;
  const int tc = valid ? t : tile.t1 - 1;

  float qv[DS], acc[DS];
  {
    const float* qp = q + ((size_t)tc * Hq + h) * D + j * DS;
#pragma unroll
    for (int i = 0; i < DS; ++i) { qv[i] = qp[i]; acc[i] = 0.f; }
  }
  float m = -INFINITY, l = 0.f;
  const size_t kv_stride = (size_t)Hkv * D;

  for (int si = tile.seg_begin; si <= tile.seg_end; ++si) {
    int start, end, full;
    if (si < tile.seg_end) { start = segs[si].start; end = segs[si].end; full = segs[si].full; }
    else { start = tile.t0; end = tile.t1; full = 0; }   // the tile's own keys
    for (int c0 = start; c0 < end; c0 += kChunk) {
      const int n = min(kChunk, end - c0);
      __syncthreads();
      stage_rows<D>(Ks, k + (size_t)c0 * kv_stride + (size_t)g * D, kv_stride, n);
      stage_rows<D>(Vs, v + (size_t)c0 * kv_stride + (size_t)g * D, kv_stride, n);
      if (threadIdx.x < n) kendS[threadIdx.x] = kend[c0 + threadIdx.x];
      __syncthreads();
      for (int i = 0; i < n; ++i) {
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < DS; ++e) s = fmaf(qv[e], Ks[i][j * DS + e], s);
        s = group_sum(s) * scale;
        const bool vis = full || (c0 + i <= tc && tc < kendS[i]);
        if (vis) {
          const float mn = fmaxf(m, s);
          const float a = expf(m - mn), p = expf(s - mn);
          l = l * a + p;
#pragma unroll
          for (int e = 0; e < DS; ++e) acc[e] = fmaf(acc[e], a, p * Vs[i][j * DS + e]);
          m = mn;
        }
      }
    }
  }
  if (valid) {
    const float inv = 1.f / l;
    float* op = o + ((size_t)t * Hq + h) * D + j * DS;
#pragma unroll
    for (int i = 0; i < DS; ++i) op[i] = acc[i] * inv;
    if (j == 0) lse[(size_t)t * Hq + h] = m + logf(l);
  }
}

// D[t,h] = dO[t,h] . O[t,h]
template <int D>
__global__ __launch_bounds__(256) void delta_f32_kernel(const float* __restrict__ o,
                                                        const float* __restrict__ d_o,
                                                        float* __restrict__ delta, size_t rows) {
  constexpr int DS = D / kLanes;
  size_t row = (size_t)blockIdx.x * kRows + threadIdx.x / kLanes;
  int j = threadIdx.x % kLanes;
  float s = 0.f;
  if (row < rows) {
    const float* a = o + row * D + j * DS;
    const float* b = d_o + row * D + j * DS;
#pragma unroll
    for (int i = 0; i < DS; ++i) s = fmaf(a[i], b[i], s);
  }
  s = group_sum(s);
  if (row < rows && j == 0) delta[row] = s;
}

template <int D>
__global__ __launch_bounds__(256) void dq_f32_kernel(const QTile* __restrict__ tiles,
                                                     const KeySeg* __restrict__ segs,
                                                     const int32_t* __restrict__ kend,
                                                     const float* __restrict__ q,
                                                     const float* __restrict__ k,
                                                     const float* __restrict__ v,
                                                     const float* __restrict__ d_o,
                                                     const float* __restrict__ lse,
                                                     const float* __restrict__ delta,
                                                     float* __restrict__ dq, int Hq, int Hkv,
                                                     float scale) {
  constexpr int DS = D / kLanes;
  __shared__ float Ks[kChunk][D];
  __shared__ float Vs[kChunk][D];
  __shared__ int32_t kendS[kChunk];
  const QTile tile = tiles[blockIdx.x];
  const int h = blockIdx.y, g = h / (Hq / Hkv);
  const int r = threadIdx.x / kLanes, j = threadIdx.x % kLanes;
  const int t = tile.t0 + r;
  const bool valid = t < tile.t1;
  const int tc = valid ? t : tile.t1 - 1;

  float qv[DS], dov[DS], acc[DS];
  {
    const size_t base = ((size_t)tc * Hq + h) * D + j * DS;
#pragma unroll
    for (int i = 0; i < DS; ++i) { qv[i] = q[base + i]; dov[i] = d_o[base + i]; acc[i] = 0.f; }
  }
  const float lse_t = lse[(size_t)tc * Hq + h], delta_t = delta[(size_t)tc * Hq + h];
  const size_t kv_stride = (size_t)Hkv * D;

  for (int si = tile.seg_begin; si <= tile.seg_end; ++si) {
    int start, end, full;
    if (si < tile.seg_end) { start = segs[si].start; end = segs[si].end; full = segs[si].full; }
    else { start = tile.t0; end = tile.t1; full = 0; }
    for (int c0 = start; c0 < end; c0 += kChunk) {
      const int n = min(kChunk, end - c0);
      __syncthreads();
      stage_rows<D>(Ks, k + (size_t)c0 * kv_stride + (size_t)g * D, kv_stride, n);
      stage_rows<D>(Vs, v + (size_t)c0 * kv_stride + (size_t)g * D, kv_stride, n);
      if (threadIdx.x < n) kendS[threadIdx.x] = kend[c0 + threadIdx.x];
      __syncthreads();
      for (int i = 0; i < n; ++i) {
        float s = 0.f, dp = 0.f;
#pragma unroll
        for (int e = 0; e < DS; ++e) {
          s = fmaf(qv[e], Ks[i][j * DS + e], s);
          dp = fmaf(dov[e], Vs[i][j * DS + e], dp);
        }
        s = group_sum(s) * scale;
        dp = group_sum(dp);
        const bool vis = full || (c0 + i <= tc && tc < kendS[i]);
        const float p = vis ? expf(s - lse_t) : 0.f;
        const float ds = p * (dp - delta_t);
#pragma unroll
        for (int e = 0; e < DS; ++e) acc[e] = fmaf(ds, Ks[i][j * DS + e], acc[e]);
      }
    }
  }
  if (valid) {
    float* op = dq + ((size_t)t * Hq + h) * D + j * DS;
#pragma unroll
    for (int i = 0; i < DS; ++i) op[i] = acc[i] * scale;
  }
}

// One block owns kRows consecutive keys of one kv head and walks every query
// row that can see any of them, for all q heads of the group, so each dK/dV
// element is produced by exactly one lane group and written once.
template <int D>
__global__ __launch_bounds__(256) void dkdv_f32_kernel(const KvTile* __restrict__ tiles,
                                                       const int32_t* __restrict__ kend,
                                                       const float* __restrict__ q,
                                                       const float* __restrict__ k,
                                                       const float* __restrict__ v,
                                                       const float* __restrict__ d_o,
                                                       const float* __restrict__ lse,
                                                       const float* __restrict__ delta,
                                                       float* __restrict__ dk, float* __restrict__ dv,
                                                       int accumulate, int Hq, int Hkv,
                                                       float scale) {
  constexpr int DS = D / kLanes;
  __shared__ float Qs[kChunk][D];
  __shared__ float dOs[kChunk][D];
  __shared__ float lseS[kChunk], deltaS[kChunk];
  const KvTile tile = tiles[blockIdx.x];
  const int g = blockIdx.y, G = Hq / Hkv;
  const int r = threadIdx.x / kLanes, j = threadIdx.x % kLanes;
  const int kk = tile.k0 + r;
  const bool valid = kk < tile.k1;
  const int kc = valid ? kk : tile.k1 - 1;
  const int my_kend = kend[kc];

  float kv_[DS], vv[DS], dka[DS], dva[DS];
  {
    const size_t base = ((size_t)kc * Hkv + g) * D + j * DS;
#pragma unroll
    for (int i = 0; i < DS; ++i) { kv_[i] = k[base + i]; vv[i] = v[base + i]; dka[i] = 0.f; dva[i] = 0.f; }
  }
  const size_t q_stride = (size_t)Hq * D;

  for (int hh = 0; hh < G; ++hh) {
    const int h = g * G + hh;
    for (int c0 = tile.q_begin; c0 < tile.q_end; c0 += kChunk) {
      const int n = min(kChunk, tile.q_end - c0);
      __syncthreads();
      stage_rows<D>(Qs, q + (size_t)c0 * q_stride + (size_t)h * D, q_stride, n);
      stage_rows<D>(dOs, d_o + (size_t)c0 * q_stride + (size_t)h * D, q_stride, n);
      if (threadIdx.x < n) {
        lseS[threadIdx.x] = lse[(size_t)(c0 + threadIdx.x) * Hq + h];
        deltaS[threadIdx.x] = delta[(size_t)(c0 + threadIdx.x) * Hq + h];
      }
      __syncthreads();
      for (int i = 0; i < n; ++i) {
        const int t = c0 + i;
        float s = 0.f, dp = 0.f;
#pragma unroll
        for (int e = 0; e < DS; ++e) {
          s = fmaf(Qs[i][j * DS + e], kv_[e], s);
          dp = fmaf(dOs[i][j * DS + e], vv[e], dp);
        }
        s = group_sum(s) * scale;
        dp = group_sum(dp);
        const bool vis = kc <= t && t < my_kend;
        const float p = vis ? expf(s - lseS[i]) : 0.f;
        const float ds = p * (dp - deltaS[i]);
#pragma unroll
        for (int e = 0; e < DS; ++e) {
          dva[e] = fmaf(p, dOs[i][j * DS + e], dva[e]);
          dka[e] = fmaf(ds, Qs[i][j * DS + e], dka[e]);
        }
      }
    }
  }
  if (valid) {
    const size_t base = ((size_t)kk * Hkv + g) * D + j * DS;
#pragma unroll
    for (int i = 0; i < DS; ++i) {
      // a segment call adds to the caller's accumulators (this lane group is the
      // only owner of the key in the launch)
      dk[base + i] = (accumulate ? dk[base + i] : 0.f) + dka[i] * scale;
      dv[base + i] = (accumulate ? dv[base + i] : 0.f) + dva[i];
    }
  }
}

template <int D>
int fwd_impl(const LaunchArgs& a) {
  hipStream_t st = (hipStream_t)a.stream;
  clear_hip_error();
  dim3 grid((unsigned)a.sched->q_tiles.size(), (unsigned)a.p.n_q_heads);
  fwd_f32_kernel<D><<<grid, 256, 0, st>>>(a.sched->d_q_tiles, a.sched->d_segs, a.d_kend,
                                          (const float*)a.q, (const float*)a.k, (const float*)a.v,
                                          (float*)a.o_out, a.lse_out, a.p.n_q_heads, a.p.n_kv_heads,
                                          a.p.softmax_scale);
  return launch_status(__func__);
}

template <int D>
int bwd_impl(const LaunchArgs& a) {
  hipStream_t st = (hipStream_t)a.stream;
  clear_hip_error();
  const size_t row0 = (size_t)a.row_begin * a.p.n_q_heads;
  const size_t rows = (size_t)(a.row_end - a.row_begin) * a.p.n_q_heads;
  if (a.stages & DTA_BWD_DELTA) {
    delta_f32_kernel<D><<<(unsigned)((rows + kRows - 1) / kRows), 256, 0, st>>>(
        (const float*)a.o + row0 * D, (const float*)a.d_o + row0 * D, a.delta + row0, rows);
    { int ls = launch_status(__func__); if (ls != DTA_OK) return ls; }
  }
  if (a.stages & DTA_BWD_DQ) {
    dim3 gq((unsigned)a.sched->q_tiles.size(), (unsigned)a.p.n_q_heads);
    dq_f32_kernel<D><<<gq, 256, 0, st>>>(a.sched->d_q_tiles, a.sched->d_segs, a.d_kend,
                                         (const float*)a.q, (const float*)a.k, (const float*)a.v,
                                         (const float*)a.d_o, a.lse_in, a.delta, (float*)a.dq,
                                         a.p.n_q_heads, a.p.n_kv_heads, a.p.softmax_scale);
    { int ls = launch_status(__func__); if (ls != DTA_OK) return ls; }
  }
  if (a.stages & DTA_BWD_DKDV) {
    dim3 gk((unsigned)a.sched->kv_tiles.size(), (unsigned)a.p.n_kv_heads);
    dkdv_f32_kernel<D><<<gk, 256, 0, st>>>(a.sched->d_kv_tiles, a.d_kend, (const float*)a.q,
                                           (const float*)a.k, (const float*)a.v,
                                           (const float*)a.d_o, a.lse_in, a.delta,
                                           a.dk_acc ? a.dk_acc : (float*)a.dk,
                                           a.dk_acc ? a.dv_acc : (float*)a.dv, a.dk_acc != nullptr,
                                           a.p.n_q_heads, a.p.n_kv_heads, a.p.softmax_scale);
    { int ls = launch_status(__func__); if (ls != DTA_OK) return ls; }
  }
  return DTA_OK;
}

}  // namespace

int launch_fwd_f32(const LaunchArgs& a) {
  return a.p.head_dim == 64 ? fwd_impl<64>(a) : fwd_impl<128>(a);
}
int launch_bwd_f32(const LaunchArgs& a) {
  return a.p.head_dim == 64 ? bwd_impl<64>(a) : bwd_impl<128>(a);
}

}  // namespace dta
