// Matrix-pipe rate probe: what the bf16 MFMA pipes of this GPU deliver when
// nothing else limits them, and the shader clock they run at while doing so.
// A measurement helper for the roofline denominator: the attention kernels are
// priced against the published peak, and this gives the sustained figure the
// same chip reaches under the same power limit with the same instruction
// (v_mfma_f32_32x32x16_bf16), the same block shape (4 waves, two blocks per
// CU) and changing, non-trivial operands.
#include "dta_probe.h"
#include "dta_mfma.h"

namespace dta {

constexpr int kProbeThreads = 256;
constexpr int kProbeProductsPerIter = 16;

// Every wave keeps four independent 32x32 accumulators and four A and four B
// operand registers sets, and issues 16 products per iteration (each A with
// each B, a different accumulator for consecutive products so that no product
// waits for the previous one).  No memory traffic inside the loop.
__global__ __launch_bounds__(kProbeThreads, 2) void mfma_rate_kernel(float* __restrict__ out,
                                                                     uint64_t* __restrict__ ticks, int iters) {
  uint32_t s = (blockIdx.x * kProbeThreads + threadIdx.x) * 2654435761u + 12345u;
  bf16x8 a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      // values on a grid of 1/64 in [-2, 2): exact in bf16, every mantissa bit in use
      s = s * 1664525u + 1013904223u;
      a[i][e] = (__bf16)(((int)((s >> 16) & 0xff) - 128) * (1.0f / 64.0f));
      s = s * 1664525u + 1013904223u;
      b[i][e] = (__bf16)(((int)((s >> 16) & 0xff) - 128) * (1.0f / 64.0f));
    }
  f32x16 acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[j][v] = 0.0f;

  const uint64_t c0 = clock64();
  const uint64_t r0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] = mfma32(a[i], b[(i + j) & 3], acc[j]);
  }
  const uint64_t c1 = clock64();
  const uint64_t r1 = wall_clock64();

  float sum = 0.0f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) sum += acc[j][v];
  out[(size_t)blockIdx.x * kProbeThreads + threadIdx.x] = sum;
  if (threadIdx.x == 0) {
    ticks[2 * (size_t)blockIdx.x] = c1 - c0;
    ticks[2 * (size_t)blockIdx.x + 1] = r1 - r0;
  }
}

// Do the matrix products of one wave and the vector-ALU work of ANOTHER wave on
// the same SIMD overlap?  Block = 8 waves, two per SIMD (wave i runs on SIMD
// i % 4): waves 0-3 do mfma_iters x 16 independent products, waves 4-7 do
// valu_iters x 64 independent v_exp_f32.  Registers only.  Timed three times by
// the caller (products only, exponentials only, both), it shows how much of
// the shorter part the hardware can hide behind the longer one, which bounds
// what any schedule of the attention kernels can reach.
constexpr int kOverlapThreads = 512;

__global__ __launch_bounds__(kOverlapThreads) void overlap_kernel(float* __restrict__ out, int mfma_iters,
                                                                  int valu_iters) {
  const int w = threadIdx.x >> 6;
  float acc = 0.f;
  if (w < 4) {
    bf16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      a[e] = (__bf16)(0.01f * (float)(threadIdx.x % 7 + e));
      b[e] = (__bf16)(0.02f * (float)(threadIdx.x % 5 + e));
    }
    f32x16 c[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) c[j][e] = 0.f;
    for (int it = 0; it < mfma_iters; ++it)
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int j = 0; j < 4; ++j) c[j] = mfma32(a, b, c[j]);
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc += c[j][e];
  } else {
    float x[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) x[i] = 0.001f * (float)(threadIdx.x + i);
    for (int it = 0; it < valu_iters; ++it)
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int i = 0; i < 16; ++i) x[i] = __builtin_amdgcn_exp2f(-x[i]);   // stays in (0.5, 1]
#pragma unroll
    for (int i = 0; i < 16; ++i) acc += x[i];
  }
  out[(size_t)blockIdx.x * kOverlapThreads + threadIdx.x] = acc;
}

}  // namespace dta

extern "C" int dta_probe_overlap(int32_t n_blocks, int32_t mfma_iters, int32_t valu_iters, float* out,
                                 void* hip_stream) {
  if (n_blocks < 1 || n_blocks > (1 << 20) || mfma_iters < 0 || valu_iters < 0 || mfma_iters > (1 << 24) ||
      valu_iters > (1 << 24) || !out)
    return DTA_ERR_INVALID_ARG;
  (void)hipGetLastError();
  hipLaunchKernelGGL(dta::overlap_kernel, dim3(n_blocks), dim3(dta::kOverlapThreads), 0, (hipStream_t)hip_stream, out,
                     mfma_iters, valu_iters);
  return hipGetLastError() == hipSuccess ? DTA_OK : DTA_ERR_HIP;
}

extern "C" int dta_probe_mfma_bf16(int32_t n_blocks, int32_t iters, float* out, uint64_t* ticks, void* hip_stream,
                                   int64_t* flop, int32_t* wall_clock_khz) {
  if (n_blocks < 1 || n_blocks > (1 << 20) || iters < 1 || iters > (1 << 24) || !out || !ticks) return DTA_ERR_INVALID_ARG;
  (void)hipGetLastError();
  hipLaunchKernelGGL(dta::mfma_rate_kernel, dim3(n_blocks), dim3(dta::kProbeThreads), 0, (hipStream_t)hip_stream, out,
                     ticks, iters);
  if (hipGetLastError() != hipSuccess) return DTA_ERR_HIP;
  if (wall_clock_khz) {
    int dev = 0, khz = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess)
      return DTA_ERR_HIP;
    *wall_clock_khz = khz;
  }
  if (flop)
    *flop = (int64_t)n_blocks * (dta::kProbeThreads / 64) * iters * dta::kProbeProductsPerIter * (2LL * 32 * 32 * 16);
  return DTA_OK;
}
