// bf16 forward tree attention for gfx950 (the attention inside the paper's FWD
// primitive, pseudocode appendix, for every segment of the tree in one launch).
//
// One block = 4 waves works on one query tile of the DFS-packed tree and one kv
// head.  Each wave owns 64 query rows of one q head of the group, so a K/V tile
// staged in LDS is shared by the whole GQA group.  The block streams the key
// intervals of the tile's root path (full rectangles), then the tile's own
// keys (visibility mask k <= t < kend[k]), 64 keys at a time:
//   S^T = K Q^T  (32x32x16 bf16 MFMA, K rows from LDS, Q^T held in registers)
//   online softmax in fp32; in the transposed product every lane owns one
//   query column, so max / sum / rescale need one cross-lane exchange only
//   O^T += V^T P^T  (V columns via the transposing LDS read, P^T straight from
//   the S^T accumulators)
#include <hip/hip_runtime.h>

#include "dta_internal.h"
#include "dta_mfma.h"

namespace dta {
namespace {

constexpr int kBN = 64;  // keys per streamed tile

// Walks the key intervals of a query tile in 64-key chunks: root-path pieces
// first, the tile's own range last.
struct KeyChunks {
  const KeySeg* segs;
  int si, seg_end, t0, t1;
  int cur, end, full;
  __device__ __forceinline__ void load_seg() {
    if (si < seg_end) {
      cur = segs[si].start; end = segs[si].end; full = segs[si].full;
    } else {
      cur = t0; end = t1; full = 0;
    }
  }
  __device__ __forceinline__ void init(const KeySeg* s, const QTile& t) {
    segs = s; si = t.seg_begin; seg_end = t.seg_end; t0 = t.t0; t1 = t.t1;
    load_seg();
  }
  __device__ __forceinline__ bool next(int& c0, int& n, int& is_full) {
    if (si > seg_end) return false;
    c0 = cur; n = min(kBN, end - cur); is_full = full;
    cur += kBN;
    if (cur >= end) { ++si; if (si <= seg_end) load_seg(); }
    return true;
  }
};

__global__ __launch_bounds__(256) void fwd_bf16_kernel(
    const QTile* __restrict__ tiles, const KeySeg* __restrict__ segs,
    const int32_t* __restrict__ kend, const uint16_t* __restrict__ q,
    const uint16_t* __restrict__ k, const uint16_t* __restrict__ v, uint16_t* __restrict__ o,
    float* __restrict__ lse, int Hq, int Hkv, int HB, int hblocks, float scale) {
  __shared__ __attribute__((aligned(16))) uint16_t Ks[kBN * kPitch];
  __shared__ __attribute__((aligned(16))) uint16_t Vs[kBN * kPitch];
  __shared__ int32_t kendS[kBN];

  const int inner = blockIdx.x % (Hkv * hblocks);
  const QTile tile = tiles[blockIdx.x / (Hkv * hblocks)];
  const int g = inner % Hkv, hblk = inner / Hkv;
  const int G = Hq / Hkv;
  const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
  const int c = l & 31, hh = l >> 5;
  const int h = g * G + hblk * HB + (w % HB);
  const int row_base = tile.t0 + 64 * (w / HB);
  const float sc = scale * kLog2e;

  int qrow[2];
  bf16x8 Qr[2][8];
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    qrow[nb] = min(row_base + 32 * nb + c, tile.t1 - 1);
    const uint16_t* qp = q + ((size_t)qrow[nb] * Hq + h) * kHeadDim + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) Qr[nb][ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks);
  }

  f32x16 O[4][2];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) O[a][b][e] = 0.f;
  float m[2] = {-INFINITY, -INFINITY}, lsum[2] = {0.f, 0.f};

  const size_t kv_stride = (size_t)Hkv * kHeadDim;
  const uint16_t* kbase = k + (size_t)g * kHeadDim;
  const uint16_t* vbase = v + (size_t)g * kHeadDim;

  KeyChunks it;
  it.init(segs, tile);
  int c0, n, full;
  bool have = it.next(c0, n, full);
  TileRegs kreg, vreg;
  tile_load(kreg, kbase + (size_t)c0 * kv_stride, kv_stride, n);
  tile_load(vreg, vbase + (size_t)c0 * kv_stride, kv_stride, n);

  while (have) {
    __syncthreads();
    tile_store(kreg, Ks);
    tile_store(vreg, Vs);
    if (!full && threadIdx.x < kBN) kendS[threadIdx.x] = threadIdx.x < n ? kend[c0 + threadIdx.x] : 0;
    __syncthreads();
    const int cc0 = c0, cn = n, cfull = full;
    have = it.next(c0, n, full);
    if (have) {
      tile_load(kreg, kbase + (size_t)c0 * kv_stride, kv_stride, n);
      tile_load(vreg, vbase + (size_t)c0 * kv_stride, kv_stride, n);
    }

    // ---- S^T = K Q^T
    f32x16 S[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int e = 0; e < 16; ++e) S[a][b][e] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const bf16x8 a0 = lds_read_row8(Ks + c * kPitch + 16 * ks + 8 * hh);
      const bf16x8 a1 = lds_read_row8(Ks + (32 + c) * kPitch + 16 * ks + 8 * hh);
      S[0][0] = mfma32(a0, Qr[0][ks], S[0][0]);
      S[0][1] = mfma32(a0, Qr[1][ks], S[0][1]);
      S[1][0] = mfma32(a1, Qr[0][ks], S[1][0]);
      S[1][1] = mfma32(a1, Qr[1][ks], S[1][1]);
    }

    // ---- scale, mask
    const bool need_mask = !cfull || cn < kBN;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int e = 0; e < 16; ++e) S[mb][nb][e] *= sc;
    if (need_mask) {
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int kvl = 32 * mb + 8 * (e / 4) + 4 * hh + (e % 4);
          const int kv = cc0 + kvl;
          const int ke = cfull ? 0x7fffffff : kendS[kvl];
#pragma unroll
          for (int nb = 0; nb < 2; ++nb) {
            const bool ok = kvl < cn && (cfull || kv <= qrow[nb]) && qrow[nb] < ke;
            if (!ok) S[mb][nb][e] = -INFINITY;
          }
        }
    }

    // ---- online softmax, one query column per lane
    bf16x8 Pb[2][4];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      float mx = -INFINITY;
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int e = 0; e < 16; ++e) mx = fmaxf(mx, S[mb][nb][e]);
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float mnew = fmaxf(m[nb], mx);
      const float mref = mnew == -INFINITY ? 0.f : mnew;
      const float alpha = __builtin_amdgcn_exp2f(m[nb] - mref);
      m[nb] = mnew;
      float ps = 0.f;
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const float p = __builtin_amdgcn_exp2f(S[mb][nb][e] - mref);
          S[mb][nb][e] = p;
          ps += p;
        }
        Pb[nb][2 * mb] = pack8(S[mb][nb], 0);
        Pb[nb][2 * mb + 1] = pack8(S[mb][nb], 1);
      }
      lsum[nb] = lsum[nb] * alpha + ps;
#pragma unroll
      for (int dmb = 0; dmb < 4; ++dmb)
#pragma unroll
        for (int e = 0; e < 16; ++e) O[dmb][nb][e] *= alpha;
    }

    // ---- O^T += V^T P^T
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
#pragma unroll
      for (int dmb = 0; dmb < 4; ++dmb) {
        const bf16x8 va = lds_read_col8(Vs, 16 * kk, 32 * dmb);
        O[dmb][0] = mfma32(va, Pb[0][kk], O[dmb][0]);
        O[dmb][1] = mfma32(va, Pb[1][kk], O[dmb][1]);
      }
    }
  }

  // ---- normalise and store
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    const float lt = lsum[nb] + __shfl_xor(lsum[nb], 32);
    const float inv = 1.f / lt;
    const int token = row_base + 32 * nb + c;
    if (token < tile.t1) {
      uint16_t* op = o + ((size_t)token * Hq + h) * kHeadDim + 4 * hh;
#pragma unroll
      for (int dmb = 0; dmb < 4; ++dmb)
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4) {
          bf16x4 r;
#pragma unroll
          for (int e = 0; e < 4; ++e) r[e] = (__bf16)(O[dmb][nb][4 * v4 + e] * inv);
          *reinterpret_cast<bf16x4*>(op + 32 * dmb + 8 * v4) = r;
        }
      if (hh == 0) lse[(size_t)token * Hq + h] = (m[nb] + log2f(lt)) * kLn2;
    }
  }
}

}  // namespace

int launch_fwd_bf16(const LaunchArgs& a) {
  hipStream_t st = (hipStream_t)a.stream;
  clear_hip_error();
  const size_t blocks = a.sched->q_tiles.size() * (size_t)a.p.n_kv_heads * (size_t)a.tc.hblocks;
  if (blocks == 0 || blocks > 0x7fffffffu) return DTA_ERR_UNSUPPORTED;
  fwd_bf16_kernel<<<(unsigned)blocks, 256, 0, st>>>(
      a.sched->d_q_tiles, a.sched->d_segs, a.d_kend, (const uint16_t*)a.q, (const uint16_t*)a.k,
      (const uint16_t*)a.v, (uint16_t*)a.o_out, a.lse_out, a.p.n_q_heads, a.p.n_kv_heads, a.tc.hb,
      a.tc.hblocks, a.p.softmax_scale);
  return launch_status(__func__);
}

}  // namespace dta
