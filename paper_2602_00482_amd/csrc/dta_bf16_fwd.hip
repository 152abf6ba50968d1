// bf16 forward tree attention for gfx950 (the attention inside the paper's FWD
// primitive, pseudocode appendix, for every segment of the tree in one launch).
//
// One block = 8 waves works on one query tile of the DFS-packed tree and one kv
// head.  Each wave owns 32 query rows of one q head of the group, so a K/V tile
// staged in LDS is shared by the whole GQA group, and everything a wave keeps
// fits in 256 registers: two waves per SIMD let the hardware overlap one
// wave's softmax arithmetic with the other's matrix products.  The block
// streams the key intervals of the tile's root path (full rectangles), then the
// tile's own keys (visibility mask k <= t < kend[k]), 64 keys at a time:
//   S^T = K Q^T  (32x32x16 bf16 MFMA, K rows from LDS, Q^T held in registers)
//   online softmax in fp32; in the transposed product every lane owns one
//   query column, so max / sum / rescale need one cross-lane exchange only
//   O^T += V^T P^T  (V columns via the transposing LDS read, P^T straight from
//   the S^T accumulators)
#include <hip/hip_runtime.h>

#include "dta_internal.h"
#include "dta_mfma.h"
#include "dta_queue.h"
#include "dta_tile_walk.h"

namespace dta {
namespace {

constexpr int kThreads = 512;

// max over both halves of the wave: lane l gets max(x[l], x[l ^ 32]).  The
// lane-half swap (v_permlane32_swap: upper 32 lanes of the first operand <->
// lower 32 lanes of the second) runs in the vector ALU, without the LDS round
// trip of a shuffle.
__device__ __forceinline__ float max_across_halves(float x) {
  const unsigned u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// kCh = keys per streamed chunk (one or two 64-row LDS tiles per operand): one
// barrier, one round of bookkeeping and one online-softmax step per chunk, so
// long key intervals run faster with 128, while every interval is padded to a
// multiple of the chunk, so forests of short segments want 64.
template <int kCh, int HD>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void fwd_bf16_kernel(
    const QTile* __restrict__ tiles, const KeySeg* __restrict__ segs,
    const int32_t* __restrict__ kend, const uint16_t* __restrict__ q,
    const uint16_t* __restrict__ k, const uint16_t* __restrict__ v, uint16_t* __restrict__ o,
    float* __restrict__ lse, int Hq, int Hkv, int HB, int hblocks, float scale,
    int* __restrict__ tickets, int n_items) {
  using TL = TileLayout<HD>;
  constexpr int kSub = kCh / 64, kTileElems = TL::kTileElems, kHeadDim = HD;
  constexpr int KS = TL::kSteps, DB = TL::kBlocks;   // k-steps over head_dim, 32-wide output blocks
  __shared__ __attribute__((aligned(1024))) uint16_t Ks[2][kSub][kTileElems];
  __shared__ __attribute__((aligned(1024))) uint16_t Vs[2][kSub][kTileElems];
  __shared__ __attribute__((aligned(16))) int32_t kendS[2][kCh];
  __shared__ int next_item[2];

  // tickets == nullptr: one (tile, kv head, head block) per block, from the block
  // index.  Otherwise resident blocks that draw (tile, head block) items from one
  // queue per kv head.
  ItemQueues queues;
  queues.init(tickets, n_items, Hkv);
  int item_idx = blockIdx.x / (Hkv * hblocks) * hblocks + (blockIdx.x % (Hkv * hblocks)) / Hkv;
  int g_idx = blockIdx.x % Hkv;
  if (tickets != nullptr && !queues.draw(next_item, item_idx, g_idx, false)) return;
  for (;;) {
  const QTile tile = tiles[item_idx / hblocks];
  const int g = g_idx, hblk = item_idx % hblocks;
  const int G = Hq / Hkv;
  const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
  const int c = l & 31, hh = l >> 5;
  const int h = g * G + hblk * HB + (w % HB);
  const int row_base = tile.t0 + 32 * (w / HB);
  // scores stay unscaled; the softmax scale (times log2 e) is folded into the
  // exponent.  A negative scale is moved into the sign of Q so that sc > 0.
  const float sc = fabsf(scale) * kLog2e;

  const int qrow = min(row_base + c, tile.t1 - 1);
  bf16x8 Qr[KS];
  {
    const uint16_t* qp = q + ((size_t)qrow * Hq + h) * kHeadDim + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      uint4 raw = *reinterpret_cast<const uint4*>(qp + 16 * ks);
      if (scale < 0.f) {
        raw.x ^= 0x80008000u; raw.y ^= 0x80008000u; raw.z ^= 0x80008000u; raw.w ^= 0x80008000u;
      }
      Qr[ks] = *reinterpret_cast<bf16x8*>(&raw);
    }
  }

  f32x16 O[DB];
#pragma unroll
  for (int a = 0; a < DB; ++a)
#pragma unroll
    for (int e = 0; e < 16; ++e) O[a][e] = 0.f;
  float m = -INFINITY, lsum = 0.f;   // running max of unscaled scores, partial row sum

  const size_t kv_stride = (size_t)Hkv * kHeadDim;
  const uint16_t* kbase = k + (size_t)g * kHeadDim;
  const uint16_t* vbase = v + (size_t)g * kHeadDim;
  const uint32_t kv_bytes = (uint32_t)kv_stride * 2;

  // Chunk i lives in buffer i & 1 and is copied global -> LDS one iteration ahead
  // of its use, so one barrier per chunk is enough.
  KeyChunksT<kCh> it;
  it.init(segs, tile);
  int c0, n, full;
  bool have = it.next(c0, n, full);
  auto issue = [&](int b) {
    if (!full || n < kCh) {   // rare: a chunk that needs the visibility mask
      if (threadIdx.x < kCh) {   // kendS is indexed by matrix position within each 64-key half
        const int row = 64 * (threadIdx.x >> 6) + TL::row_of_pos(threadIdx.x & 63);
        kendS[b][threadIdx.x] = row >= n ? 0 : (full ? 0x7fffffff : kend[c0 + row]);
      }
    }
#pragma unroll
    for (int sub = 0; sub < kSub; ++sub) {
      // a half with no valid key re-reads the chunk's first row (finite data the mask hides)
      const int nv = n - 64 * sub;
      const int r0 = nv > 0 ? c0 + 64 * sub : c0;
      const int nvalid = nv > 0 ? min(nv, 64) : 1;
      tile_async_load<kThreads, HD>(Ks[b][sub], kbase + (size_t)r0 * kv_stride, kv_bytes, nvalid);
      tile_async_load<kThreads, HD>(Vs[b][sub], vbase + (size_t)r0 * kv_stride, kv_bytes, nvalid);
    }
  };
  issue(0);
  int buf = 0;
  const int rlo = TL::row_lane_off(), clo = TL::col_lane_off();

  while (have) {
    async_wait_all();
    __syncthreads();   // chunk `buf` has landed; everyone is done with the other buffer
    const int cc0 = c0;
    const bool need_mask = !full || n < kCh;
    have = it.next(c0, n, full);
    if (have) issue(buf ^ 1);
    const uint16_t* Kt = Ks[buf][0] + rlo;
    const uint16_t* Vt = Vs[buf][0] + clo;

    // ---- S^T = K Q^T : 64 keys x 32 queries
    f32x16 S[2 * kSub];
#pragma unroll
    for (int a = 0; a < 2 * kSub; ++a)
#pragma unroll
      for (int e = 0; e < 16; ++e) S[a][e] = 0.f;
#pragma unroll
    for (int sub = 0; sub < kSub; ++sub)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 a0 = tile_row8(Kt + sub * kTileElems, 0, ks);
        const bf16x8 a1 = tile_row8(Kt + sub * kTileElems, 1, ks);
        S[2 * sub] = mfma32(a0, Qr[ks], S[2 * sub]);
        S[2 * sub + 1] = mfma32(a1, Qr[ks], S[2 * sub + 1]);
      }

    // ---- mask: key kv is visible to row t iff kv <= t < kend[kv]; kendS holds
    // 0 for padding keys and INT_MAX for keys every row of the tile sees (those
    // lie before the tile, so the causal test is true for them anyway)
    if (need_mask) {
#pragma unroll
      for (int mb = 0; mb < 2 * kSub; ++mb)
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
          const int kvl0 = 32 * mb + 8 * e4 + 4 * hh;
          const int4 ke = *reinterpret_cast<const int4*>(&kendS[buf][kvl0]);
          const int kev[4] = {ke.x, ke.y, ke.z, ke.w};
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const bool ok = (cc0 + 64 * (mb >> 1) + TL::row_of_acc(mb & 1, 4 * e4 + j, hh) <= qrow) & (qrow < kev[j]);
            S[mb][4 * e4 + j] = ok ? S[mb][4 * e4 + j] : -INFINITY;
          }
        }
    }

    // ---- online softmax, one query column per lane
    float mx = -INFINITY;
#pragma unroll
    for (int mb = 0; mb < 2 * kSub; ++mb)
#pragma unroll
      for (int e = 0; e < 16; ++e) mx = fmaxf(mx, S[mb][e]);
    mx = max_across_halves(mx);
    const float mnew = fmaxf(m, mx);
    const float mref = mnew == -INFINITY ? 0.f : mnew;
    const float alpha = __builtin_amdgcn_exp2f((m - mref) * sc);
    m = mnew;
    const float msc = mref * sc;
    float ps = 0.f;
    bf16x8 Pb[4 * kSub];
#pragma unroll
    for (int mb = 0; mb < 2 * kSub; ++mb) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const float p = __builtin_amdgcn_exp2f(fmaf(S[mb][e], sc, -msc));
        S[mb][e] = p;
        ps += p;
      }
      Pb[2 * mb] = pack8(S[mb], 0);
      Pb[2 * mb + 1] = pack8(S[mb], 1);
    }
    lsum = lsum * alpha + ps;
    // the accumulators are rescaled only when some row's running max moved
    if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0) {
#pragma unroll
      for (int dmb = 0; dmb < DB; ++dmb)
#pragma unroll
        for (int e = 0; e < 16; ++e) O[dmb][e] *= alpha;
    }

    // ---- O^T += V^T P^T
#pragma unroll
    for (int sub = 0; sub < kSub; ++sub)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
#pragma unroll
        for (int dmb = 0; dmb < DB; ++dmb) {
          const bf16x8 va = tile_col8(Vt + sub * kTileElems, 16 * kk, 32 * dmb);
          O[dmb] = mfma32(va, Pb[4 * sub + kk], O[dmb]);
        }
      }
    buf ^= 1;
  }

  // ---- normalise and store
  if (tickets != nullptr) queues.prefetch();
  const float lt = lsum + __shfl_xor(lsum, 32);
  const float inv = 1.f / lt;
  const int token = row_base + c;
  if (token < tile.t1) {
    uint16_t* op = o + ((size_t)token * Hq + h) * kHeadDim + 4 * hh;
#pragma unroll
    for (int dmb = 0; dmb < DB; ++dmb)
#pragma unroll
      for (int v4 = 0; v4 < 4; ++v4) {
        bf16x4 r;
#pragma unroll
        for (int e = 0; e < 4; ++e) r[e] = (__bf16)(O[dmb][4 * v4 + e] * inv);
        *reinterpret_cast<bf16x4*>(op + 32 * dmb + 8 * v4) = r;
      }
    if (hh == 0) lse[(size_t)token * Hq + h] = (m * sc + log2f(lt)) * kLn2;
  }
  if (tickets == nullptr || !queues.draw(next_item, item_idx, g_idx, true)) break;
  }   // next item
}

// Sets n ints to zero (the ticket counters; a fill kernel rather than a memset
// so that the launch sequence can be captured in a graph).
__global__ void zero_i32_kernel(int* __restrict__ p, int n) {
  for (int i = threadIdx.x; i < n; i += blockDim.x) p[i] = 0;
}

}  // namespace

int launch_fwd_bf16(const LaunchArgs& a) {
  hipStream_t st = (hipStream_t)a.stream;
  clear_hip_error();
  const size_t blocks = a.sched->q_tiles.size() * (size_t)a.p.n_kv_heads * (size_t)a.tc.hblocks;
  if (blocks == 0 || blocks > 0x7fffffffu) return DTA_ERR_UNSUPPORTED;
  // With a workspace for the counters and enough items, resident blocks draw the
  // items from per-head queues (see dta_queue.h); otherwise one block per item.
  const bool queues = a.tickets != nullptr && blocks >= 8 * (size_t)kNumCUs;
  if (queues) {
    zero_i32_kernel<<<1, 256, 0, st>>>(a.tickets, a.p.n_kv_heads);
    { int ls = launch_status(__func__); if (ls != DTA_OK) return ls; }
  }
  // chunk size: 128 keys when padding every key interval to 128 instead of 64 adds
  // at most 6 % to the keys streamed (measured: 5 % faster at +0.5 %, 1.4 % faster
  // at +5.6 %, 2 % slower at +9.6 %)
  const bool wide = 2 * a.sched->fwd_chunks128 * 100 <= a.sched->fwd_chunks64 * 106;
  auto kernel = a.p.head_dim == 128 ? (wide ? fwd_bf16_kernel<128, 128> : fwd_bf16_kernel<64, 128>)
                                    : (wide ? fwd_bf16_kernel<128, 64> : fwd_bf16_kernel<64, 64>);
  kernel<<<(unsigned)(queues ? (size_t)kNumCUs : blocks), kThreads, 0, st>>>(
      a.sched->d_q_tiles, a.sched->d_segs, a.d_kend, (const uint16_t*)a.q, (const uint16_t*)a.k,
      (const uint16_t*)a.v, (uint16_t*)a.o_out, a.lse_out, a.p.n_q_heads, a.p.n_kv_heads, a.tc.hb,
      a.tc.hblocks, a.p.softmax_scale, queues ? a.tickets : nullptr,
      (int)(a.sched->q_tiles.size() * (size_t)a.tc.hblocks));
  return launch_status(__func__);
}

}  // namespace dta
