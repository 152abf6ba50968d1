// bf16 backward tree attention for gfx950 (the attention inside the paper's BWD
// primitive, pseudocode appendix; gradients of every descendant query are
// accumulated into a shared key/value, pop step of section 3.1).
//
// Three launches, no atomics, every output element written exactly once:
//   delta  D[t,h] = dO[t,h] . O[t,h]
//   dQ     query-stationary: same tile walk as the forward kernel; per 64-key
//          tile S^T = K Q^T, P^T = exp(S^T - LSE), dP^T = V dO^T,
//          dS^T = P^T (dP^T - D), dQ^T += K^T dS^T
//   dK/dV  key-stationary: a block owns 128 consecutive packed keys of one kv
//          head (32 per wave, K and V rows held in registers) and walks the
//          contiguous query range [k0, q_end) that can see them, in reverse
//          DFS sense "all descendants", for all q heads of the group:
//          S = Q K^T, dP = dO V^T, dV^T += dO^T P, dK^T += Q^T dS
// Products run on the 32x32x16 bf16 MFMA with fp32 accumulation; operands that
// must be read along tile rows come from the transposing LDS read.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "dta_internal.h"
#include "dta_mfma.h"
#include "dta_queue.h"
#include "dta_tile_walk.h"

namespace dta {
namespace {

constexpr int kBQ = 64;   // query rows per streamed tile in the dK/dV kernel

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) {
  return __uint_as_float((uint32_t)b << 16);
}

// HD / 8 lanes per (token, head) row, 8 elements each.
template <int HD>
__global__ __launch_bounds__(256) void delta_bf16_kernel(const uint16_t* __restrict__ o,
                                                         const uint16_t* __restrict__ d_o,
                                                         const float* __restrict__ lse,
                                                         float* __restrict__ neg_delta,
                                                         float* __restrict__ neg_lse_s,
                                                         float inv_scale, size_t rows) {
  constexpr int kLanes = HD / 8, kRows = 256 / kLanes;   // per row, per block
  const size_t row = (size_t)blockIdx.x * kRows + threadIdx.x / kLanes;
  const int j = threadIdx.x % kLanes;
  float s = 0.f;
  if (row < rows) {
    const uint4 a = *reinterpret_cast<const uint4*>(o + row * HD + 8 * j);
    const uint4 b = *reinterpret_cast<const uint4*>(d_o + row * HD + 8 * j);
    const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      s = fmaf(bf16_bits_to_float((uint16_t)(aw[i] & 0xffff)), bf16_bits_to_float((uint16_t)(bw[i] & 0xffff)), s);
      s = fmaf(bf16_bits_to_float((uint16_t)(aw[i] >> 16)), bf16_bits_to_float((uint16_t)(bw[i] >> 16)), s);
    }
  }
  s += __shfl_xor(s, 1);
  s += __shfl_xor(s, 2);
  s += __shfl_xor(s, 4);
  if (HD == 128) s += __shfl_xor(s, 8);
  // Stored negated, and lse divided by the softmax scale: the dK/dV kernel
  // starts its score and dP accumulators from these values, so that
  // P = exp(scale * acc) and dS = P * acc need no further subtraction.
  if (row < rows && j == 0) {
    neg_delta[row] = -s;
    neg_lse_s[row] = -lse[row] * inv_scale;
  }
}

constexpr int kDqThreads = 512;

// Query-stationary dQ: 8 waves, each 32 query rows of one q head (same walk and
// wave layout as the forward kernel).
template <int HD>
__global__ __launch_bounds__(kDqThreads) void dq_bf16_kernel(
    const QTile* __restrict__ tiles, const KeySeg* __restrict__ segs,
    const int32_t* __restrict__ kend, const uint16_t* __restrict__ q,
    const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const uint16_t* __restrict__ d_o, const float* __restrict__ lse,
    const uint16_t* __restrict__ o, float* __restrict__ neg_delta, float* __restrict__ neg_lse_s,
    uint16_t* __restrict__ dq, int Hq, int Hkv, int HB, int hblocks, float scale,
    int* __restrict__ tickets, int n_items) {
  using TL = TileLayout<HD>;
  constexpr int kTileElems = TL::kTileElems, kHeadDim = HD;
  constexpr int KS = TL::kSteps;   // products per phase: k-steps over head_dim = 2 x output blocks
  __shared__ __attribute__((aligned(1024))) uint16_t Ks[2][kTileElems];
  __shared__ __attribute__((aligned(1024))) uint16_t Vs[2][kTileElems];
  __shared__ __attribute__((aligned(16))) int32_t kendS[2][kKeyChunk];
  // With head_dim 128 the last two k-steps of this wave's Q and dO operands live in
  // LDS instead of registers (each lane reads back what it wrote): with all 16 in
  // registers the kernel needs a few more than 256, and reloads from scratch
  // memory would wait for, i.e. serialise, the tile copies in flight.
  constexpr int kReg = HD == 128 ? 6 : KS;
  constexpr int kStash = KS - kReg;
  __shared__ __attribute__((aligned(16))) uint16_t stashS[kDqThreads / 64][kStash ? 2 * kStash : 1][64 * 8];

  // Which (query tile, head block, kv head) this block works on.  tickets ==
  // nullptr: the block index says so.  Otherwise every block draws ONE item from
  // the queues (its home head's first, blockIdx mod Hkv, then the others') and the
  // grid holds a quarter more blocks than there are items; blocks that find the
  // queues empty leave at once.  The hardware gives every XCD the same number of
  // blocks, so this is what lets an XCD that runs faster do more of the items
  // (a loop over items inside the block, as in the other two kernels, costs this
  // kernel its register allocation).
  int item_idx = blockIdx.x / Hkv, g_idx = blockIdx.x % Hkv;
  if (tickets != nullptr) {
    ItemQueues queues;
    queues.init(tickets, n_items, Hkv);
    if (!queues.draw(reinterpret_cast<int*>(&kendS[0][0]), item_idx, g_idx, false)) return;
    __syncthreads();   // the slot is part of kendS: nobody may still be reading it below
  }
  const QTile tile = tiles[item_idx / hblocks];
  const int g = g_idx, hblk = item_idx % hblocks;
  const int G = Hq / Hkv;
  const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
  const int c = l & 31, hh = l >> 5;
  const int h = g * G + hblk * HB + (w % HB);
  const int row_base = tile.t0 + 32 * (w / HB);
  const float sc = scale * kLog2e;

  const int qrow = min(row_base + c, tile.t1 - 1);
  const size_t rh = (size_t)qrow * Hq + h;
  bf16x8 Qr[kReg], dOr[kReg];
  uint16_t* stash = &stashS[w][0][l * 8];
  // With o != nullptr this launch also does the work of delta_bf16_kernel for
  // its rows (every (row, q head) belongs to exactly one lane pair of one
  // block): D = dO . O, summed in that kernel's order so that the value is the
  // same to the last bit, and the two row statistics are left in the workspace
  // for the dK/dV launch that follows.
  float dpart[KS];
  {
    const uint16_t* qp = q + rh * kHeadDim + 8 * hh;
    const uint16_t* dop = d_o + rh * kHeadDim + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const bf16x8 qx = *reinterpret_cast<const bf16x8*>(qp + 16 * ks);
      const bf16x8 dx = *reinterpret_cast<const bf16x8*>(dop + 16 * ks);
      if (o != nullptr) {
        const bf16x8 ox = *reinterpret_cast<const bf16x8*>(o + rh * kHeadDim + 8 * hh + 16 * ks);
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) s = fmaf((float)ox[e], (float)dx[e], s);
        dpart[ks] = s;
      }
      if (ks < kReg) {
        Qr[ks < kReg ? ks : 0] = qx;
        dOr[ks < kReg ? ks : 0] = dx;
      } else {
        *reinterpret_cast<bf16x8*>(stash + (2 * (ks - kReg)) * 512) = qx;
        *reinterpret_cast<bf16x8*>(stash + (2 * (ks - kReg) + 1) * 512) = dx;
      }
    }
  }
  auto q_op = [&](int ks) {
    return ks < kReg ? Qr[ks < kReg ? ks : 0]
                     : *reinterpret_cast<const bf16x8*>(stash + (2 * (ks - kReg)) * 512);
  };
  auto do_op = [&](int ks) {
    return ks < kReg ? dOr[ks < kReg ? ks : 0]
                     : *reinterpret_cast<const bf16x8*>(stash + (2 * (ks - kReg) + 1) * 512);
  };
  // accumulator start values of this lane's query row: the scores start from
  // -lse/scale so that P = exp(scale * acc), dP from -delta so that dS = P * acc
  const float nlse = -lse[rh] / scale;
  float ndlt;
  if (o != nullptr) {
    // delta_bf16_kernel's tree over HD / 8 lanes of 8 elements: lane 2*ks + hh there
    // is k-step ks of lane half hh here
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) dpart[ks] += __shfl_xor(dpart[ks], 32);
    float d = (dpart[0] + dpart[1]) + (dpart[2] + dpart[3]);
    if constexpr (HD == 128) d += (dpart[KS - 4] + dpart[KS - 3]) + (dpart[KS - 2] + dpart[KS - 1]);
    ndlt = -d;
    if (hh == 0 && row_base + c < tile.t1) {
      neg_delta[rh] = ndlt;
      neg_lse_s[rh] = -lse[rh] * (1.f / scale);
    }
  } else {
    ndlt = neg_delta[rh];
  }

  f32x16 dQ[TL::kBlocks];
#pragma unroll
  for (int a = 0; a < TL::kBlocks; ++a)
#pragma unroll
    for (int e = 0; e < 16; ++e) dQ[a][e] = 0.f;

  const size_t kv_stride = (size_t)Hkv * kHeadDim;
  const uint16_t* kbase = k + (size_t)g * kHeadDim;
  const uint16_t* vbase = v + (size_t)g * kHeadDim;
  const uint32_t kv_bytes = (uint32_t)kv_stride * 2;

  // chunk i lives in buffer i & 1 and is copied global -> LDS one iteration ahead
  KeyChunks it;
  it.init(segs, tile);
  int c0, n, full;
  bool have = it.next(c0, n, full);
  auto issue = [&](int b) {
    if (!full || n < kKeyChunk) {   // rare: a chunk that needs the visibility mask
      if (threadIdx.x < kKeyChunk) {   // kendS is indexed by matrix position
        const int row = TL::row_of_pos(threadIdx.x);
        kendS[b][threadIdx.x] = row >= n ? 0 : (full ? 0x7fffffff : kend[c0 + row]);
      }
    }
    tile_async_load<kDqThreads, HD>(Ks[b], kbase + (size_t)c0 * kv_stride, kv_bytes, n);
    tile_async_load<kDqThreads, HD>(Vs[b], vbase + (size_t)c0 * kv_stride, kv_bytes, n);
  };
  issue(0);
  int buf = 0;
  const int rlo = TL::row_lane_off(), clo = TL::col_lane_off();

  while (have) {
    async_wait_all();
    __syncthreads();   // chunk `buf` has landed; everyone is done with the other buffer
    const int cc0 = c0;
    const bool need_mask = !full || n < kKeyChunk;
    have = it.next(c0, n, full);
    if (have) issue(buf ^ 1);
    const uint16_t* Kt = Ks[buf] + rlo;
    const uint16_t* Vt = Vs[buf] + rlo;
    const uint16_t* Kc = Ks[buf] + clo;

    // The chunk's two 32-key halves as one sequence of 6 x KS matrix products (48
    // with head_dim 128) in six phases, in an issue order written out by hand (a scheduling barrier
    // after every product keeps it):
    //   S0 | dP0 + exp(S0) | S1 + dS0 | dP1 + exp(S1) | dQ0 + dS1 | dQ1
    // The LDS operand of product i + kAhead is read before product i is issued,
    // across phase boundaries too (ring of kAhead + 1 operands), and the
    // vector-ALU work of a phase is issued under products that do not depend on
    // it, so that both pipes of the SIMD work from within one wave.
    constexpr int kAhead = 2, kRing = kAhead + 1;
    f32x16 S[2], dP[2];
    bf16x8 dSb[2][2];
    bf16x8 a[kRing];
    // LDS operand j of phase ph: K rows (S), V rows (dP), K columns (dQ^T += K^T
    // dS^T: product j of a half uses columns 32*(j/2).., keys 16*(j%2).. of K)
    auto fetch = [&](auto ph_c, int j) {
      constexpr int ph = decltype(ph_c)::value;
      if constexpr (ph == 0 || ph == 2) return tile_row8(Kt, ph >> 1, j);
      else if constexpr (ph == 1 || ph == 3) return tile_row8(Vt, ph >> 1, j);
      else return tile_col8(Kc, 32 * (ph - 4) + 16 * (j & 1), 32 * (j >> 1));
    };
    constexpr int VP = 16 / KS;   // accumulator values whose vector work runs under one product
    auto phase = [&](auto ph_c) {
      constexpr int ph = decltype(ph_c)::value;
      constexpr int mb = (ph >> 1) & 1;
#pragma unroll
      for (int j = 0; j < KS; ++j) {
        const int i = KS * ph + j;   // product number in the chunk
        if (j + kAhead < KS) a[(i + kAhead) % kRing] = fetch(ph_c, j + kAhead);
        else if (ph < 5) a[(i + kAhead) % kRing] = fetch(std::integral_constant<int, (ph < 5 ? ph + 1 : 5)>{}, j + kAhead - KS);
        const bf16x8 av = a[i % kRing];
        if constexpr (ph == 0 || ph == 2) {          // S(mb), starting from -lse/scale
          if (j == 0) {
#pragma unroll
            for (int e = 0; e < 16; ++e) S[mb][e] = nlse;
          }
          S[mb] = mfma32(av, q_op(j), S[mb]);
        } else if constexpr (ph == 1 || ph == 3) {   // dP(mb), starting from -delta; P = exp(scale * S) under it
          if (j == 0) {
#pragma unroll
            for (int e = 0; e < 16; ++e) dP[mb][e] = ndlt;
          }
          dP[mb] = mfma32(av, do_op(j), dP[mb]);
#pragma unroll
          for (int t = 0; t < VP; ++t) S[mb][VP * j + t] = __builtin_amdgcn_exp2f(S[mb][VP * j + t] * sc);
        } else {                                     // dQ
          dQ[j >> 1] = mfma32(av, dSb[ph - 4][j & 1], dQ[j >> 1]);
        }
        if constexpr (ph == 2 || ph == 4) {          // dS of the previous half = P * dP, two values per product
          constexpr int pv = (ph - 2) >> 1;
#pragma unroll
          for (int t = 0; t < VP; ++t) {
            const int e = VP * j + t;
            dSb[pv][e >> 3][e & 7] = (__bf16)(S[pv][e] * dP[pv][e]);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      if constexpr (ph == 1 || ph == 3) {
        if (need_mask) {   // uniform branch
#pragma unroll
          for (int e4 = 0; e4 < 4; ++e4) {
            const int4 ke = *reinterpret_cast<const int4*>(&kendS[buf][32 * mb + 8 * e4 + 4 * hh]);
            const int kev[4] = {ke.x, ke.y, ke.z, ke.w};
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
              const int e = 4 * e4 + jj;
              const bool ok = (cc0 + TL::row_of_acc(mb, e, hh) <= qrow) & (qrow < kev[jj]);
              S[mb][e] = ok ? S[mb][e] : 0.f;
            }
          }
        }
      }
    };
#pragma unroll
    for (int j = 0; j < kAhead; ++j) a[j] = fetch(std::integral_constant<int, 0>{}, j);
    __builtin_amdgcn_sched_barrier(0);
    phase(std::integral_constant<int, 0>{});
    phase(std::integral_constant<int, 1>{});
    phase(std::integral_constant<int, 2>{});
    phase(std::integral_constant<int, 3>{});
    phase(std::integral_constant<int, 4>{});
    phase(std::integral_constant<int, 5>{});
    buf ^= 1;
  }

  const int token = row_base + c;
  if (token < tile.t1) {
    uint16_t* op = dq + ((size_t)token * Hq + h) * kHeadDim + 4 * hh;
#pragma unroll
    for (int dmb = 0; dmb < TL::kBlocks; ++dmb)
#pragma unroll
      for (int v4 = 0; v4 < 4; ++v4) {
        bf16x4 r;
#pragma unroll
        for (int e = 0; e < 4; ++e) r[e] = (__bf16)(dQ[dmb][4 * v4 + e] * scale);
        *reinterpret_cast<bf16x4*>(op + 32 * dmb + 8 * v4) = r;
      }
  }
}

// Key-stationary dK/dV: NW waves, 32 key columns each, K and V rows in
// registers.  NW = 4 (tiles of 128 keys): two blocks share a CU (everything
// fits in 256 registers), so one block's global loads and barriers are covered
// by the other's matrix work.  NW = 8 (tiles of 256 keys, schedules of long
// walks): one block per CU, and every 64-row chunk copied into LDS meets twice
// the keys.
template <int HD, int NW>
__global__ __launch_bounds__(64 * NW, 8 / NW) void dkdv_bf16_kernel(
    const KvItem* __restrict__ items, const int32_t* __restrict__ kend,
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
    const uint16_t* __restrict__ v, const uint16_t* __restrict__ d_o,
    const float* __restrict__ neg_lse_s, const float* __restrict__ neg_delta,
    uint16_t* __restrict__ dk, uint16_t* __restrict__ dv, float* __restrict__ partial,
    float* __restrict__ dk_acc, float* __restrict__ dv_acc, int Hq, int Hkv, float scale,
    int* __restrict__ tickets, int n_items) {
  using TL = TileLayout<HD>;
  constexpr int kTileElems = TL::kTileElems, kHeadDim = HD;
  constexpr int KS = TL::kSteps, DB = TL::kBlocks;
  constexpr int kKvThreads = 64 * NW, kKvTile = 32 * NW;
  // One object, so that every tile read is "per-lane base + compile-time offset".
  // With head_dim 128 the last k-steps of this wave's K and V operands (kStashK
  // and kStashV of the 8) live in LDS instead of registers, and so do the
  // per-lane mask bounds (key position, end of its visibility): with all of them
  // in registers the kernel needs a few more than 256, and the compiler's scratch
  // reloads (vector memory) would wait for, i.e. serialise, the tile copies in
  // flight.  Each lane reads back only what it wrote itself.
  constexpr int kStashK = HD == 128 ? 1 : 0, kStashV = HD == 128 ? 2 : 0;
  constexpr int kRegK = KS - kStashK, kRegV = KS - kStashV;
  struct Smem {
    uint16_t Q[2][kTileElems];
    uint16_t dO[2][kTileElems];
    float stat[2][2][kBQ];   // [buffer][-lse/scale | -delta][position]
    uint16_t stash[NW][kStashK + kStashV ? kStashK + kStashV : 1][64 * 8];
    int2 bound[kKvThreads];
  };
  __shared__ __attribute__((aligned(256))) Smem sm;
  // The drawn item travels through two words of the second statistics buffer:
  // nothing writes that buffer between the barrier at the end of an item and the
  // first barrier of the next item's walk, and with four waves the block's LDS
  // must stay at exactly 80 KB for two blocks to fit on a CU.
  int* next_item = reinterpret_cast<int*>(&sm.stat[1][0][0]);

  // Which (work item, kv head) this block works on.  tickets == nullptr: the
  // block index says so, one item per block.  Otherwise the launch is a fixed
  // number of resident blocks that draw items from one queue per kv head.
  ItemQueues queues;
  queues.init(tickets, n_items, Hkv);
  int item_idx = blockIdx.x / Hkv, g_idx = blockIdx.x % Hkv;
  if (tickets != nullptr && !queues.draw(next_item, item_idx, g_idx, false)) return;
  for (;;) {
  const KvItem tile = items[item_idx];
  const int g = g_idx;
  const int G = Hq / Hkv;
  const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
  const int c = l & 31, hh = l >> 5;
  const float sc = scale * kLog2e;

  // this lane's key column
  const int kcol = tile.k0 + 32 * w + c;
  const int kc = min(kcol, tile.k1 - 1);
  const int my_kend = kcol < tile.k1 ? kend[kc] : 0;   // padded columns see nothing
  sm.bound[threadIdx.x] = make_int2(kcol, my_kend);
  // rows [wave_lo, wave_hi) are the only ones any of this wave's 32 keys can see
  int wave_hi = my_kend;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) wave_hi = max(wave_hi, __shfl_xor(wave_hi, off));
  wave_hi = __builtin_amdgcn_readfirstlane(wave_hi);
  const int wave_lo = tile.k0 + 32 * __builtin_amdgcn_readfirstlane(w);
  bf16x8 Kr[kRegK], Vr[kRegV];
  uint16_t* stash = &sm.stash[w][0][l * 8];
  {
    const uint16_t* kp = k + ((size_t)kc * Hkv + g) * kHeadDim + 8 * hh;
    const uint16_t* vp = v + ((size_t)kc * Hkv + g) * kHeadDim + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const bf16x8 kx = *reinterpret_cast<const bf16x8*>(kp + 16 * ks);
      const bf16x8 vx = *reinterpret_cast<const bf16x8*>(vp + 16 * ks);
      if (ks < kRegK) Kr[ks < kRegK ? ks : 0] = kx;
      else *reinterpret_cast<bf16x8*>(stash + (ks - kRegK) * 512) = kx;
      if (ks < kRegV) Vr[ks < kRegV ? ks : 0] = vx;
      else *reinterpret_cast<bf16x8*>(stash + (kStashK + ks - kRegV) * 512) = vx;
    }
  }
  f32x16 dK[DB], dV[DB];
#pragma unroll
  for (int a = 0; a < DB; ++a)
#pragma unroll
    for (int e = 0; e < 16; ++e) { dK[a][e] = 0.f; dV[a][e] = 0.f; }

  const size_t q_stride = (size_t)Hq * kHeadDim;
  const uint32_t q_bytes = (uint32_t)q_stride * 2;
  // flat iteration over (64-row query chunk, head of the group), heads innermost.
  // Chunks are walked from the END of the range backwards (reverse DFS order):
  // key tiles of one node share the end of their query range, and k0 is a
  // multiple of the chunk size, so blocks that start together read exactly the
  // same 64-row chunks at the same time and find them in L2.  Step `it` lives
  // in buffer (it - it_begin) & 1 and is copied global -> LDS one iteration ahead of its use
  // (a third buffer and two iterations ahead, which the eight-wave form has the LDS for, is 1 % slower)
  // (this item covers iterations [it_begin, it_end) of the tile's walk)
  const int n_chunks = (tile.q_end - tile.q_begin + kBQ - 1) / kBQ;
  const int total = tile.it_end;
  auto issue = [&](int it, int b) {
    const int cq = it / G, hsub = it - cq * G;
    const int ch = n_chunks - 1 - cq;
    const int h = g * G + hsub;
    const int r0 = tile.q_begin + ch * kBQ;
    const int nv = min(kBQ, tile.q_end - r0);
    if (__builtin_amdgcn_readfirstlane(w) == 0) {   // stat is indexed by matrix position
      const uint32_t off = (uint32_t)min(TL::row_of_pos(l), nv - 1) * (uint32_t)Hq;
      row_async_load(sm.stat[b][0], neg_lse_s + (size_t)r0 * Hq + h, off);
      row_async_load(sm.stat[b][1], neg_delta + (size_t)r0 * Hq + h, off);
    }
    tile_async_load<kKvThreads, HD>(sm.Q[b], q + (size_t)r0 * q_stride + (size_t)h * kHeadDim, q_bytes, nv);
    tile_async_load<kKvThreads, HD>(sm.dO[b], d_o + (size_t)r0 * q_stride + (size_t)h * kHeadDim, q_bytes, nv);
  };
  if (tile.it_begin < total) issue(tile.it_begin, 0);
  const int rlo = TL::row_lane_off(), clo = TL::col_lane_off();

  // one step of the walk; the buffer index is a compile-time constant
  auto step = [&](int it, auto buf_c) {
    constexpr int buf = decltype(buf_c)::value;
    async_wait_all();
    __syncthreads();   // chunk `buf` has landed; everyone is done with the other buffer
    if (it + 1 < total) issue(it + 1, buf ^ 1);
    const int ch = n_chunks - 1 - it / G;
    const int r0 = tile.q_begin + ch * kBQ;
    const int nv = min(kBQ, tile.q_end - r0);
    const bool need_mask = !(r0 >= tile.k1 && r0 + kBQ <= tile.q_full_end);
    const uint16_t* Qt = sm.Q[buf] + rlo;
    const uint16_t* dOt = sm.dO[buf] + rlo;
    const uint16_t* Qc = sm.Q[buf] + clo;
    const uint16_t* dOc = sm.dO[buf] + clo;

    // Small per-lane LDS addresses are recomputed every step from a value the
    // compiler cannot see through: kept across the loop they would be spilled,
    // and a reload from scratch waits for the copies just issued.
    int tid_now = threadIdx.x;
    asm volatile("" : "+v"(tid_now));
    const float* stat = &sm.stat[buf][0][4 * ((tid_now >> 5) & 1)];
    // Half a chunk (32 query rows) against this wave's 32 keys, as one
    // straight-line block in four phases.  Each phase pairs matrix products with
    // the vector-ALU work of the previous phase's result, so that both pipes of
    // the SIMD are busy from within one wave:
    //   1  S  = -lse/scale + Q K^T
    //   2  dP = -delta + dO V^T      |  P = exp(scale * S)
    //      (mask P where the chunk needs it), pack P
    //   3  dV += P^T dO              |  dS = P * dP, pack dS
    //   4  dK += dS^T Q
    // The accumulators start from the row statistics (values 4*e4 .. 4*e4+3 of a
    // lane are four consecutive matrix positions), so no subtraction is left.
    auto half = [&](auto mq_c) {
      constexpr int mq = decltype(mq_c)::value;
      // The issue order is written out by hand: operand reads run kAhead
      // products ahead (which also bounds their registers), and a scheduling
      // barrier after each product keeps the compiler from regrouping the
      // vector-ALU work away from the product it is meant to run under.
      constexpr int kAhead = 2;
      auto k_op = [&](int ks) {
        return ks < kRegK ? Kr[ks < kRegK ? ks : 0]
                          : *reinterpret_cast<const bf16x8*>(stash + (ks - kRegK) * 512);
      };
      auto v_op = [&](int ks) {
        return ks < kRegV ? Vr[ks < kRegV ? ks : 0]
                          : *reinterpret_cast<const bf16x8*>(stash + (kStashK + ks - kRegV) * 512);
      };
      constexpr int VP = 16 / KS;   // accumulator values whose vector work runs under one product
      f32x16 S, dP;
      bf16x8 a[KS];
      // ---- phase 1
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        const f32x4 ls = *reinterpret_cast<const f32x4*>(stat + (32 * mq + 8 * e4));
#pragma unroll
        for (int j = 0; j < 4; ++j) S[4 * e4 + j] = ls[j];
      }
#pragma unroll
      for (int ks = 0; ks < kAhead; ++ks) a[ks] = tile_row8(Qt, mq, ks);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        if (ks + kAhead < KS) a[ks + kAhead] = tile_row8(Qt, mq, ks + kAhead);
        S = mfma32(a[ks], k_op(ks), S);
        __builtin_amdgcn_sched_barrier(0);
      }
      // ---- phase 2
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        const f32x4 dl = *reinterpret_cast<const f32x4*>(stat + (kBQ + 32 * mq + 8 * e4));
#pragma unroll
        for (int j = 0; j < 4; ++j) dP[4 * e4 + j] = dl[j];
      }
#pragma unroll
      for (int ks = 0; ks < kAhead; ++ks) a[ks] = tile_row8(dOt, mq, ks);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        if (ks + kAhead < KS) a[ks + kAhead] = tile_row8(dOt, mq, ks + kAhead);
        dP = mfma32(a[ks], v_op(ks), dP);
#pragma unroll
        for (int t = 0; t < VP; ++t) S[VP * ks + t] = __builtin_amdgcn_exp2f(S[VP * ks + t] * sc);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (need_mask) {   // query row t sees this lane's key iff kcol <= t < kend[kcol]
        // row_of_acc(mq, e, hh) = kHalf*hh + (compile-time part): compare against per-lane bounds
        constexpr int kHalf = TL::row_of_acc(0, 0, 1) - TL::row_of_acc(0, 0, 0);
        const int2 bnd = sm.bound[tid_now];
        const int lo = bnd.x - r0 - kHalf * hh;
        const int hi = min(bnd.y - r0, nv) - kHalf * hh;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int rc = TL::row_of_acc(mq, e, 0);
          S[e] = ((rc >= lo) & (rc < hi)) ? S[e] : 0.f;
        }
      }
      // ---- phase 3: product i uses columns 32*(i/2).., rows 16*(i%2).. of dO
      const bf16x8 Pb[2] = {pack8(S, 0), pack8(S, 1)};
      bf16x8 dSb[2];
#pragma unroll
      for (int i = 0; i < kAhead; ++i) a[i] = tile_col8(dOc, 32 * mq + 16 * (i & 1), 32 * (i >> 1));
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < KS; ++i) {
        if (i + kAhead < KS)
          a[i + kAhead] = tile_col8(dOc, 32 * mq + 16 * ((i + kAhead) & 1), 32 * ((i + kAhead) >> 1));
        dV[i >> 1] = mfma32(a[i], Pb[i & 1], dV[i >> 1]);
#pragma unroll
        for (int t = 0; t < VP; ++t) {
          const int e = VP * i + t;
          dSb[e >> 3][e & 7] = (__bf16)(dP[e] * S[e]);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      // ---- phase 4
#pragma unroll
      for (int i = 0; i < kAhead; ++i) a[i] = tile_col8(Qc, 32 * mq + 16 * (i & 1), 32 * (i >> 1));
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < KS; ++i) {
        if (i + kAhead < KS)
          a[i + kAhead] = tile_col8(Qc, 32 * mq + 16 * ((i + kAhead) & 1), 32 * ((i + kAhead) >> 1));
        dK[i >> 1] = mfma32(a[i], dSb[i & 1], dK[i >> 1]);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    // a chunk none of this wave's keys can see contributes nothing (wave-uniform)
    const bool wave_sees = r0 + nv > wave_lo && r0 < wave_hi;
    if (wave_sees) {
      half(std::integral_constant<int, 0>{});
      half(std::integral_constant<int, 1>{});
    }
  };
  for (int it = tile.it_begin; it < total; it += 2) {
    step(it, std::integral_constant<int, 0>{});
    if (it + 1 < total) step(it + 1, std::integral_constant<int, 1>{});
  }
  if (tickets != nullptr) queues.prefetch();

  if (tile.slot >= 0) {
    // one of several items of this key tile: fp32 partial sums, [dK | dV] x keys of a tile x head_dim
    float* pk = partial + ((size_t)tile.slot * Hkv + g) * (2 * kKvTile * kHeadDim) +
                (size_t)(32 * w + c) * kHeadDim + 4 * hh;
    float* pv = pk + kKvTile * kHeadDim;
#pragma unroll
    for (int dmb = 0; dmb < DB; ++dmb)
#pragma unroll
      for (int v4 = 0; v4 < 4; ++v4) {
        f32x4 rk, rv;
#pragma unroll
        for (int e = 0; e < 4; ++e) { rk[e] = dK[dmb][4 * v4 + e]; rv[e] = dV[dmb][4 * v4 + e]; }
        *reinterpret_cast<f32x4*>(pk + 32 * dmb + 8 * v4) = rk;
        *reinterpret_cast<f32x4*>(pv + 32 * dmb + 8 * v4) = rv;
      }
  } else if (dk_acc != nullptr) {
    // segment call: this block is the only one that owns these keys in this
    // launch; add to the caller's fp32 accumulators
    if (kcol < tile.k1) {
      const size_t base = ((size_t)kcol * Hkv + g) * kHeadDim + 4 * hh;
#pragma unroll
      for (int dmb = 0; dmb < DB; ++dmb)
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4) {
          f32x4 rk = *reinterpret_cast<const f32x4*>(dk_acc + base + 32 * dmb + 8 * v4);
          f32x4 rv = *reinterpret_cast<const f32x4*>(dv_acc + base + 32 * dmb + 8 * v4);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            rk[e] += dK[dmb][4 * v4 + e] * scale;
            rv[e] += dV[dmb][4 * v4 + e];
          }
          *reinterpret_cast<f32x4*>(dk_acc + base + 32 * dmb + 8 * v4) = rk;
          *reinterpret_cast<f32x4*>(dv_acc + base + 32 * dmb + 8 * v4) = rv;
        }
    }
  } else if (kcol < tile.k1) {
    const size_t base = ((size_t)kcol * Hkv + g) * kHeadDim + 4 * hh;
#pragma unroll
    for (int dmb = 0; dmb < DB; ++dmb)
#pragma unroll
      for (int v4 = 0; v4 < 4; ++v4) {
        bf16x4 rk, rv;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          rk[e] = (__bf16)(dK[dmb][4 * v4 + e] * scale);
          rv[e] = (__bf16)(dV[dmb][4 * v4 + e]);
        }
        *reinterpret_cast<bf16x4*>(dk + base + 32 * dmb + 8 * v4) = rk;
        *reinterpret_cast<bf16x4*>(dv + base + 32 * dmb + 8 * v4) = rv;
      }
  }
  if (tickets == nullptr || !queues.draw(next_item, item_idx, g_idx, true)) break;
  }   // next item
}

// Sets n ints to zero (the ticket counters; a fill kernel rather than a memset
// so that the launch sequence can be captured in a graph).
__global__ void zero_i32_kernel(int* __restrict__ p, int n) {
  for (int i = threadIdx.x; i < n; i += blockDim.x) p[i] = 0;
}

// Adds the partial sums of a split key tile in slot order and writes dK/dV.
template <int HD>
__global__ __launch_bounds__(256) void dkdv_reduce_kernel(const KvReduce* __restrict__ red,
                                                          const float* __restrict__ partial,
                                                          uint16_t* __restrict__ dk,
                                                          uint16_t* __restrict__ dv, int Hkv,
                                                          float scale, int kKvTile) {
  // 8 blocks per (tile, kv head), an eighth of the tile's kKvTile keys each, so that even a handful of split
  // tiles fills the chip
  const int sub = blockIdx.x & 7;
  const KvReduce r = red[(blockIdx.x >> 3) / Hkv];
  constexpr int kHeadDim = HD;
  const int g = (blockIdx.x >> 3) % Hkv;
  const size_t slot_stride = (size_t)Hkv * (2 * kKvTile * kHeadDim);
  const float* base = partial + ((size_t)r.first_slot * Hkv + g) * (2 * kKvTile * kHeadDim);
  const int key_lo = sub * (kKvTile / 8), key_hi = min(r.k1 - r.k0, key_lo + kKvTile / 8);
  for (int i = key_lo * (kHeadDim / 4) + threadIdx.x; i < key_hi * (kHeadDim / 4); i += blockDim.x) {
    const int key = i / (kHeadDim / 4), d4 = i % (kHeadDim / 4);
    f32x4 sk = {0.f, 0.f, 0.f, 0.f}, sv = {0.f, 0.f, 0.f, 0.f};
    for (int p = 0; p < r.nparts; ++p) {
      const float* src = base + (size_t)p * slot_stride + (size_t)key * kHeadDim + 4 * d4;
      const f32x4 a = *reinterpret_cast<const f32x4*>(src);
      const f32x4 b = *reinterpret_cast<const f32x4*>(src + kKvTile * kHeadDim);
#pragma unroll
      for (int e = 0; e < 4; ++e) { sk[e] += a[e]; sv[e] += b[e]; }
    }
    bf16x4 rk, rv;
#pragma unroll
    for (int e = 0; e < 4; ++e) { rk[e] = (__bf16)(sk[e] * scale); rv[e] = (__bf16)sv[e]; }
    const size_t o = ((size_t)(r.k0 + key) * Hkv + g) * kHeadDim + 4 * d4;
    *reinterpret_cast<bf16x4*>(dk + o) = rk;
    *reinterpret_cast<bf16x4*>(dv + o) = rv;
  }
}

}  // namespace

template <int HD>
int launch_bwd_bf16_hd(const LaunchArgs& a) {
  constexpr int kHeadDim = HD;
  hipStream_t st = (hipStream_t)a.stream;
  clear_hip_error();
  // rows of (token, q head) the call covers: all of them, or one segment's
  const size_t row0 = (size_t)a.row_begin * a.p.n_q_heads;
  const size_t rows = (size_t)(a.row_end - a.row_begin) * a.p.n_q_heads;
  const size_t qblocks = a.sched->q_tiles.size() * (size_t)a.p.n_kv_heads * (size_t)a.tc.hblocks;
  const size_t kblocks = a.sched->kv_items.size() * (size_t)a.p.n_kv_heads;
  if (qblocks == 0 || qblocks > 0x7fffffffu || kblocks > 0x7fffffffu) return DTA_ERR_UNSUPPORTED;
  // the dQ launch computes the row statistics itself when both stages are asked for
  const bool fused_delta = (a.stages & DTA_BWD_DELTA) && (a.stages & DTA_BWD_DQ);
  if ((a.stages & DTA_BWD_DELTA) && !fused_delta) {
    constexpr size_t kDeltaRows = 256 / (HD / 8);   // rows per block of the delta kernel
    delta_bf16_kernel<HD><<<(unsigned)((rows + kDeltaRows - 1) / kDeltaRows), 256, 0, st>>>(
        (const uint16_t*)a.o + row0 * kHeadDim, (const uint16_t*)a.d_o + row0 * kHeadDim,
        a.lse_in + row0, a.delta + row0, a.lse2 + row0, 1.f / a.p.softmax_scale, rows);
    { int ls = launch_status(__func__); if (ls != DTA_OK) return ls; }
  }
  if (a.stages & DTA_BWD_DQ) {
    // Long blocks (at least 64 key chunks each on average) in at least 8 rounds:
    // blocks draw their item from queues, see the kernel.  Shorter blocks would
    // pay more for the draw (an atomic round trip before anything else can
    // start) than the balance between XCDs gives back.
    const size_t n_tiles = a.sched->q_tiles.size();
    const bool draw = a.tickets != nullptr && qblocks >= 8 * (size_t)kNumCUs &&
                      a.sched->fwd_chunks64 >= 64 * (int64_t)n_tiles && qblocks < 0x60000000u;
    if (draw) {
      zero_i32_kernel<<<1, 256, 0, st>>>(a.tickets, a.p.n_kv_heads);
      { int ls = launch_status(__func__); if (ls != DTA_OK) return ls; }
    }
    dq_bf16_kernel<HD><<<(unsigned)(draw ? qblocks + qblocks / 4 : qblocks), kDqThreads, 0, st>>>(
        a.sched->d_q_tiles, a.sched->d_segs, a.d_kend, (const uint16_t*)a.q, (const uint16_t*)a.k,
        (const uint16_t*)a.v, (const uint16_t*)a.d_o, a.lse_in,
        fused_delta ? (const uint16_t*)a.o : nullptr, a.delta, a.lse2, (uint16_t*)a.dq,
        a.p.n_q_heads, a.p.n_kv_heads, a.tc.hb, a.tc.hblocks, a.p.softmax_scale,
        draw ? a.tickets : nullptr, (int)(n_tiles * (size_t)a.tc.hblocks));
    { int ls = launch_status(__func__); if (ls != DTA_OK) return ls; }
  }
  if (a.stages & DTA_BWD_DKDV) {
    // One block per item, or a fixed set of resident blocks that draw the items
    // from per-head queues (the schedule decides: at least 8 rounds of items,
    // long walks cut finer).  The queues let XCDs that run faster take work from
    // the others (under this kernel the shader clocks of the 8 XCDs differ by up
    // to 10 %, and one block per item gives every XCD the same share) and save
    // the block hand-over, at the price of a barrier pair and an atomic per item.
    // Measured on MI355X (dK/dV launch, queues against blocks): forests of many
    // short items +0.6...+1.5 %, the 16 long answers and the deep tree +3...+5 %,
    // fewer than 8 rounds lose 1-2 % to the extra launch.
    const bool wide = a.sched->kv_keys == 256;   // tiles of 256 keys: eight waves, one block per CU
    if (a.sched->kv_keys != 128 && !wide) return DTA_ERR_UNSUPPORTED;
    const size_t resident = (wide ? 1 : 2) * (size_t)kNumCUs;
    const bool queues = a.sched->kv_queues && a.dk_acc == nullptr;
    int* tickets = a.tickets + a.p.n_kv_heads;   // second half: this kernel's counters
    if (queues) {
      zero_i32_kernel<<<1, 256, 0, st>>>(tickets, a.p.n_kv_heads);
      { int ls = launch_status(__func__); if (ls != DTA_OK) return ls; }
    }
    auto kernel = wide ? dkdv_bf16_kernel<HD, 8> : dkdv_bf16_kernel<HD, 4>;
    kernel<<<(unsigned)(queues ? resident : kblocks), wide ? 512 : 256, 0, st>>>(
        a.sched->d_kv_items, a.d_kend, (const uint16_t*)a.q, (const uint16_t*)a.k,
        (const uint16_t*)a.v, (const uint16_t*)a.d_o, a.lse2, a.delta, (uint16_t*)a.dk,
        (uint16_t*)a.dv, a.partial, a.dk_acc, a.dv_acc, a.p.n_q_heads, a.p.n_kv_heads,
        a.p.softmax_scale, queues ? tickets : nullptr, (int)a.sched->kv_items.size());
    { int ls = launch_status(__func__); if (ls != DTA_OK) return ls; }
    if (!a.sched->kv_reduce.empty()) {
      dkdv_reduce_kernel<HD><<<(unsigned)(a.sched->kv_reduce.size() * a.p.n_kv_heads * 8), 256, 0, st>>>(
          a.sched->d_kv_reduce, a.partial, (uint16_t*)a.dk, (uint16_t*)a.dv, a.p.n_kv_heads,
          a.p.softmax_scale, a.sched->kv_keys);
      { int ls = launch_status(__func__); if (ls != DTA_OK) return ls; }
    }
  }
  return DTA_OK;
}

int launch_bwd_bf16(const LaunchArgs& a) {
  return a.p.head_dim == 128 ? launch_bwd_bf16_hd<128>(a) : launch_bwd_bf16_hd<64>(a);
}

}  // namespace dta
