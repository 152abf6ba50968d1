// Device helpers for the bf16 matrix-core kernels (gfx950 / CDNA4, wave64).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace dta {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// D(32x32) += A(32x16) * B(16x32), bf16 inputs, fp32 accumulate.
// Lane l = (c = l % 32, hh = l / 32):
//   A: row c,     k = 8*hh .. 8*hh+7        B: column c, k = 8*hh .. 8*hh+7
//   D: column c,  row = 8*(v/4) + 4*hh + v%4   for v = 0..15
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Transposing LDS read (ds_read_b64_tr_b16).  Within each group of 16 lanes,
// lane j supplies the address of 4 consecutive bf16; lane i receives, as
// element e, element (i % 4) of what lane 4*e + i/4 addressed.  With lane j
// pointing at row r0 + j/4, column c0 + 4*(j%4) of a row-major tile, lane i ends
// up with rows r0..r0+3 of column c0 + i: a column read of a row-major tile.
__device__ __forceinline__ s16x4 lds_read_tr4(const uint16_t* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (s16x4 __attribute__((address_space(3)))*)(p));
}

__device__ __forceinline__ bf16x8 pack8(const f32x16& x, int s) {
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = (__bf16)x[8 * s + e];
  return r;
}


// ---- tiles filled by direct global-to-LDS loads -------------------------------
// A tile is 64 rows (keys or query rows) of HD bf16, HD = 128 or 64.  A wave's
// 16-byte direct loads land in 1 KB of consecutive LDS = 4 rows of 128 (8 rows of
// 64) bf16, so padding is only possible between such groups of rows.  Bank
// conflicts are avoided by choosing WHICH tile row each matrix position uses: the
// matrix products only need keys (or query rows) to sit at consistent positions,
// not in order.  With sigma(y) = 4 * (y & 3) + (y >> 2), position x (0..63) uses
//     HD = 128:  group sigma(x & 15),      row (x >> 4) of the group's 4
//     HD = 64 :  group sigma(x & 15) & 7,  row (sigma(x & 15) >> 3) + 2 * (x >> 4) of its 8
// and group g starts at g * 1040 bytes.  Then the 16 lanes of one pass of a
// 16-byte row read touch 16 different 16-byte bank offsets, the 4 rows of one pass
// of a transposing read (32 lanes: 4 rows x 64 bytes) sit 64 bytes of bank offset
// apart, and every read address is a per-lane base plus a compile-time constant,
// the same constants for both head dimensions.
constexpr int kGroupPitch = 512 + 8;              // elements between groups of rows (1040 bytes)

__device__ __forceinline__ int sigma16(int y) { return ((y & 3) << 2) | (y >> 2); }

template <int HD>
struct TileLayout {
  static_assert(HD == 128 || HD == 64, "head_dim 64 or 128");
  static constexpr int kRowsPerGroup = 512 / HD;            // rows one wave-wide direct load covers
  static constexpr int kGroups = 64 / kRowsPerGroup;        // per 64-row tile
  static constexpr int kTileElems = kGroups * kGroupPitch;  // one 64 x HD tile
  static constexpr int kSteps = HD / 16;                    // k-steps of a product that contracts over HD
  static constexpr int kBlocks = HD / 32;                   // 32-wide output blocks along HD

  __device__ __forceinline__ static int row_of_pos(int x) {
    const int s = sigma16(x & 15);
    return HD == 128 ? 4 * s + (x >> 4) : 8 * (s & 7) + (s >> 3) + 2 * (x >> 4);
  }
  // For lane half hh, accumulator value e (0..15) of 32-position block mb holds
  // position 32*mb + 8*(e/4) + 4*hh + e%4, i.e. tile row
  __device__ __forceinline__ static constexpr int row_of_acc(int mb, int e, int hh) {
    return HD == 128 ? 16 * (e & 3) + 8 * ((e >> 2) & 1) + 4 * hh + 2 * mb + (e >> 3)
                     : 32 * (e & 1) + 16 * ((e >> 2) & 1) + 8 * hh + ((e >> 1) & 1) + 4 * mb + 2 * (e >> 3);
  }
  // element offset of position x's row inside a tile
  __device__ __forceinline__ static int pos_off(int x) {
    const int s = sigma16(x & 15);
    return HD == 128 ? s * kGroupPitch + (x >> 4) * 128
                     : (s & 7) * kGroupPitch + ((s >> 3) + 2 * (x >> 4)) * 64;
  }
  // Per-lane element offsets into a tile; add compile-time constants per read.
  // Row operand (lane = position c of a 32-block, half hh): 8 elements at
  //   tile + row_lane_off() + 256 * mb + 16 * ks          (block mb, k-step ks)
  __device__ __forceinline__ static int row_lane_off() {
    const int l = threadIdx.x & 63, c = l & 31, hh = l >> 5;
    return pos_off(c) + hh * 8;
  }
  // Column operand (contraction over positions r0 .. r0+15, r0 a multiple of 16,
  // columns col0 .. col0+31), for tile_col8: at
  //   tile + col_lane_off() + 128 * (r0 / 16) + col0   and   + 2 * kGroupPitch for the upper 8
  __device__ __forceinline__ static int col_lane_off() {
    const int l = threadIdx.x & 63, i = l & 15, g16 = l >> 4, hh = g16 >> 1;
    return pos_off(4 * hh + (i >> 2)) + 16 * (g16 & 1) + 4 * (i & 3);
  }
};

// Starts the copy of rows [0, 64) x HD bf16 (global row pitch stride_bytes,
// `base` uniform over the block) into `tile`; rows >= nvalid re-read row
// nvalid-1 (finite data the mask hides).  Completion: async_wait_all() by every
// thread, then a block barrier.
template <int NT, int HD>
__device__ __forceinline__ void tile_async_load(uint16_t* tile, const uint16_t* base,
                                                uint32_t stride_bytes, int nvalid) {
  using TL = TileLayout<HD>;
  constexpr int NW = NT / 64;
  constexpr int kRowShift = HD == 128 ? 4 : 3;   // lanes per row = HD / 8
  constexpr int kPieceMask = (1 << kRowShift) - 1;
  static_assert(TL::kGroups % NW == 0, "every wave copies the same number of row groups");
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), l = threadIdx.x & 63;
  const uint32_t tile_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)tile;
  // The base is the same for every lane; make that visible so it lands in SGPRs.
  // (readfirstlane returns a signed int: widen through uint32_t, or a low half
  // with its top bit set would sign-extend into the high half.)
  const uint64_t base_bits = (uint64_t)(uintptr_t)base;
  const uint32_t base_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(base_bits >> 32));
  const uint32_t base_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)base_bits);
  const uint64_t sbase = ((uint64_t)base_hi << 32) | (uint64_t)base_lo;
  // lane part of the address for a full tile: row (l >> kRowShift) of a group, 16-byte piece l & kPieceMask
  const uint32_t lane_off = (uint32_t)(l >> kRowShift) * stride_bytes + (l & kPieceMask) * 16;
#pragma unroll
  for (int p = 0; p < TL::kGroups / NW; ++p) {
    const int grp = w + NW * p;
    uint64_t gbase = sbase + (uint64_t)(TL::kRowsPerGroup * grp) * stride_bytes;   // scalar
    uint32_t voff = lane_off;
    if (nvalid < 64) {   // ragged tail of an interval (uniform branch)
      gbase = sbase;
      voff = (uint32_t)min(TL::kRowsPerGroup * grp + (l >> kRowShift), nvalid - 1) * stride_bytes +
             (l & kPieceMask) * 16;
    }
    // Written as inline assembly on purpose: for the builtin form the compiler
    // drains every outstanding load before the next LDS read, which would undo
    // the prefetch.  Address = scalar base + 32-bit lane offset; LDS destination
    // = M0 + 16 * lane.
    const uint32_t lds_addr = __builtin_amdgcn_readfirstlane(tile_addr + grp * kGroupPitch * 2);
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(voff), "s"(gbase), "s"(lds_addr)
                 : "memory");
  }
}

// Starts the copy of 64 floats into dst[0..63] (LDS): lane l of the calling
// wave fetches base[elem_off] with its own elem_off, so the copy can permute.
// One wave calls this; completion as for tile_async_load.
__device__ __forceinline__ void row_async_load(float* dst, const float* base, uint32_t elem_off) {
  const uint32_t dst_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)dst;
  const uint64_t base_bits = (uint64_t)(uintptr_t)base;
  const uint32_t base_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(base_bits >> 32));
  const uint32_t base_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)base_bits);
  const uint64_t sbase = ((uint64_t)base_hi << 32) | (uint64_t)base_lo;
  const uint32_t lds_addr = __builtin_amdgcn_readfirstlane(dst_addr);
  const uint32_t voff = elem_off * 4;
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dword %0, %1"
               :
               : "v"(voff), "s"(sbase), "s"(lds_addr)
               : "memory");
}

// Waits for every vector-memory load of this wave, the tile copies included.
// Issued through the builtin (vmcnt = 0, other counters untouched) so that the
// compiler's own wait tracking sees it: otherwise it keeps loads from before a
// loop pending across the back edge and adds partial vmcnt waits inside the
// loop, which stall on the copies in flight.
__device__ __forceinline__ void async_wait_all() {
  __builtin_amdgcn_s_waitcnt(0x0F70);
  asm volatile("" ::: "memory");
}

// Reads at a lane pointer made from TileLayout<HD>::row_lane_off() / col_lane_off().
__device__ __forceinline__ bf16x8 tile_row8(const uint16_t* lane_ptr, int mb, int ks) {
  return *reinterpret_cast<const bf16x8*>(lane_ptr + 256 * mb + 16 * ks);
}
__device__ __forceinline__ bf16x8 tile_col8(const uint16_t* lane_ptr, int r0, int col0) {
  const uint16_t* p = lane_ptr + 128 * (r0 >> 4) + col0;
  s16x4 lo = lds_read_tr4(p);
  s16x4 hi = lds_read_tr4(p + 2 * kGroupPitch);
  union {
    struct { s16x4 a, b; } s;
    bf16x8 v;
  } u;
  u.s.a = lo;
  u.s.b = hi;
  return u.v;
}

}  // namespace dta
