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

// LDS tiles hold 128 bf16 per row plus padding chosen for how the tile is read
// (64 banks of 4 bytes).  16-byte row reads are served 16 lanes (rows) at a
// time and need a row pitch of 4*odd banks; the transposing 8-byte reads are
// served per 16-lane group (4 rows x 32 bytes) and need >= 8 banks between rows.
constexpr int kHeadDim = 128;
constexpr int kPitchRow = kHeadDim + 8;    // 68 banks  = 4 mod 64: row reads only
constexpr int kPitchCol = kHeadDim + 32;   // 80 banks  = 16 mod 64: column (transposing) reads only
constexpr int kPitchBoth = kHeadDim + 24;  // 76 banks  = 12 mod 64: both kinds of read

// D(32x32) += A(32x16) * B(16x32), bf16 inputs, fp32 accumulate.
// Lane l = (c = l % 32, hh = l / 32):
//   A: row c,     k = 8*hh .. 8*hh+7        B: column c, k = 8*hh .. 8*hh+7
//   D: column c,  row = 8*(v/4) + 4*hh + v%4   for v = 0..15
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ bf16x8 lds_read_row8(const uint16_t* p) {
  return *reinterpret_cast<const bf16x8*>(p);
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

// Operand for a matrix product that contracts over tile ROWS: for lane
// (c, hh) returns rows {r0+4hh..r0+4hh+3, r0+8+4hh..r0+8+4hh+3} of column
// col0 + c of a row-major LDS tile.  This row order is exactly the order in
// which a 32x32 accumulator block hands its 8 values v = 8s..8s+7 to the next
// product when reused as the other operand (r0 = 16*s inside the block).
template <int PITCH>
__device__ __forceinline__ bf16x8 lds_read_col8(const uint16_t* tile, int r0, int col0) {
  const int l = threadIdx.x & 63;
  const int i = l & 15, g16 = l >> 4;
  const int hh = g16 >> 1;
  const int col = col0 + 16 * (g16 & 1) + 4 * (i & 3);
  const int row = r0 + 4 * hh + (i >> 2);
  s16x4 lo = lds_read_tr4(tile + row * PITCH + col);
  s16x4 hi = lds_read_tr4(tile + (row + 8) * PITCH + col);
  union {
    struct { s16x4 a, b; } s;
    bf16x8 v;
  } u;
  u.s.a = lo;
  u.s.b = hi;
  return u.v;
}

__device__ __forceinline__ bf16x8 pack8(const f32x16& x, int s) {
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = (__bf16)x[8 * s + e];
  return r;
}

// 64 rows x 128 bf16 from global (row pitch `stride` elements) into registers,
// 16 bytes per thread per pass, NT threads; rows >= nvalid come back as zeros.
template <int NT>
struct TileRegs {
  uint4 r[1024 / NT];
};

template <int NT>
__device__ __forceinline__ void tile_load(TileRegs<NT>& t, const uint16_t* base, size_t stride,
                                          int nvalid) {
#pragma unroll
  for (int i = 0; i < 1024 / NT; ++i) {
    const int id = threadIdx.x + NT * i;
    const int row = id >> 4, col = id & 15;
    if (row < nvalid)
      t.r[i] = *reinterpret_cast<const uint4*>(base + (size_t)row * stride + col * 8);
    else
      t.r[i] = make_uint4(0, 0, 0, 0);
  }
}

template <int PITCH, int NT>
__device__ __forceinline__ void tile_store(const TileRegs<NT>& t, uint16_t* lds) {
#pragma unroll
  for (int i = 0; i < 1024 / NT; ++i) {
    const int id = threadIdx.x + NT * i;
    const int row = id >> 4, col = id & 15;
    *reinterpret_cast<uint4*>(lds + row * PITCH + col * 8) = t.r[i];
  }
}


// ---- tiles filled by direct global-to-LDS loads -------------------------------
// A wave's 16-byte direct loads land in 1 KB of consecutive LDS = 4 rows of 128
// bf16, so padding is only possible between such 4-row groups.  Bank conflicts
// are avoided by choosing WHICH tile row each matrix position uses: the matrix
// products only need keys (or query rows) to sit at consistent positions, not in
// order.  Position x (0..63) of a product uses tile row
//     row_of_pos(x) = 4 * sigma(x & 15) + (x >> 4),  sigma(y) = 4 * (y & 3) + (y >> 2),
// and group g starts at g * 1040 bytes.  Then the 16 lanes of one pass of a
// 16-byte row read touch 16 different groups (16 different 16-byte bank offsets),
// the 4 rows of one pass of a transposing read (32 lanes: 4 rows x 64 bytes) sit
// 64 bytes of bank offset apart, and every read address is a per-lane base plus
// a compile-time constant.
constexpr int kGroupPitch = 4 * kHeadDim + 8;     // elements between 4-row groups (1040 bytes)
constexpr int kTileElems = 16 * kGroupPitch;      // one 64 x 128 tile

__device__ __forceinline__ int sigma16(int y) { return ((y & 3) << 2) | (y >> 2); }
__device__ __forceinline__ int row_of_pos(int x) { return 4 * sigma16(x & 15) + (x >> 4); }
// For lane half hh, accumulator value e (0..15) of 32-position block mb holds
// position 32*mb + 8*(e/4) + 4*hh + e%4, i.e. tile row
__device__ __forceinline__ int row_of_acc(int mb, int e, int hh) {
  return 16 * (e & 3) + 8 * ((e >> 2) & 1) + 4 * hh + 2 * mb + (e >> 3);
}

// Starts the copy of rows [0, 64) x 128 bf16 (global row pitch stride_bytes,
// `base` uniform over the block) into `tile`; rows >= nvalid re-read row
// nvalid-1 (finite data the mask hides).  Completion: async_wait_all() by every
// thread, then a block barrier.
template <int NT>
__device__ __forceinline__ void tile_async_load(uint16_t* tile, const uint16_t* base,
                                                uint32_t stride_bytes, int nvalid) {
  constexpr int NW = NT / 64;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), l = threadIdx.x & 63;
  const uint32_t tile_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)tile;
  // The base is the same for every lane; make that visible so it lands in SGPRs.
  // (readfirstlane returns a signed int: widen through uint32_t, or a low half
  // with its top bit set would sign-extend into the high half.)
  const uint64_t base_bits = (uint64_t)(uintptr_t)base;
  const uint32_t base_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(base_bits >> 32));
  const uint32_t base_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)base_bits);
  const uint64_t sbase = ((uint64_t)base_hi << 32) | (uint64_t)base_lo;
  // lane part of the address for a full tile: row (l >> 4) of a 4-row group, piece l & 15
  const uint32_t lane_off = (uint32_t)(l >> 4) * stride_bytes + (l & 15) * 16;
#pragma unroll
  for (int p = 0; p < 16 / NW; ++p) {
    const int grp = w + NW * p;
    uint64_t gbase = sbase + (uint64_t)(4 * grp) * stride_bytes;   // scalar
    uint32_t voff = lane_off;
    if (nvalid < 64) {   // ragged tail of an interval (uniform branch)
      gbase = sbase;
      voff = (uint32_t)min(4 * grp + (l >> 4), nvalid - 1) * stride_bytes + (l & 15) * 16;
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

// Per-lane element offsets into a tile; add compile-time constants per read.
// Row operand (lane = position c of a 32-block, half hh): 8 elements at
//   tile + row_lane_off() + 256 * mb + 16 * ks          (block mb, k-step ks)
__device__ __forceinline__ int row_lane_off() {
  const int l = threadIdx.x & 63, c = l & 31, hh = l >> 5;
  return sigma16(c & 15) * kGroupPitch + (c >> 4) * kHeadDim + hh * 8;
}
// Column operand (contraction over positions r0 .. r0+15, r0 a multiple of 16,
// columns col0 .. col0+31): same value order as lds_read_col8, at
//   tile + col_lane_off() + 128 * (r0 / 16) + col0   and   + 2 * kGroupPitch for the upper 8
__device__ __forceinline__ int col_lane_off() {
  const int l = threadIdx.x & 63, i = l & 15, g16 = l >> 4, hh = g16 >> 1;
  return sigma16(4 * hh + (i >> 2)) * kGroupPitch + 16 * (g16 & 1) + 4 * (i & 3);
}
__device__ __forceinline__ bf16x8 tile_row8(const uint16_t* lane_ptr, int mb, int ks) {
  return *reinterpret_cast<const bf16x8*>(lane_ptr + 256 * mb + 16 * ks);
}
__device__ __forceinline__ bf16x8 tile_col8(const uint16_t* lane_ptr, int r0, int col0) {
  const uint16_t* p = lane_ptr + kHeadDim * (r0 >> 4) + col0;
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
