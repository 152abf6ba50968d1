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

}  // namespace dta
