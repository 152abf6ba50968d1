// Device-side walk over the key intervals of one query tile, shared by the
// forward and dQ kernels.
#pragma once

#include "dta_internal.h"

namespace dta {

constexpr int kKeyChunk = 64;  // keys per LDS tile

// Yields the key intervals of a query tile in chunks of CH keys: the pieces of
// the tile's root path first (root to parent), the tile's own token range last.
template <int CH>
struct KeyChunksT {
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
    if (si < seg_end) {   // the first interval travels with the tile record
      cur = t.first.start; end = t.first.end; full = t.first.full;
    } else {
      cur = t0; end = t1; full = 0;
    }
  }
  // number of chunks the walk will yield
  __device__ __forceinline__ static int count(const KeySeg* s, const QTile& t) {
    int nch = (t.t1 - t.t0 + CH - 1) / CH;
    for (int i = t.seg_begin; i < t.seg_end; ++i) nch += (s[i].end - s[i].start + CH - 1) / CH;
    return nch;
  }
  // c0 = first key, n = keys in the chunk (<= CH), is_full = no mask needed
  __device__ __forceinline__ bool next(int& c0, int& n, int& is_full) {
    if (si > seg_end) return false;
    c0 = cur; n = min(CH, end - cur); is_full = full;
    cur += CH;
    if (cur >= end) { ++si; if (si <= seg_end) load_seg(); }
    return true;
  }
};
using KeyChunks = KeyChunksT<kKeyChunk>;

}  // namespace dta
