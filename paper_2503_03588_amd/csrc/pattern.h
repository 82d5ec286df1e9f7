// Closed-form enumeration of one row of the block-sparse pattern, usable from
// host code and from kernels.  Algorithm 1 (Section 3.3) decides per token
// pair; lifted to blocks, query block i attends key block j <= i when
// i-j < W, or i-j has at most one bit set, or j < S.  The three sets are a
// prefix [0,S), isolated blocks i-2^k, and a suffix [i-W+1, i] of the row, so
// the ascending duplicate-free union can be emitted without sorting.
#pragma once
#include <stdint.h>
#include "../../include/powattn.h"

#if defined(__HIPCC__)
#define PA_HD __host__ __device__ __forceinline__
#else
#define PA_HD inline
#endif

struct pa_row_shape {
  int64_t sink_end;  // sink blocks not inside the window: [0, sink_end)
  int64_t win_start; // window (suffix) blocks: [win_start, i]
  int64_t pow_lo;    // power blocks are emitted only inside [pow_lo, win_start)
};

PA_HD pa_row_shape pa_shape_of_row(int32_t W, int32_t S, uint32_t flags, int64_t i) {
  // the power test admits distance 0, so the diagonal is attended even with W == 0
  int64_t weff = (flags & POWATTN_POWER) ? (W > 1 ? W : 1) : W;
  pa_row_shape r;
  r.win_start = i - weff + 1;
  if (r.win_start < 0) r.win_start = 0;
  int64_t s_end = (int64_t)S < i + 1 ? (int64_t)S : i + 1;
  r.pow_lo = s_end;
  r.sink_end = s_end < r.win_start ? s_end : r.win_start;
  return r;
}

// Calls emit(j) for every attended key block of query block i in ascending
// order and returns how many there were.
template <class F>
PA_HD int64_t pa_for_each_block(int32_t W, int32_t S, uint32_t flags, int64_t i, F&& emit) {
  int64_t n = 0;
  if (flags & POWATTN_DENSE) {
    for (int64_t j = 0; j <= i; ++j) { emit(j); ++n; }
    return n;
  }
  pa_row_shape r = pa_shape_of_row(W, S, flags, i);
  for (int64_t j = 0; j < r.sink_end; ++j) { emit(j); ++n; }
  if (flags & POWATTN_POWER) {
    int64_t p = 1;
    while ((p << 1) <= i) p <<= 1;  // largest power of two <= i (i >= 1), else 1
    for (; p >= 1; p >>= 1) {
      int64_t j = i - p;
      if (j >= r.pow_lo && j < r.win_start) { emit(j); ++n; }
    }
  }
  for (int64_t j = r.win_start; j <= i; ++j) { emit(j); ++n; }
  return n;
}

PA_HD bool pa_block_attended(int32_t W, int32_t S, uint32_t flags, int64_t i, int64_t j) {
  if (j > i || j < 0) return false;
  if (flags & POWATTN_DENSE) return true;
  int64_t d = i - j;
  if (d < W || j < S) return true;
  return (flags & POWATTN_POWER) && ((d & (d - 1)) == 0);
}
