// Row copy shared by the gather / scatter kernels and by the selection kernels when they are asked
// to gather their own rows (Eq. 7).
#pragma once

#include "up_common.h"

namespace up {

// One wave copies one row with 128-bit non-temporal accesses.  All loads of a round are issued
// before the first store; the round length is matched to the row (rows of up to 16 KB move in one
// round trip), which is worth a few percent of the gather's bandwidth over a fixed short round.
template <int U>
__device__ __forceinline__ void copy_row_rounds(const char* __restrict__ src, char* __restrict__ dst,
                                                long long row_bytes, int lane) {
  for (long long off = (long long)lane * 16; off < row_bytes; off += U * 1024) {
    u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (off + u * 1024 < row_bytes) v[u] = __builtin_nontemporal_load((const u32x4*)(src + off + u * 1024));
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (off + u * 1024 < row_bytes) __builtin_nontemporal_store(v[u], (u32x4*)(dst + off + u * 1024));
  }
}

__device__ __forceinline__ void copy_row_wave(const char* __restrict__ src, char* __restrict__ dst,
                                              long long row_bytes, int lane) {
  const long long chunks = (row_bytes + 1023) >> 10;     // the same for every lane of the wave
  if (chunks <= 4) copy_row_rounds<4>(src, dst, row_bytes, lane);
  else if (chunks <= 8) copy_row_rounds<8>(src, dst, row_bytes, lane);
  else if (chunks <= 10) copy_row_rounds<10>(src, dst, row_bytes, lane);
  else if (chunks <= 12) copy_row_rounds<12>(src, dst, row_bytes, lane);
  else copy_row_rounds<16>(src, dst, row_bytes, lane);
}

}  // namespace up
