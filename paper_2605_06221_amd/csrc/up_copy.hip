// Ragged row gather / scatter (Eq. 7 compaction, Eq. 8 reconstitution).
//
// Pure HBM traffic: one wavefront moves one row with 128-bit loads and stores,
// a whole row (up to 16 KB) in flight; rows are multiples of 16 bytes (checked on
// the host).  Streaming data is marked non-temporal so that it does not evict the
// key tensor from the last-level cache between the two scoring passes.
#include "up_common.h"
#include "up_copy.h"
#include "up_kernels.h"
#include "up_select.h"

namespace up {

template <bool SCATTER>
__global__ __launch_bounds__(256) void k_rows(const char* __restrict__ src, char* __restrict__ dst,
                                              const int32_t* __restrict__ idx, long long total_kept,
                                              long long row_bytes, long long stride_bytes,
                                              const int32_t* __restrict__ pos,
                                              int32_t* __restrict__ pos_out,
                                              const int32_t* __restrict__ count_dev) {
  const int lane = threadIdx.x & 63;
  const long long t = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  // (count_dev: the number of rows lives on the device; the launch covers the capacity, which
  // also bounds the output buffers whatever the device count says)
  if (t >= total_kept || (count_dev != nullptr && t >= (long long)count_dev[0])) return;
  const long long row = idx[t];
  if (SCATTER) {
    copy_row_wave(src + t * stride_bytes, dst + row * stride_bytes, row_bytes, lane);
  } else {
    copy_row_wave(src + row * stride_bytes, dst + t * stride_bytes, row_bytes, lane);
    if (pos != nullptr && lane == 0) pos_out[t] = pos[row];
  }
}

// Index map of two successive drops: out[t] = outer[inner[t]].
__global__ __launch_bounds__(256) void k_compose(const int32_t* __restrict__ outer,
                                                 const int32_t* __restrict__ inner, long long n,
                                                 const int32_t* __restrict__ count_dev,
                                                 int32_t* __restrict__ out) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t >= n || (count_dev != nullptr && t >= (long long)count_dev[0])) return;
  out[t] = outer[inner[t]];
}

// Gather of one per-token column of 4- or 8-byte elements (Eq. 7 for position ids of either
// width, token ids, ...): out[t] = column[idx[t]].
template <typename E>
__global__ __launch_bounds__(256) void k_column(const E* __restrict__ column, const int32_t* __restrict__ idx,
                                                long long n, const int32_t* __restrict__ count_dev,
                                                E* __restrict__ out) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t >= n || (count_dev != nullptr && t >= (long long)count_dev[0])) return;
  out[t] = column[idx[t]];
}

// Physical KV-cache slot of every retained token (Eq. 16): token t of sequence r (found from
// the compacted stream's offsets) at logical position p goes to block_table[r][p / B] * B + p % B.
__global__ __launch_bounds__(256) void k_slot_mapping(const int32_t* __restrict__ pos_kept,
                                                      const int32_t* __restrict__ new_cu, int R,
                                                      const int32_t* __restrict__ block_table,
                                                      long long table_stride, int kv_block,
                                                      long long capacity, int64_t* __restrict__ slots) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t >= capacity || t >= (long long)new_cu[R]) return;
  const int r = locate_token(new_cu, R, (int)t);
  const int p = pos_kept[t];
  slots[t] = (int64_t)block_table[(long long)r * table_stride + p / kv_block] * kv_block + p % kv_block;
}

hipError_t launch_slot_mapping(const int32_t* pos_kept, const int32_t* new_cu, int R,
                               const int32_t* block_table, long long table_stride, int kv_block,
                               long long capacity, int64_t* slots, hipStream_t s) {
  if (capacity == 0 || R == 0) return hipSuccess;
  hipLaunchKernelGGL(k_slot_mapping, dim3((unsigned)((capacity + 255) / 256)), dim3(256), 0, s, pos_kept, new_cu,
                     R, block_table, table_stride, kv_block, capacity, slots);
  return hipGetLastError();
}

hipError_t launch_column(const void* column, int elem_bytes, const int32_t* idx, long long n,
                         const int32_t* count_dev, void* out, hipStream_t s) {
  if (n == 0) return hipSuccess;
  const dim3 grid((unsigned)((n + 255) / 256));
  if (elem_bytes == 8)
    hipLaunchKernelGGL(k_column<uint64_t>, grid, dim3(256), 0, s, (const uint64_t*)column, idx, n, count_dev,
                       (uint64_t*)out);
  else
    hipLaunchKernelGGL(k_column<uint32_t>, grid, dim3(256), 0, s, (const uint32_t*)column, idx, n, count_dev,
                       (uint32_t*)out);
  return hipGetLastError();
}

// Token keep mask from the ascending list of kept rows: token t is kept iff the list holds t
// (binary search; every token writes its own byte, so nothing has to be cleared first).
__global__ __launch_bounds__(256) void k_keep_mask(const int32_t* __restrict__ kept_idx, long long capacity,
                                                   const int32_t* __restrict__ count_dev, long long T,
                                                   uint8_t* __restrict__ mask) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t >= T) return;
  long long n = capacity;
  if (count_dev != nullptr && (long long)count_dev[0] < n) n = count_dev[0];
  long long lo = 0, hi = n;            // first position with kept_idx[pos] >= t
  while (lo < hi) {
    const long long mid = (lo + hi) >> 1;
    if ((long long)kept_idx[mid] < t) lo = mid + 1; else hi = mid;
  }
  mask[t] = (lo < n && (long long)kept_idx[lo] == t) ? 1 : 0;
}

hipError_t launch_keep_mask(const int32_t* kept_idx, long long capacity, const int32_t* count_dev, long long T,
                            uint8_t* mask, hipStream_t s) {
  if (T == 0) return hipSuccess;
  hipLaunchKernelGGL(k_keep_mask, dim3((unsigned)((T + 255) / 256)), dim3(256), 0, s, kept_idx, capacity, count_dev, T, mask);
  return hipGetLastError();
}

// KV length that layer l sees during decode (Eq. 17): the length request r kept at the last drop
// event at a layer before l (the whole prompt if none), plus the tokens appended since prefill.
__global__ __launch_bounds__(256) void k_seqused(DropLayers drops, const int32_t* __restrict__ retained,
                                                 const int32_t* __restrict__ kv_len,
                                                 const int32_t* __restrict__ orig_len, int R, int num_layers,
                                                 int32_t* __restrict__ out) {
  const int r = blockIdx.x * 256 + threadIdx.x;
  const int layer = blockIdx.y;
  if (r >= R || layer >= num_layers) return;
  int last = -1;
  for (int k = 0; k < drops.n; ++k)
    if (drops.layer[k] < layer) last = k;
  const int orig = orig_len[r];
  const int s = last < 0 ? orig : retained[(long long)last * R + r];
  out[(long long)layer * R + r] = s + (kv_len[r] - orig);
}

hipError_t launch_seqused(const DropLayers& drops, const int32_t* retained, const int32_t* kv_len,
                          const int32_t* orig_len, int R, int num_layers, int32_t* out, hipStream_t s) {
  if (R == 0 || num_layers == 0) return hipSuccess;
  hipLaunchKernelGGL(k_seqused, dim3((unsigned)((R + 255) / 256), (unsigned)num_layers), dim3(256), 0, s, drops,
                     retained, kv_len, orig_len, R, num_layers, out);
  return hipGetLastError();
}

hipError_t launch_compose(const int32_t* outer, const int32_t* inner, long long n,
                          const int32_t* count_dev, int32_t* out, hipStream_t s) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(k_compose, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, outer, inner, n, count_dev, out);
  return hipGetLastError();
}

hipError_t launch_compact(const Problem& pb, const void* hidden, const int32_t* pos,
                          const int32_t* kept_idx, long long total_kept, void* hidden_out,
                          int32_t* pos_out, hipStream_t s) {
  if (total_kept == 0) return hipSuccess;
  const long long row_bytes = (long long)pb.d * pb.hidden_elem_bytes;
  const long long stride_bytes = pb.h_stride * pb.hidden_elem_bytes;
  const unsigned grid = (unsigned)((total_kept + 3) / 4);
  hipLaunchKernelGGL(k_rows<false>, dim3(grid), dim3(256), 0, s, (const char*)hidden,
                     (char*)hidden_out, kept_idx, total_kept, row_bytes, stride_bytes, pos, pos_out, (const int32_t*)nullptr);
  return hipGetLastError();
}

hipError_t launch_compact_counted(const Problem& pb, const void* hidden, const int32_t* pos,
                                  const int32_t* kept_idx, const int32_t* count_dev, long long capacity,
                                  void* hidden_out, int32_t* pos_out, hipStream_t s) {
  if (capacity == 0) return hipSuccess;
  const long long row_bytes = (long long)pb.d * pb.hidden_elem_bytes;
  const long long stride_bytes = pb.h_stride * pb.hidden_elem_bytes;
  const unsigned grid = (unsigned)((capacity + 3) / 4);
  hipLaunchKernelGGL(k_rows<false>, dim3(grid), dim3(256), 0, s, (const char*)hidden,
                     (char*)hidden_out, kept_idx, capacity, row_bytes, stride_bytes, pos, pos_out, count_dev);
  return hipGetLastError();
}

hipError_t launch_scatter(const Problem& pb, const void* hidden_compact, const int32_t* kept_idx,
                          long long total_kept, void* hidden_full, hipStream_t s) {
  if (total_kept == 0) return hipSuccess;
  const long long row_bytes = (long long)pb.d * pb.hidden_elem_bytes;
  const long long stride_bytes = pb.h_stride * pb.hidden_elem_bytes;
  const unsigned grid = (unsigned)((total_kept + 3) / 4);
  hipLaunchKernelGGL(k_rows<true>, dim3(grid), dim3(256), 0, s, (const char*)hidden_compact,
                     (char*)hidden_full, kept_idx, total_kept, row_bytes, stride_bytes,
                     (const int32_t*)nullptr, (int32_t*)nullptr, (const int32_t*)nullptr);
  return hipGetLastError();
}

}  // namespace up
