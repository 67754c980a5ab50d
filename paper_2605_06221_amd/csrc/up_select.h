// Block-local top-k selection with forced retention (device code shared by the
// stand-alone selection kernel and the scoring kernels that go on to select).
//
// One selection block is G <= 128 consecutive tokens of one sequence.  Each
// token builds the 64-bit ordering key of Eq. 14 -- the order-preserving
// integer image of its float score in the upper word, the complemented in-block
// index in the lower word, forced tokens (sinks, query window) lifted above
// every score -- and finds its rank by counting larger keys in LDS.  Keys are
// unique, so ranks are a permutation and "rank < k_g" keeps exactly k_g tokens
// with ties going to the lower index.  Wavefront ballots give the ordered
// output positions; the block's output offset is closed-form (kept_before), so
// no scan over blocks is needed.
#pragma once

#include "up_common.h"

namespace up {

constexpr int kMaxKeyBlock = 512;    // most tokens a work-group of the fused kernel owns

struct SelectArgs {
  const float* scores;      // stand-alone kernel: given scores
  const int32_t* cu;
  const int32_t* cu_k;      // key-side offsets when the tokens follow earlier context, else nullptr
  const float* ratio;
  const int32_t* new_cu;
  int32_t* kept_idx;
  int R, T, G, n_obs, n_sink;
};

struct SelectSmem {
  unsigned long long keys[128];
  float score[kMaxKeyBlock];
  int kept_rows[kMaxKeyBlock];   // a kernel that also gathers: the packed rows it has kept, ascending
  int cnt0, base;
};

#if defined(__HIPCC__)
// Sinks among the N tokens of sequence r: the first A tokens of the sequence so far, of which
// the earlier context (cu_k given: keys minus tokens) already holds some or all.
__device__ __forceinline__ int sinks_of(const int32_t* cu_k, int n_sink, int r, int N) {
  if (cu_k == nullptr) return n_sink;
  return imax(0, n_sink - ((cu_k[r + 1] - cu_k[r]) - N));
}

// Per-sequence kept totals and their exclusive prefix (the compacted stream's sequence
// offsets), by one work-group of NT threads (whole waves, at most 1024); sequences are scanned
// NT at a time.  wave_tot (16 ints) and carry are LDS of the caller.
template <int NT>
__device__ __forceinline__ void plan_scan(const int32_t* __restrict__ cu, const int32_t* __restrict__ cu_k,
                                          const float* __restrict__ ratio, int R, int G, int n_obs, int n_sink,
                                          int32_t* __restrict__ new_cu, int* wave_tot, int* carry) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) { *carry = 0; new_cu[0] = 0; }
  __syncthreads();
  for (int base = 0; base < R; base += NT) {
    const int r = base + tid;
    int v = 0;
    if (r < R) {
      const int N = cu[r + 1] - cu[r];
      SeqGeom sg{N, G, n_obs, sinks_of(cu_k, n_sink, r, N), (double)ratio[r]};
      v = seq_kept(sg);
    }
    // inclusive scan inside the wave, then over the wave totals
    int incl = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int up_v = __shfl_up(incl, o);
      if (lane >= o) incl += up_v;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    int before = *carry;
    for (int w2 = 0; w2 < wave; ++w2) before += wave_tot[w2];
    if (r < R) new_cu[r + 1] = before + incl;
    __syncthreads();
    if (tid == NT - 1) *carry = before + incl;
    __syncthreads();
  }
}

// Monotone IEEE-754 -> unsigned map of Eq. 14 (sign read from the sign bit).
__device__ __forceinline__ unsigned phi(float x) {
  const unsigned b = __float_as_uint(x);
  return (b & 0x80000000u) ? ~b : (b ^ 0x80000000u);
}

// Select block g of sequence r: writes the kept packed row ids, ascending.  Called by all
// threads of the work-group (at least 128; whole waves); `block_scores` points at the block's scores
// (LDS or global), indexed by the token's position inside the block.
// list_base >= 0: the kept rows also go to sm.kept_rows, at their output position minus list_base.
__device__ __forceinline__ void select_block(const SelectArgs& a, SelectSmem& sm, int r, int c0, int N,
                                             int g, const float* block_scores, int list_base = -1) {
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int n_sink = sinks_of(a.cu_k, a.n_sink, r, N);
  SeqGeom sg{N, a.G, a.n_obs, n_sink, (double)a.ratio[r]};
  const int lo = g * a.G;
  const int L = imin(a.G, N - lo);
  const int kg = block_kept(sg, g);
  if (tid == 0) sm.base = a.new_cu[r] + kept_before(sg, g);

  if (tid < L) {
    const int i = lo + tid;
    const bool forced = (i < n_sink) || (i >= N - a.n_obs);
    const unsigned hi = forced ? 0xFFFFFFFFu : phi(block_scores[tid]);
    sm.keys[tid] = ((unsigned long long)hi << 32) | (unsigned)(a.G - 1 - tid);
  }
  __syncthreads();
  bool keep = false;
  if (tid < L) {
    if (kg >= L) {
      keep = true;
    } else {
      const unsigned long long mine = sm.keys[tid];
      int rank = 0;
      for (int j = 0; j < L; ++j) rank += sm.keys[j] > mine ? 1 : 0;
      keep = rank < kg;
    }
  }
  // ordered positions: wave 0 holds tokens 0..63, wave 1 tokens 64..127
  const unsigned long long bal = __ballot(keep);
  const int before = __popcll(bal & ((1ull << lane) - 1ull));
  if (wave == 0 && lane == 0) sm.cnt0 = __popcll(bal);
  __syncthreads();
  if (keep) {
    const int at = sm.base + before + (wave == 1 ? sm.cnt0 : 0);
    a.kept_idx[at] = c0 + lo + tid;
    if (list_base >= 0) sm.kept_rows[at - list_base] = c0 + lo + tid;
  }
  __syncthreads();   // the shared arrays are reused by the next block
}

#endif  // __HIPCC__

}  // namespace up
