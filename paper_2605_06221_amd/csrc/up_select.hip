// Block-local top-k selection with forced retention, optionally fused with the
// gather of the kept rows.
//
// One work-group owns one selection block (G <= 128 consecutive tokens of one
// sequence).  Each token builds the 64-bit ordering key of Eq. 14 -- the
// order-preserving integer image of its float score in the upper word, the
// complemented in-block index in the lower word, forced tokens (sinks, query
// window) lifted above every score -- and finds its rank by counting larger
// keys in LDS.  Keys are unique, so ranks are a permutation and "rank < k_g"
// keeps exactly k_g tokens with ties going to the lower index.  Wavefront
// ballots give the ordered output positions; the block's output offset is
// closed-form (kept_before), so no scan over blocks is needed.
#include "up_common.h"
#include "up_kernels.h"

namespace up {

// Per-sequence kept totals and their exclusive prefix (the compacted stream's
// sequence offsets).  One work-group; sequences are scanned 1024 at a time.
__global__ __launch_bounds__(1024) void k_plan(const int32_t* __restrict__ cu,
                                               const float* __restrict__ ratio, int R, int G,
                                               int n_obs, int n_sink, int32_t* __restrict__ new_cu) {
  __shared__ int sh[1024];
  __shared__ int carry;
  const int tid = threadIdx.x;
  if (tid == 0) { carry = 0; new_cu[0] = 0; }
  __syncthreads();
  for (int base = 0; base < R; base += 1024) {
    const int r = base + tid;
    int v = 0;
    if (r < R) {
      SeqGeom sg{cu[r + 1] - cu[r], G, n_obs, n_sink, (double)ratio[r]};
      v = seq_kept(sg);
    }
    sh[tid] = v;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
      const int add = tid >= o ? sh[tid - o] : 0;
      __syncthreads();
      sh[tid] += add;
      __syncthreads();
    }
    if (r < R) new_cu[r + 1] = carry + sh[tid];
    __syncthreads();
    if (tid == 1023) carry += sh[1023];
    __syncthreads();
  }
}

// Monotone IEEE-754 -> unsigned map of Eq. 14 (sign read from the sign bit).
__device__ __forceinline__ unsigned phi(float x) {
  const unsigned b = __float_as_uint(x);
  return (b & 0x80000000u) ? ~b : (b ^ 0x80000000u);
}

__device__ __forceinline__ void copy_row_wave_sel(const char* __restrict__ src,
                                                  char* __restrict__ dst, long long row_bytes,
                                                  int lane) {
  constexpr int U = 4;
  long long off = (long long)lane * 16;
  for (; off + (U - 1) * 1024 < row_bytes; off += U * 1024) {
    u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load((const u32x4*)(src + off + u * 1024));
#pragma unroll
    for (int u = 0; u < U; ++u) __builtin_nontemporal_store(v[u], (u32x4*)(dst + off + u * 1024));
  }
  for (; off < row_bytes; off += 1024) {
    u32x4 v = __builtin_nontemporal_load((const u32x4*)(src + off));
    __builtin_nontemporal_store(v, (u32x4*)(dst + off));
  }
}

struct SelectArgs {
  const float* scores;      // given scores, or nullptr
  const double* parts;      // [n_parts][T] partial column sums, used when scores == nullptr
  int n_parts;
  const int32_t* cu;
  const float* ratio;
  const int32_t* new_cu;
  int32_t* kept_idx;
  float* scores_out;        // optional
  const char* hidden;       // nullptr => selection only
  const int32_t* pos;
  char* hidden_out;
  int32_t* pos_out;
  long long row_bytes, stride_bytes;
  int R, T, G, n_obs, n_sink, Hq;
};

__global__ __launch_bounds__(256) void k_select(SelectArgs a) {
  __shared__ unsigned long long keys[128];
  __shared__ int kept_local[128];
  __shared__ int sh_cnt0, sh_base;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int slot = blockIdx.x;
  const int r = locate_slot(a.cu, a.R, a.G, slot);
  const int c0 = a.cu[r];
  const int N = a.cu[r + 1] - c0;
  const int g = slot - slot_base(c0, r, a.G);
  if (g * a.G >= N) return;   // slack slot (also every slot of an empty sequence)

  SeqGeom sg{N, a.G, a.n_obs, a.n_sink, (double)a.ratio[r]};
  const int lo = g * a.G;
  const int L = imin(a.G, N - lo);
  const int kg = block_kept(sg, g);
  if (tid == 0) sh_base = a.new_cu[r] + kept_before(sg, g);

  bool keep = false;
  if (tid < 128) {
    if (tid < L) {
      const int i = lo + tid;
      const int tok = c0 + i;
      float sc;
      if (a.scores != nullptr) {
        sc = a.scores[tok];
      } else {
        double o = 0.0;
        for (int p = 0; p < a.n_parts; ++p) o += a.parts[(size_t)p * a.T + tok];
        const int n_eff = imin(a.n_obs, N);
        o = o / (double)(n_eff * a.Hq);
        sc = o < 0x1p-64 ? 0.0f : (float)o;
        if (a.scores_out != nullptr) a.scores_out[tok] = sc;
      }
      const bool forced = (i < a.n_sink) || (i >= N - a.n_obs);
      const unsigned hi = forced ? 0xFFFFFFFFu : phi(sc);
      keys[tid] = ((unsigned long long)hi << 32) | (unsigned)(a.G - 1 - tid);
    }
  }
  __syncthreads();
  if (tid < L) {
    if (kg >= L) {
      keep = true;
    } else {
      const unsigned long long mine = keys[tid];
      int rank = 0;
      for (int j = 0; j < L; ++j) rank += keys[j] > mine ? 1 : 0;
      keep = rank < kg;
    }
  }
  // ordered positions: wave 0 holds tokens 0..63, wave 1 tokens 64..127
  const unsigned long long bal = __ballot(keep);
  const int before = __popcll(bal & ((1ull << lane) - 1ull));
  if (wave == 0 && lane == 0) sh_cnt0 = __popcll(bal);
  __syncthreads();
  const int base = sh_base;
  if (keep) {
    const int at = before + (wave == 1 ? sh_cnt0 : 0);
    kept_local[at] = tid;
    a.kept_idx[base + at] = c0 + lo + tid;
  }
  if (a.hidden == nullptr) return;
  __syncthreads();
  // gather the kept rows: one wave per row, 128-bit accesses
  for (int j = wave; j < kg; j += 4) {
    const long long srow = c0 + lo + kept_local[j];
    copy_row_wave_sel(a.hidden + srow * a.stride_bytes, a.hidden_out + (long long)(base + j) * a.stride_bytes,
                      a.row_bytes, lane);
  }
  if (a.pos != nullptr && tid < kg) a.pos_out[base + tid] = a.pos[c0 + lo + kept_local[tid]];
}

hipError_t launch_plan(const Problem& pb, const int32_t* cu, const float* ratio, int32_t* new_cu,
                       hipStream_t s) {
  hipLaunchKernelGGL(k_plan, dim3(1), dim3(1024), 0, s, cu, ratio, pb.R, pb.G, pb.n_obs, pb.n_sink,
                     new_cu);
  return hipGetLastError();
}

hipError_t launch_select(const Problem& pb, const float* scores, const double* parts, int n_parts,
                         const int32_t* cu, const float* ratio, const int32_t* new_cu,
                         int32_t* kept_idx, float* scores_out, const void* hidden,
                         const int32_t* pos, void* hidden_out, int32_t* pos_out, hipStream_t s) {
  if (pb.T == 0) return hipSuccess;
  SelectArgs a;
  a.scores = scores; a.parts = parts; a.n_parts = n_parts; a.cu = cu; a.ratio = ratio;
  a.new_cu = new_cu; a.kept_idx = kept_idx; a.scores_out = scores_out;
  a.hidden = (const char*)hidden; a.pos = pos; a.hidden_out = (char*)hidden_out; a.pos_out = pos_out;
  a.row_bytes = (long long)pb.d * pb.hidden_elem_bytes;
  a.stride_bytes = pb.h_stride * pb.hidden_elem_bytes;
  a.R = pb.R; a.T = pb.T; a.G = pb.G; a.n_obs = pb.n_obs; a.n_sink = pb.n_sink; a.Hq = pb.Hq;
  const unsigned grid = (unsigned)(pb.T / pb.G + pb.R);
  hipLaunchKernelGGL(k_select, dim3(grid), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace up
