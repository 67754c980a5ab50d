// Block-level top-p selection (Eq. 4-6; top-p kernel and expansion kernel of the
// kernel-design paragraph): per sequence, the mass of every block of G tokens,
// blocks ordered by the packed integer key of Eq. 14, the shortest prefix of
// that order whose mass reaches p of the total, expanded to tokens with the
// attention sinks and the query window always kept.
//
// Kept counts depend on the data, so the outputs are sized for the worst case
// and the totals stay on the device (new_cu_seqlens).  Four launches, five for batches of more than
// 128 sequences:
//   k_block_mass     one wave per block: its mass
//   k_top_p_rank     place of every block in the descending order of the keys, by counting the
//                    larger keys: 256 x 256 pairs per work-group, spread over the chip
//   k_top_p_blocks   one work-group per sequence: the masses put in that order, their running sum
//                    (chunks of 64 positions, one wave each), threshold, keep flags and in-sequence
//                    output offsets of the blocks
//   k_top_p_offsets  prefix sum of the per-sequence totals (large batches only: for up to 128
//                    sequences every work-group of k_top_p_emit forms the few sums it needs itself)
//   k_top_p_emit     one work-group per block: kept token ids, ascending
//
// Arithmetic that decides integers is fixed so that it can be matched bit for
// bit: a block's mass is the double sum of its float scores in index order,
// rounded to float; the running sum over the ordered blocks is a double sum of a
// fixed two-level shape -- the positions are cut into chunks of 64, inside a chunk
// the sum runs from zero one addition after the other, the chunks' totals are added
// one after the other, and a position's running sum is (the total of the earlier
// chunks) + (its sum inside its chunk) -- so that the chunks can be summed by
// different waves at once; the threshold is (double)p times the last running sum.
#include <type_traits>

#include "up_common.h"
#include "up_kernels.h"
#include "up_select.h"

namespace up {

constexpr int kTopPThreads = 1024;

constexpr int kTopPChunk = 64;                                  // positions per chunk of the running sum
constexpr int kMaxTopPChunks = kMaxTopPBlocks / kTopPChunk;

struct TopPSmem {
  double chunk_tot[kMaxTopPChunks];   // sum of every chunk's masses
  double chunk_off[kMaxTopPChunks];   // total of the chunks before it
  int wave_tot[16];
  int kstar_part[16];
  double thr;
};

// Mass of one block per wave: the lanes fetch the block's scores in one coalesced access
// each, then every lane adds them in index order (lane after lane, through broadcasts), so
// the sum is the same sequence of double additions as a plain loop over the block.
__global__ __launch_bounds__(256) void k_block_mass(TopPArgs a) {
  const int G = a.G;
  const int slot = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (slot >= a.T / G + a.R) return;
  const int lane = threadIdx.x & 63;
  const int r = locate_slot(a.cu, a.R, G, slot);
  const int c0 = a.cu[r];
  const int N = a.cu[r + 1] - c0;
  const int g = slot - slot_base(c0, r, G);
  if (g * G >= N) return;   // slack slot (also every slot of an empty sequence)
  const int L = imin(G, N - g * G);
  const float* s = a.scores + c0 + (long long)g * G;
  const float v0 = lane < L ? s[lane] : 0.0f;            // (+0 leaves a sum of non-negative terms as it is)
  const float v1 = 64 + lane < L ? s[64 + lane] : 0.0f;
  double acc = 0.0;
#pragma unroll
  for (int i = 0; i < 64; ++i) acc += (double)__shfl(v0, i);
  if (G > 64) {
#pragma unroll
    for (int i = 0; i < 64; ++i) acc += (double)__shfl(v1, i);
  }
  if (lane == 0) {
    a.blk_mass[slot] = (float)acc;
    a.blk_rank[slot] = 0;      // k_top_p_rank adds to it
  }
}

// Place of every block in the descending order of the packed keys of Eq. 14 (mass, then the
// lower block index first) = the number of larger keys; the keys are distinct.  A sequence
// of nb blocks is covered by ceil(nb/256)^2 work-groups: each counts, for 256 blocks, the larger
// keys among 256 others (LDS broadcasts, eight reads in flight) and adds its count to the
// block's total -- integer additions, so their order does not matter.  For the few thousand
// blocks of a sequence this beats a sorting network, whose every stage ends in a barrier.
__global__ __launch_bounds__(256) void k_top_p_rank(TopPArgs a, int chunks) {
  __shared__ unsigned long long others[256];
  const int r = blockIdx.x / (chunks * chunks);
  const int pair = blockIdx.x % (chunks * chunks);
  const int c0 = a.cu[r];
  const int N = a.cu[r + 1] - c0;
  const int nb = ceil_div(N, a.G);
  const int ci = pair / chunks, cj = pair % chunks;
  if (ci * 256 >= nb || cj * 256 >= nb) return;
  const int slot0 = slot_base(c0, r, a.G);
  const int tid = threadIdx.x;
  auto key_of = [&](int g) {
    return ((unsigned long long)phi(a.blk_mass[slot0 + g]) << 32) | (unsigned)(nb - 1 - g);
  };
  const int j = cj * 256 + tid, i = ci * 256 + tid;
  others[tid] = j < nb ? key_of(j) : 0ull;                       // zero is larger than no key
  const unsigned long long mine = i < nb ? key_of(i) : ~0ull;
  __syncthreads();
  int cnt = 0;
  for (int j0 = 0; j0 < 256; j0 += 8) {
    unsigned long long o[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) o[u] = others[j0 + u];
#pragma unroll
    for (int u = 0; u < 8; ++u) cnt += o[u] > mine ? 1 : 0;
  }
  if (i < nb && cnt > 0) atomicAdd(&a.blk_rank[slot0 + i], cnt);
}

__global__ __launch_bounds__(kTopPThreads) void k_top_p_blocks(TopPArgs a) {
  __shared__ TopPSmem sm;
  const int r = blockIdx.x;
  const int c0 = a.cu[r];
  const int N = a.cu[r + 1] - c0;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (N == 0) {
    if (tid == 0) a.seq_kept[r] = 0;
    return;
  }
  const int G = a.G;
  const int nb = ceil_div(N, G);
  const int slot0 = slot_base(c0, r, G);

  // 1. the masses in the descending order of the keys (every block's place was counted by
  // k_top_p_rank); the list lives in the workspace: a sequence may have more blocks than LDS holds
  float* sorted = a.blk_sorted + slot0;
  for (int g = tid; g < nb; g += kTopPThreads) sorted[a.blk_rank[slot0 + g]] = a.blk_mass[slot0 + g];
  __syncthreads();      // (the work-group's own global writes are visible to it after the barrier)
  // 2. every chunk's total: a wave per chunk, the lanes fetch the chunk's 64 masses and every lane
  // adds them in order through broadcasts (the same sequence of double additions as a plain loop)
  const int nchunks = ceil_div(nb, kTopPChunk);
  for (int c = wave; c < nchunks; c += kTopPThreads / 64) {
    const int k = c * kTopPChunk + lane;
    const float v = k < nb ? sorted[k] : 0.0f;            // (+0 leaves a sum of non-negative terms as it is)
    double acc = 0.0;
#pragma unroll
    for (int i = 0; i < kTopPChunk; ++i) acc += (double)__shfl(v, i);
    if (lane == 0) sm.chunk_tot[c] = acc;
  }
  __syncthreads();
  // 3. the chunks' totals added one after the other; the threshold on the last running sum
  if (tid == 0) {
    double off = 0.0;
    for (int c = 0; c < nchunks; ++c) {
      sm.chunk_off[c] = off;
      off += sm.chunk_tot[c];
    }
    sm.thr = (double)a.top_p[r] * off;
  }
  __syncthreads();
  // 4. k* = 1 + number of positions whose running sum is still below the threshold (it never
  // decreases).  The sums inside the chunks are formed again, lane j stopping after its own position.
  const double thr = sm.thr;
  int below = 0;
  for (int c = wave; c < nchunks; c += kTopPThreads / 64) {
    const int k = c * kTopPChunk + lane;
    const float v = k < nb ? sorted[k] : 0.0f;
    double acc = 0.0;
#pragma unroll
    for (int i = 0; i < kTopPChunk; ++i) {
      const double vi = (double)__shfl(v, i);
      if (i <= lane) acc += vi;
    }
    below += (k < nb && sm.chunk_off[c] + acc < thr) ? 1 : 0;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) below += __shfl_xor(below, o);
  if (lane == 0) sm.kstar_part[wave] = below;
  __syncthreads();
  int kstar = 1;
  for (int w2 = 0; w2 < kTopPThreads / 64; ++w2) kstar += sm.kstar_part[w2];
  kstar = imin(kstar, nb);
  // 5. tokens kept per block and their exclusive prefix inside the sequence
  SeqGeom sg{N, G, a.n_obs, sinks_of(a.cu_k, a.n_sink, r, N), 1.0};
  int carry = 0;
  for (int base = 0; base < nb; base += kTopPThreads) {
    const int g = base + tid;
    int cnt = 0, keep = 0;
    if (g < nb) {
      const int lo = g * G, hi = imin(N, lo + G);
      keep = a.blk_rank[slot0 + g] < kstar ? 1 : 0;
      cnt = keep ? hi - lo : forced_in(sg, lo, hi);
    }
    int incl = cnt;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int up_v = __shfl_up(incl, o);
      if (lane >= o) incl += up_v;
    }
    if (lane == 63) sm.wave_tot[wave] = incl;
    __syncthreads();
    int before = carry;
    for (int w2 = 0; w2 < wave; ++w2) before += sm.wave_tot[w2];
    if (g < nb) {
      a.blk_keep[slot0 + g] = keep;
      a.blk_off[slot0 + g] = before + incl - cnt;
    }
    int total = carry;
    for (int w2 = 0; w2 < kTopPThreads / 64; ++w2) total += sm.wave_tot[w2];
    carry = total;
    __syncthreads();
  }
  if (tid == 0) a.seq_kept[r] = carry;
}

// Exclusive prefix of the per-sequence totals: the compacted stream's sequence offsets.
__global__ __launch_bounds__(1024) void k_top_p_offsets(const int32_t* __restrict__ seq_kept, int R,
                                                        int32_t* __restrict__ new_cu) {
  __shared__ int wave_tot[16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int carry = 0;
  if (tid == 0) new_cu[0] = 0;
  for (int base = 0; base < R; base += 1024) {
    const int r = base + tid;
    const int v = r < R ? seq_kept[r] : 0;
    int incl = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int up_v = __shfl_up(incl, o);
      if (lane >= o) incl += up_v;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    int before = carry;
    for (int w2 = 0; w2 < wave; ++w2) before += wave_tot[w2];
    if (r < R) new_cu[r + 1] = before + incl;
    int total = carry;
    for (int w2 = 0; w2 < 16; ++w2) total += wave_tot[w2];
    carry = total;
    __syncthreads();
  }
}

// Expansion to tokens: block g of sequence r keeps all its tokens if the block was chosen,
// otherwise only its sinks / window tokens; ids are written in ascending order.
// FOLD: there is no k_top_p_offsets launch (batches of few sequences): every work-group adds up
// the kept totals of the sequences before its own, and the first slot of a sequence -- which exists
// for empty sequences too -- writes the sequence's entry of new_cu.
template <bool FOLD>
__global__ __launch_bounds__(128) void k_top_p_emit(TopPArgs a) {
  __shared__ int cnt0;
  __shared__ int part[2];
  const int G = a.G;
  const int slot = blockIdx.x;
  const int r = locate_slot(a.cu, a.R, G, slot);
  const int c0 = a.cu[r];
  const int N = a.cu[r + 1] - c0;
  const int g = slot - slot_base(c0, r, G);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int seq_base;
  if (FOLD) {
    int acc = 0;
    for (int q = tid; q < r; q += 128) acc += a.seq_kept[q];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
    if (lane == 0) part[wave] = acc;
    __syncthreads();
    seq_base = part[0] + part[1];
    if (g == 0 && tid == 0) {
      a.new_cu[r] = seq_base;
      if (r == a.R - 1) a.new_cu[a.R] = seq_base + a.seq_kept[r];
    }
  } else {
    seq_base = a.new_cu[r];
  }
  if (g * G >= N) return;   // slack slot (also every slot of an empty sequence)
  const int i = g * G + tid;
  const bool in_block = tid < G && i < N;
  const bool keep = in_block && (a.blk_keep[slot] != 0 || i < sinks_of(a.cu_k, a.n_sink, r, N) || i >= N - a.n_obs);
  const unsigned long long bal = __ballot(keep);
  const int before = __popcll(bal & ((1ull << lane) - 1ull));
  if (wave == 0 && lane == 0) cnt0 = __popcll(bal);
  __syncthreads();
  if (keep) a.kept_idx[seq_base + a.blk_off[slot] + before + (wave == 1 ? cnt0 : 0)] = c0 + i;
}

hipError_t launch_top_p(const Problem& pb, const float* scores, const int32_t* cu, const int32_t* cu_k,
                        const float* top_p, int32_t* kept_idx, int32_t* new_cu, void* workspace, int max_blocks,
                        hipStream_t s) {
  const Workspace w = workspace_layout(pb);
  char* ws = (char*)workspace;
  TopPArgs a;
  a.scores = scores; a.cu = cu; a.cu_k = cu_k; a.top_p = top_p; a.kept_idx = kept_idx; a.new_cu = new_cu;
  a.blk_keep = (int32_t*)(ws + w.tp_keep_off);
  a.blk_off = (int32_t*)(ws + w.tp_off_off);
  a.seq_kept = (int32_t*)(ws + w.tp_seq_off);
  a.blk_mass = (float*)(ws + w.tp_mass_off);
  a.blk_rank = (int32_t*)(ws + w.tp_rank_off);
  a.blk_sorted = (float*)(ws + w.tp_sorted_off);
  a.R = pb.R; a.T = pb.T; a.G = pb.G; a.n_obs = pb.n_obs; a.n_sink = pb.n_sink;
  if (pb.T > 0)
    hipLaunchKernelGGL(k_block_mass, dim3((unsigned)((pb.T / pb.G + pb.R + 3) / 4)), dim3(256), 0, s, a);
  if (pb.T > 0 && max_blocks > 0) {
    const int chunks = (max_blocks + 255) / 256;
    hipLaunchKernelGGL(k_top_p_rank, dim3((unsigned)(chunks * chunks * pb.R)), dim3(256), 0, s, a, chunks);
  }
  if (pb.R > 0)
    hipLaunchKernelGGL(k_top_p_blocks, dim3((unsigned)pb.R), dim3(kTopPThreads), 0, s, a);
  // the sequences' offsets: a launch of their own when there are many sequences, else every
  // work-group of the expansion adds the few totals before its sequence up itself
  const bool fold = pb.T > 0 && pb.R <= 128;
  if (!fold) hipLaunchKernelGGL(k_top_p_offsets, dim3(1), dim3(1024), 0, s, a.seq_kept, pb.R, new_cu);
  if (pb.T > 0) {
    const dim3 grid((unsigned)(pb.T / pb.G + pb.R));
    if (fold) hipLaunchKernelGGL(k_top_p_emit<true>, grid, dim3(128), 0, s, a);
    else hipLaunchKernelGGL(k_top_p_emit<false>, grid, dim3(128), 0, s, a);
  }
  return hipGetLastError();
}

}  // namespace up
