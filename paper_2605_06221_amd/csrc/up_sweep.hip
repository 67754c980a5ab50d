// Token-importance scoring (Eq. 2-3) on the gfx950 matrix cores, and the fused
// score -> select -> compact kernel.
//
// The softmax of a query row is normalised over *all* visible keys, so the
// Q.K^T product runs twice:
//
//   pass 1 (row statistics)  S^T = K Q^T tiles: a lane owns one query row and
//           32 of the work-group's 256 keys; it takes the row maximum and the
//           sum of exponentials over those keys.  Lane halves and the four
//           waves are merged, giving one (reference, sum) pair per row and key
//           block; k_combine merges the key blocks of a sequence.
//   pass 2 (column sums)  S = Q K^T tiles: a lane owns one key and 16 query
//           rows per tile; it applies each row's final (reference, 1/sum) and
//           adds the normalised weights.  One wave sees every row of every head
//           for its keys, so the per-token score is complete inside the wave:
//           no partial planes, no atomics, fixed summation order.
//
// Work decomposition ("key-stationary"): one work-group = 256 consecutive keys
// of one sequence, four waves of 64 keys each.  A wave keeps its keys of the
// current kv head in registers as MFMA operands (2 tiles x 8 k-steps) and
// sweeps all query rows of that head's GQA group; the rows stream through LDS
// in units of 64 (coalesced 128-bit loads, padded rows, read back in operand
// layout), shared by the four waves.  v_mfma_f32_32x32x16_bf16: bf16 products
// are exact in fp32 and accumulate in fp32.
//
// Because a pass-2 work-group ends with the final scores of 256 consecutive
// tokens, it owns whole selection blocks (G divides 256) and goes straight on
// to the block-local top-k and the gather of the kept rows: the HBM-bound copy
// of one work-group overlaps the matrix work of the others.
//
// Logits are handled in log2 units: x = s_raw * c + negref, c = scale*log2(e),
// so the exponential is a bare v_exp_f32.
#include "up_common.h"
#include "up_kernels.h"
#include "up_select.h"

namespace up {

constexpr int kUnit = 64;            // query rows per LDS staging unit
constexpr int kQRow = 272;           // LDS bytes per query row: 256 + 16 pad (conflict-free b128 reads)
constexpr int kSweepThreads = 256;

typedef float f32x16 __attribute__((ext_vector_type(16)));

struct SweepArgs {
  const char* q;
  const char* k;
  const int32_t* cu;
  float2* stat_part;   // [key_block_slots][Hq * n_obs]  (reference in log2 units, sum)
  float2* stat_fin;    // [Hq][row_slots]                 (negative reference, 1/sum)
  float* scores_out;   // pass 2: optional
  long long q_stride_b, k_stride_b;   // bytes between tokens
  float c;             // scale * log2(e)
  int R, T, Hq, Hkv, Gq, n_obs, row_slots;
  int do_select;       // pass 2: run the block-local top-k (+ gather if sel.hidden != nullptr)
  SelectArgs sel;
};

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ __forceinline__ float exp2_hw(float x) { return __builtin_amdgcn_exp2f(x); }

// x -> (x / d, x % d) with a precomputed magic = 0xFFFFFFFF / d  (x < 2^31).
__device__ __forceinline__ void divmod(unsigned x, unsigned d, unsigned magic, int& qo, int& ro) {
  unsigned qq = __umulhi(x, magic);
  unsigned rr = x - qq * d;
  if (rr >= d) { ++qq; rr -= d; }
  qo = (int)qq;
  ro = (int)rr;
}

struct SweepSmem {
  __align__(16) unsigned char q[2][kUnit * kQRow];   // staged query rows (bf16), double-buffered
  __align__(16) float2 cst[2][kUnit];                // pass 2: (negative reference, 1/sum) per staged row
  __align__(16) int rowpos[2][kUnit];                // local position of each staged row, -1 = no such row
  float2 wstat[2][4][kUnit];                         // pass 1: per-wave (reference, sum) per staged row
  double o64[kKeyBlock];                             // pass 2: column sums of the block's keys
  SelectSmem sel;
};

template <int PASS, bool EDGE>
__device__ __forceinline__ void sweep_block(const SweepArgs& a, SweepSmem& sm, int r, int c0, int N,
                                            int kblock, int slot) {
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int l32 = lane & 31, half = lane >> 5;
  const int n_eff = imin(a.n_obs, N);
  const int first_q = N - n_eff;
  const int rows_total = n_eff * a.Gq;
  const int n_units = (rows_total + kUnit - 1) / kUnit;
  const int n_flat = a.Hkv * n_units;
  const unsigned magic = 0xFFFFFFFFu / (unsigned)n_eff;
  const int key_base = kblock * kKeyBlock + wave * 64;     // first local key of this wave
  const float c = a.c;
  const int rs0 = rowslot_base(c0, r, a.n_obs);

  // ---- key operands of one kv head: [key tile][k-step], lane = (key l32, k-slice half)
  bf16x8 kf[2][8];
  auto load_keys = [&](bf16x8 (&dst)[2][8], int g) {
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
      const int key = key_base + kt * 32 + l32;
      const char* kp = a.k + (long long)(c0 + key) * a.k_stride_b + (long long)g * 256 + half * 16;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        u32x4 v = {0u, 0u, 0u, 0u};
        if (key < N) v = *(const u32x4*)(kp + kk * 32);
        dst[kt][kk] = as_bf16x8(v);
      }
    }
  };

  // ---- staging of one unit of query rows (and their per-row constants)
  u32x4 pre_q[4];
  float2 pre_cst = make_float2(0.0f, 0.0f);
  int pre_pos = -1;
  auto fetch_unit = [&](int f) {
    const int g = f / n_units;
    const int u = f - g * n_units;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int piece = tid + i * kSweepThreads;     // 1024 pieces of 16 bytes: 64 rows x 16
      const int rho = u * kUnit + (piece >> 4);
      u32x4 v = {0u, 0u, 0u, 0u};
      if (rho < rows_total) {
        int hh, jj;
        divmod((unsigned)rho, (unsigned)n_eff, magic, hh, jj);
        v = *(const u32x4*)(a.q + (long long)(c0 + first_q + jj) * a.q_stride_b +
                            (long long)(g * a.Gq + hh) * 256 + (piece & 15) * 16);
      }
      pre_q[i] = v;
    }
    if (tid < kUnit) {
      const int rho = u * kUnit + tid;
      pre_cst = make_float2(0.0f, 0.0f);
      pre_pos = -1;
      if (rho < rows_total) {
        int hh, jj;
        divmod((unsigned)rho, (unsigned)n_eff, magic, hh, jj);
        pre_pos = first_q + jj;
        if (PASS == 2) pre_cst = a.stat_fin[(size_t)(g * a.Gq + hh) * a.row_slots + rs0 + jj];
      }
    }
  };
  auto stash_unit = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int piece = tid + i * kSweepThreads;
      *(u32x4*)(&sm.q[buf][(piece >> 4) * kQRow + (piece & 15) * 16]) = pre_q[i];
    }
    if (tid < kUnit) {
      sm.cst[buf][tid] = pre_cst;
      sm.rowpos[buf][tid] = pre_pos;
    }
  };

  double col64[2] = {0.0, 0.0};   // pass 2: running column sums of this lane's two keys

  load_keys(kf, 0);
  fetch_unit(0);
  stash_unit(0);
  __syncthreads();

  for (int f = 0; f < n_flat; ++f) {
    const int buf = f & 1;
    const int g = f / n_units;
    const int u = f - g * n_units;
    const bool last_of_head = (u == n_units - 1);
    if (f + 1 < n_flat) fetch_unit(f + 1);

#pragma unroll 1
    for (int rt = 0; rt < 2; ++rt) {
      f32x16 acc0, acc1;
#pragma unroll
      for (int e = 0; e < 16; ++e) { acc0[e] = 0.0f; acc1[e] = 0.0f; }
      const unsigned char* qrow = &sm.q[buf][(rt * 32 + l32) * kQRow + half * 16];
      if (PASS == 1) {
        // S^T: element e of key tile kt = key kt*32 + 8*(e/4) + 4*half + e%4, query row rt*32 + l32
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
          const bf16x8 qv = as_bf16x8(*(const u32x4*)(qrow + kk * 32));
          acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[0][kk], qv, acc0, 0, 0, 0);
          acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[1][kk], qv, acc1, 0, 0, 0);
        }
        if (EDGE) {
          const int rp = sm.rowpos[buf][rt * 32 + l32];
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int key = key_base + 8 * (e >> 2) + 4 * half + (e & 3);
            if (key > rp) acc0[e] = -INFINITY;
            if (key + 32 > rp) acc1[e] = -INFINITY;
          }
        }
        float m = fmaxf(acc0[0], acc1[0]);
#pragma unroll
        for (int e = 1; e < 16; ++e) m = fmaxf(m, fmaxf(acc0[e], acc1[e]));
        float ref = m * c;                        // reference in log2 units
        float l = 0.0f;
        if (!EDGE || m != -INFINITY) {
          const float negref = -ref;
          float l0 = 0.0f, l1 = 0.0f;
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            l0 += exp2_hw(fmaf(acc0[e], c, negref));
            l1 += exp2_hw(fmaf(acc1[e], c, negref));
          }
          l = l0 + l1;
        } else {
          ref = -INFINITY;
        }
        // merge the two lane halves (same row, other 32 keys)
        const float ref_o = __shfl_xor(ref, 32);
        const float l_o = __shfl_xor(l, 32);
        const float mm = fmaxf(ref, ref_o);
        const float s_a = ref == -INFINITY ? 0.0f : l * exp2_hw(ref - mm);
        const float s_b = ref_o == -INFINITY ? 0.0f : l_o * exp2_hw(ref_o - mm);
        if (half == 0) sm.wstat[buf][wave][rt * 32 + l32] = make_float2(mm, s_a + s_b);
      } else {
        // S: element e = query row rt*32 + 8*(e/4) + 4*half + e%4, key kt*32 + l32
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
          const bf16x8 qv = as_bf16x8(*(const u32x4*)(qrow + kk * 32));
          acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qv, kf[0][kk], acc0, 0, 0, 0);
          acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qv, kf[1][kk], acc1, 0, 0, 0);
        }
        float c0s = 0.0f, c1s = 0.0f;
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
          const int row0 = rt * 32 + 8 * e4 + 4 * half;
          const f32x4 cs01 = *(const f32x4*)(&sm.cst[buf][row0]);       // rows row0, row0+1
          const f32x4 cs23 = *(const f32x4*)(&sm.cst[buf][row0 + 2]);   // rows row0+2, row0+3
          const float negm[4] = {cs01[0], cs01[2], cs23[0], cs23[2]};
          const float wr[4] = {cs01[1], cs01[3], cs23[1], cs23[3]};
          int rp[4] = {0, 0, 0, 0};
          if (EDGE) {
#pragma unroll
            for (int i = 0; i < 4; ++i) rp[i] = sm.rowpos[buf][row0 + i];
          }
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int e = e4 * 4 + i;
            float x0 = fmaf(acc0[e], c, negm[i]);
            float x1 = fmaf(acc1[e], c, negm[i]);
            if (EDGE) {
              if (key_base + l32 > rp[i]) x0 = -INFINITY;
              if (key_base + 32 + l32 > rp[i]) x1 = -INFINITY;
            }
            c0s = fmaf(exp2_hw(x0), wr[i], c0s);
            c1s = fmaf(exp2_hw(x1), wr[i], c1s);
          }
        }
        col64[0] += (double)c0s;
        col64[1] += (double)c1s;
      }
    }

    if (f + 1 < n_flat) stash_unit(buf ^ 1);
    if (last_of_head && g + 1 < a.Hkv) load_keys(kf, g + 1);   // next head's keys replace this head's
    __syncthreads();

    if (PASS == 1 && tid < kUnit) {
      // merge the four waves' statistics of one staged row, write the key block's partial
      const int rho = u * kUnit + tid;
      if (rho < rows_total) {
        const float2 s0 = sm.wstat[buf][0][tid], s1 = sm.wstat[buf][1][tid];
        const float2 s2 = sm.wstat[buf][2][tid], s3 = sm.wstat[buf][3][tid];
        const float mm = fmaxf(fmaxf(s0.x, s1.x), fmaxf(s2.x, s3.x));
        float l = 0.0f;
        if (s0.x != -INFINITY) l += s0.y * exp2_hw(s0.x - mm);
        if (s1.x != -INFINITY) l += s1.y * exp2_hw(s1.x - mm);
        if (s2.x != -INFINITY) l += s2.y * exp2_hw(s2.x - mm);
        if (s3.x != -INFINITY) l += s3.y * exp2_hw(s3.x - mm);
        int hh, jj;
        divmod((unsigned)rho, (unsigned)n_eff, magic, hh, jj);
        a.stat_part[(size_t)slot * (a.Hq * a.n_obs) + (size_t)(g * a.Gq + hh) * a.n_obs + jj] =
            make_float2(mm, l);
      }
    }
  }

  if (PASS == 2) {
    // the two lane halves hold the same keys over different rows: add them (fixed order)
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
      const double other = __shfl_xor(col64[kt], 32);
      if (half == 0) sm.o64[wave * 64 + kt * 32 + l32] = col64[kt] + other;
    }
  }
}

template <int PASS>
__global__ __launch_bounds__(kSweepThreads, 2) void k_sweep(SweepArgs a) {
  __shared__ SweepSmem sm;
  const int slot = blockIdx.x;
  const int r = locate_slot(a.cu, a.R, kKeyBlock, slot);
  const int c0 = a.cu[r];
  const int N = a.cu[r + 1] - c0;
  const int kblock = slot - slot_base(c0, r, kKeyBlock);
  if (kblock * kKeyBlock >= N) return;
  const int n_eff = imin(a.n_obs, N);
  // causal masking and the ragged end only matter where keys reach the query window
  const bool edge = (kblock + 1) * kKeyBlock - 1 > N - n_eff;
  if (edge) sweep_block<PASS, true>(a, sm, r, c0, N, kblock, slot);
  else sweep_block<PASS, false>(a, sm, r, c0, N, kblock, slot);

  if (PASS == 2) {
    __syncthreads();
    const int tid = threadIdx.x;
    const int key = kblock * kKeyBlock + tid;
    float sc = 0.0f;
    if (key < N) {
      const double o = sm.o64[tid] / (double)(n_eff * a.Hq);
      sc = o < 0x1p-64 ? 0.0f : (float)o;
      if (a.scores_out != nullptr) a.scores_out[c0 + key] = sc;
    }
    if (!a.do_select) return;
    sm.sel.score[tid] = sc;
    __syncthreads();
    // the block-local top-k and the gather, one selection block after the other
    const int G = a.sel.G;
    const int nb = imin(kKeyBlock / G, ceil_div(N - kblock * kKeyBlock, G));
    for (int b = 0; b < nb; ++b)
      select_block(a.sel, sm.sel, r, c0, N, kblock * (kKeyBlock / G) + b, &sm.sel.score[b * G]);
  }
}

// Merge the per-key-block softmax statistics of every (sequence, window row, head):
// final reference = max of the block references, sum rescaled to it (double).
// Threads run along the window rows of one head (coalesced); eight threads share
// a row and split its key blocks.
__global__ __launch_bounds__(256) void k_combine(const int32_t* __restrict__ cu,
                                                 const float2* __restrict__ stat_part,
                                                 float2* __restrict__ stat_fin, int R, int Hq,
                                                 int n_obs, int row_slots) {
  __shared__ float sh_m[8][32];
  __shared__ double sh_l[8][32];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const int u = blockIdx.x * 32 + tx;
  const int h = blockIdx.y;
  bool live = u < row_slots;
  int n_blocks = 0;
  const float2* p = stat_part;
  const size_t stride = (size_t)Hq * n_obs;
  if (live) {
    const int r = locate_rowslot(cu, R, n_obs, u);
    const int c0 = cu[r];
    const int N = cu[r + 1] - c0;
    const int jj = u - rowslot_base(c0, r, n_obs);
    live = jj < imin(n_obs, N);
    if (live) {
      n_blocks = ceil_div(N, kKeyBlock);
      p = stat_part + (size_t)slot_base(c0, r, kKeyBlock) * stride + (size_t)h * n_obs + jj;
    }
  }
  float m = -INFINITY;
  for (int b = ty; b < n_blocks; b += 8) m = fmaxf(m, p[(size_t)b * stride].x);
  sh_m[ty][tx] = m;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 8; ++i) m = fmaxf(m, sh_m[i][tx]);
  double L = 0.0;
  for (int b = ty; b < n_blocks; b += 8) {
    const float2 st = p[(size_t)b * stride];
    if (st.x != -INFINITY) L += (double)st.y * exp2((double)st.x - (double)m);
  }
  sh_l[ty][tx] = L;
  __syncthreads();
  if (ty == 0 && live) {
    double tot = 0.0;
#pragma unroll
    for (int i = 0; i < 8; ++i) tot += sh_l[i][tx];
    stat_fin[(size_t)h * row_slots + u] = make_float2(-m, (float)(1.0 / tot));
  }
}

Workspace workspace_layout(const Problem& pb) {
  auto al = [](size_t x) { return (x + 255) & ~(size_t)255; };
  Workspace w;
  size_t off = 0;
  w.stat_part_off = off;
  off = al(off + (size_t)pb.key_block_slots * pb.Hq * pb.n_obs * sizeof(float2));
  w.stat_fin_off = off;
  off = al(off + (size_t)pb.row_slots * pb.Hq * sizeof(float2));
  w.total = off;
  return w;
}

static SweepArgs make_sweep_args(const Problem& pb, const void* q, const void* k, const int32_t* cu,
                                 void* workspace) {
  const Workspace w = workspace_layout(pb);
  char* ws = (char*)workspace;
  SweepArgs a{};
  a.q = (const char*)q; a.k = (const char*)k; a.cu = cu;
  a.stat_part = (float2*)(ws + w.stat_part_off);
  a.stat_fin = (float2*)(ws + w.stat_fin_off);
  a.scores_out = nullptr;
  a.q_stride_b = pb.q_stride * 2; a.k_stride_b = pb.k_stride * 2;
  a.c = pb.scale * 1.44269504088896340736f;
  a.R = pb.R; a.T = pb.T; a.Hq = pb.Hq; a.Hkv = pb.Hkv; a.Gq = pb.Gq; a.n_obs = pb.n_obs;
  a.row_slots = pb.row_slots;
  a.do_select = 0;
  return a;
}

hipError_t launch_row_stats(const Problem& pb, const void* q, const void* k, const int32_t* cu,
                            void* workspace, hipStream_t s) {
  if (pb.T == 0) return hipSuccess;
  const SweepArgs a = make_sweep_args(pb, q, k, cu, workspace);
  hipLaunchKernelGGL(k_sweep<1>, dim3((unsigned)pb.key_block_slots), dim3(kSweepThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_merge_stats(const Problem& pb, const int32_t* cu, void* workspace, hipStream_t s) {
  if (pb.T == 0) return hipSuccess;
  const SweepArgs a = make_sweep_args(pb, nullptr, nullptr, cu, workspace);
  hipLaunchKernelGGL(k_combine, dim3((unsigned)((pb.row_slots + 31) / 32), (unsigned)pb.Hq), dim3(256),
                     0, s, cu, a.stat_part, a.stat_fin, pb.R, pb.Hq, pb.n_obs, pb.row_slots);
  return hipGetLastError();
}

hipError_t launch_column_sums(const Problem& pb, const void* q, const void* k, const int32_t* cu,
                              void* workspace, float* scores_out, const SelectArgs* sel,
                              hipStream_t s) {
  if (pb.T == 0) return hipSuccess;
  SweepArgs a = make_sweep_args(pb, q, k, cu, workspace);
  a.scores_out = scores_out;
  if (sel != nullptr) { a.sel = *sel; a.do_select = 1; }
  hipLaunchKernelGGL(k_sweep<2>, dim3((unsigned)pb.key_block_slots), dim3(kSweepThreads), 0, s, a);
  return hipGetLastError();
}

}  // namespace up
