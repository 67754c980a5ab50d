// Token-importance scoring (Eq. 2-3) on the gfx950 matrix cores.
//
// For every sequence, kv head and query row of the observation window the
// operator needs softmax statistics over *all* visible keys before any
// normalised weight is final, so the Q.K^T product runs twice:
//
//   pass 1  S^T = K Q^T tiles; each lane owns one query row and keeps a
//           running (reference, sum) pair -- partial softmax statistics of one
//           key chunk, written per chunk and merged by k_combine.
//   pass 2  S = Q K^T tiles; each lane owns one key column, applies the final
//           per-row (reference, 1/sum) and adds the normalised weights of its
//           rows; column partials are reduced over lanes and waves in a fixed
//           order (double precision), one plane per (kv head, row slab).
//
// Work decomposition: one work-group = (key chunk of CK keys of one sequence,
// kv head, row slab).  Its 8 waves hold their query-row tiles (16 rows each,
// TPW tiles per wave) in registers for the whole chunk; the chunk's keys are
// streamed through LDS in stages of 64 keys, loaded once per work-group with
// coalesced 128-bit loads and read back in MFMA operand layout.  All rows of a
// GQA group share the kv head's keys, so each key byte is fetched from memory
// once per pass.  v_mfma_f32_16x16x32_bf16: products of bf16 values are exact
// in fp32 and are accumulated in fp32.
//
// Logits are handled in log2 units: x = s_raw * c + negref with
// c = scale * log2(e), so the exponential is a bare v_exp_f32.
#include "up_common.h"
#include "up_kernels.h"

namespace up {

constexpr int kWaves = 8;            // waves per work-group
constexpr int kThreads = kWaves * 64;
constexpr int kStage = 64;           // keys per LDS stage (4 MFMA key tiles)
constexpr int kKRow = 272;           // LDS bytes per key row: 256 + 16 pad (conflict-free b128 reads)
constexpr float kTauLog2 = 16.0f;    // pass 1 re-references a row only when its max grows by > 2^16

struct ScoreArgs {
  const char* q;
  const char* k;
  const int32_t* cu;
  float2* stat_part;   // [chunk_slots][Hq * n_obs]  (reference in log2 units, sum)
  float2* stat_fin;    // [row_slots * Hq]           (negative reference, 1/sum)
  double* part_o;      // [Hkv * n_slab][T]
  long long q_stride_b, k_stride_b;   // bytes between tokens
  float c;             // scale * log2(e)
  int R, T, Hq, Hkv, Gq, n_obs, CK, n_slab;
};

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ float exp2_hw(float x) { return __builtin_amdgcn_exp2f(x); }

template <int TPW, int PASS>
__global__ __launch_bounds__(kThreads) void k_score(ScoreArgs a) {
  __shared__ __align__(16) unsigned char ldsK[2][kStage * kKRow];
  __shared__ float colbuf[PASS == 2 ? 2 : 1][PASS == 2 ? 4 : 1][PASS == 2 ? kWaves : 1][PASS == 2 ? 64 : 1];

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int lr = lane & 15;   // operand row/column inside a 16-wide tile
  const int lg = lane >> 4;   // k-slice of the operands; row group of the result

  // ---- which (sequence, chunk, kv head, slab)
  const int slot = blockIdx.x;
  const int r = locate_slot(a.cu, a.R, a.CK, slot);
  const int c0 = a.cu[r];
  const int N = a.cu[r + 1] - c0;
  const int chunk = slot - slot_base(c0, r, a.CK);
  const int k0 = chunk * a.CK;
  if (k0 >= N) return;
  const int k1 = imin(N, k0 + a.CK);
  const int kvh = blockIdx.y / a.n_slab;
  const int slab = blockIdx.y - kvh * a.n_slab;
  const int n_eff = imin(a.n_obs, N);
  const int rows_total = n_eff * a.Gq;               // query rows of this kv head's group
  const int slab_base = slab * (kWaves * TPW * 16);
  const int first_q = N - n_eff;                      // local position of the first window row
  const float c = a.c;

  // ---- stationary query tiles (MFMA operand layout: lane = row lr, k-slice lg)
  bf16x8 qf[TPW][4];
  int rowpos1[TPW];   // pass 1: local position of this lane's row (-1: no such row)
#pragma unroll
  for (int t = 0; t < TPW; ++t) {
    const int rho = slab_base + (wave * TPW + t) * 16 + lr;
    const bool ok = rho < rows_total;
    const int hh = ok ? rho / n_eff : 0;
    const int jj = ok ? rho - hh * n_eff : 0;
    rowpos1[t] = ok ? first_q + jj : -1;
    const char* qp = a.q + (long long)(c0 + first_q + jj) * a.q_stride_b +
                     (long long)(kvh * a.Gq + hh) * 256 + lg * 16;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (ok) v = *(const u32x4*)(qp + kk * 64);
      qf[t][kk] = as_bf16x8(v);
    }
  }

  // ---- per-row state
  // pass 1: one row per (tile, lane): threshold (raw units), negative reference (log2), running sum
  float thr[TPW], negref[TPW], lsum[TPW];
  // pass 2: four rows per (tile, lane): rows 4*lg + e of the tile
  float negm[PASS == 2 ? TPW : 1][4], wrow[PASS == 2 ? TPW : 1][4];
  int rowpos2[PASS == 2 ? TPW : 1][4];
  if (PASS == 1) {
#pragma unroll
    for (int t = 0; t < TPW; ++t) { thr[t] = -INFINITY; negref[t] = 0.0f; lsum[t] = 0.0f; }
  } else {
    const int rs0 = rowslot_base(c0, r, a.n_obs);
#pragma unroll
    for (int t = 0; t < TPW; ++t) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int rho = slab_base + (wave * TPW + t) * 16 + lg * 4 + e;
        const bool ok = rho < rows_total;
        const int hh = ok ? rho / n_eff : 0;
        const int jj = ok ? rho - hh * n_eff : 0;
        float2 st = make_float2(0.0f, 0.0f);
        if (ok) st = a.stat_fin[(size_t)(rs0 + jj) * a.Hq + kvh * a.Gq + hh];
        negm[t][e] = st.x;
        wrow[t][e] = st.y;
        rowpos2[t][e] = ok ? first_q + jj : -1;
      }
    }
  }

  // ---- key stages
  const int n_stage = (k1 - k0 + kStage - 1) / kStage;
  const char* kbase = a.k + (long long)c0 * a.k_stride_b + (long long)kvh * 256;
  u32x4 pre[2];
  auto fetch = [&](int s) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int idx = tid + i * kThreads;       // 1024 pieces of 16 bytes: 64 keys x 16
      const int key = k0 + s * kStage + (idx >> 4);
      u32x4 v = {0u, 0u, 0u, 0u};
      if (key < k1) v = *(const u32x4*)(kbase + (long long)key * a.k_stride_b + (idx & 15) * 16);
      pre[i] = v;
    }
  };
  auto stash = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int idx = tid + i * kThreads;
      *(u32x4*)(&ldsK[buf][(idx >> 4) * kKRow + (idx & 15) * 16]) = pre[i];
    }
  };

  fetch(0);
  stash(0);
  __syncthreads();

  for (int s = 0; s < n_stage; ++s) {
    const int buf = s & 1;
    if (s + 1 < n_stage) fetch(s + 1);
    const int kb = k0 + s * kStage;
    const bool edge = kb + kStage - 1 > first_q;   // some row may not see some key of this stage

#pragma unroll
    for (int kt = 0; kt < 4; ++kt) {
      bf16x8 kf[4];
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
        kf[kk] = as_bf16x8(*(const u32x4*)(&ldsK[buf][(kt * 16 + lr) * kKRow + kk * 64 + lg * 16]));

      if (PASS == 1) {
        // result element e: key kb + kt*16 + 4*lg + e, query row lr of tile t
        const int key0 = kb + kt * 16 + lg * 4;
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
          f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
          for (int kk = 0; kk < 4; ++kk)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[kk], qf[t][kk], acc, 0, 0, 0);
          if (edge) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (key0 + e > rowpos1[t]) acc[e] = -INFINITY;
          }
          const float tmax = fmaxf(fmaxf(acc[0], acc[1]), fmaxf(acc[2], acc[3]));
          if (tmax > thr[t]) {
            const float ref = tmax * c;                       // new reference, log2 units
            lsum[t] *= exp2_hw(-negref[t] - ref);             // old reference - new reference
            negref[t] = -ref;
            thr[t] = tmax + kTauLog2 / c;
          }
#pragma unroll
          for (int e = 0; e < 4; ++e) lsum[t] += exp2_hw(fmaf(acc[e], c, negref[t]));
        }
      } else {
        // result element e: query row 4*lg + e of tile t, key kb + kt*16 + lr
        const int key = kb + kt * 16 + lr;
        float col = 0.0f;
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
          f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
          for (int kk = 0; kk < 4; ++kk)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qf[t][kk], kf[kk], acc, 0, 0, 0);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            float x = fmaf(acc[e], c, negm[t][e]);
            if (edge && key > rowpos2[t][e]) x = -INFINITY;
            col = fmaf(exp2_hw(x), wrow[t][e], col);
          }
        }
        colbuf[buf][kt][wave][lane] = col;
      }
    }

    if (s + 1 < n_stage) stash(buf ^ 1);
    __syncthreads();

    if (PASS == 2 && tid < 64) {
      // fixed-order reduction of one stage's 64 key columns over waves and row groups
      const int kt = tid >> 4, kc = tid & 15;
      double sum = 0.0;
#pragma unroll
      for (int w = 0; w < kWaves; ++w)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) sum += (double)colbuf[buf][kt][w][g4 * 16 + kc];
      const int key = kb + kt * 16 + kc;
      if (key < k1) a.part_o[(size_t)blockIdx.y * a.T + c0 + key] = sum;
    }
  }

  if (PASS == 1) {
    // merge the four lanes (k-slices lg) that share a row, then write the chunk's partial
#pragma unroll
    for (int t = 0; t < TPW; ++t) {
      float ref = thr[t] == -INFINITY ? -INFINITY : -negref[t];
      float l = lsum[t];
#pragma unroll
      for (int sh = 16; sh <= 32; sh <<= 1) {
        const float ref_o = __shfl_xor(ref, sh);
        const float l_o = __shfl_xor(l, sh);
        const float m = fmaxf(ref, ref_o);
        const float s_a = ref == -INFINITY ? 0.0f : l * exp2_hw(ref - m);
        const float s_b = ref_o == -INFINITY ? 0.0f : l_o * exp2_hw(ref_o - m);
        ref = m;
        l = s_a + s_b;
      }
      const int rho = slab_base + (wave * TPW + t) * 16 + lr;
      if (lg == 0 && rho < rows_total) {
        const int hh = rho / n_eff;
        const int jj = rho - hh * n_eff;
        a.stat_part[(size_t)slot * (a.Hq * a.n_obs) + (kvh * a.Gq + hh) * a.n_obs + jj] =
            make_float2(ref, l);
      }
    }
  }
}

// Merge the per-chunk softmax statistics of every (sequence, window row, head):
// final reference = max of the chunk references, sum rescaled to it (double).
__global__ __launch_bounds__(256) void k_combine(const int32_t* __restrict__ cu,
                                                 const float2* __restrict__ stat_part,
                                                 float2* __restrict__ stat_fin, int R, int Hq,
                                                 int n_obs, int CK, int row_slots) {
  const int gid = blockIdx.x * 256 + threadIdx.x;
  const int u = gid / Hq;
  const int h = gid - u * Hq;
  if (u >= row_slots) return;
  const int r = locate_rowslot(cu, R, n_obs, u);
  const int c0 = cu[r];
  const int N = cu[r + 1] - c0;
  const int jj = u - rowslot_base(c0, r, n_obs);
  const int n_eff = imin(n_obs, N);
  if (jj >= n_eff) return;
  const int n_chunks = ceil_div(N, CK);
  const size_t row = (size_t)h * n_obs + jj;
  const size_t stride = (size_t)Hq * n_obs;
  const float2* p = stat_part + (size_t)slot_base(c0, r, CK) * stride + row;
  float m = -INFINITY;
  for (int ch = 0; ch < n_chunks; ++ch) m = fmaxf(m, p[(size_t)ch * stride].x);
  double L = 0.0;
  for (int ch = 0; ch < n_chunks; ++ch) {
    const float2 st = p[(size_t)ch * stride];
    if (st.x != -INFINITY) L += (double)st.y * exp2((double)st.x - (double)m);
  }
  stat_fin[(size_t)u * Hq + h] = make_float2(-m, (float)(1.0 / L));
}

// scores_out[i] = (sum of the partial planes) / (n_eff * Hq), floored at 2^-64.
__global__ __launch_bounds__(256) void k_finalise(const int32_t* __restrict__ cu,
                                                  const double* __restrict__ part_o, int n_parts,
                                                  int R, int T, int n_obs, int Hq,
                                                  float* __restrict__ scores_out) {
  const int tok = blockIdx.x * 256 + threadIdx.x;
  if (tok >= T) return;
  const int r = locate_token(cu, R, tok);
  const int N = cu[r + 1] - cu[r];
  double o = 0.0;
  for (int p = 0; p < n_parts; ++p) o += part_o[(size_t)p * T + tok];
  o = o / (double)(imin(n_obs, N) * Hq);
  scores_out[tok] = o < 0x1p-64 ? 0.0f : (float)o;
}

Workspace workspace_layout(const Problem& pb) {
  auto al = [](size_t x) { return (x + 255) & ~(size_t)255; };
  Workspace w;
  size_t off = 0;
  w.stat_part_off = off;
  off = al(off + (size_t)pb.chunk_slots * pb.Hq * pb.n_obs * sizeof(float2));
  w.stat_fin_off = off;
  off = al(off + (size_t)pb.row_slots * pb.Hq * sizeof(float2));
  w.part_o_off = off;
  off = al(off + (size_t)pb.Hkv * pb.n_slab * pb.T * sizeof(double));
  w.total = off;
  return w;
}

template <int PASS>
static hipError_t launch_pass(const Problem& pb, const ScoreArgs& a, hipStream_t s) {
  const dim3 grid((unsigned)pb.chunk_slots, (unsigned)(pb.Hkv * pb.n_slab));
  const dim3 block(kThreads);
  switch (pb.tpw) {
    case 1: hipLaunchKernelGGL((k_score<1, PASS>), grid, block, 0, s, a); break;
    case 2: hipLaunchKernelGGL((k_score<2, PASS>), grid, block, 0, s, a); break;
    case 3: hipLaunchKernelGGL((k_score<3, PASS>), grid, block, 0, s, a); break;
    case 4: hipLaunchKernelGGL((k_score<4, PASS>), grid, block, 0, s, a); break;
    case 5: hipLaunchKernelGGL((k_score<5, PASS>), grid, block, 0, s, a); break;
    case 6: hipLaunchKernelGGL((k_score<6, PASS>), grid, block, 0, s, a); break;
    case 7: hipLaunchKernelGGL((k_score<7, PASS>), grid, block, 0, s, a); break;
    default: hipLaunchKernelGGL((k_score<8, PASS>), grid, block, 0, s, a); break;
  }
  return hipGetLastError();
}

static ScoreArgs make_score_args(const Problem& pb, const void* q, const void* k, const int32_t* cu,
                                 void* workspace) {
  const Workspace w = workspace_layout(pb);
  char* ws = (char*)workspace;
  ScoreArgs a;
  a.q = (const char*)q; a.k = (const char*)k; a.cu = cu;
  a.stat_part = (float2*)(ws + w.stat_part_off);
  a.stat_fin = (float2*)(ws + w.stat_fin_off);
  a.part_o = (double*)(ws + w.part_o_off);
  a.q_stride_b = pb.q_stride * 2; a.k_stride_b = pb.k_stride * 2;
  a.c = pb.scale * 1.44269504088896340736f;
  a.R = pb.R; a.T = pb.T; a.Hq = pb.Hq; a.Hkv = pb.Hkv; a.Gq = pb.Gq; a.n_obs = pb.n_obs;
  a.CK = pb.CK; a.n_slab = pb.n_slab;
  return a;
}

hipError_t launch_score_phase(const Problem& pb, int phase, const void* q, const void* k,
                              const int32_t* cu, void* workspace, hipStream_t s) {
  if (pb.T == 0) return hipSuccess;
  const ScoreArgs a = make_score_args(pb, q, k, cu, workspace);
  if (phase == 1) return launch_pass<1>(pb, a, s);
  if (phase == 2) {
    const long long threads = (long long)pb.row_slots * pb.Hq;
    hipLaunchKernelGGL(k_combine, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, cu,
                       a.stat_part, a.stat_fin, pb.R, pb.Hq, pb.n_obs, pb.CK, pb.row_slots);
    return hipGetLastError();
  }
  return launch_pass<2>(pb, a, s);
}

hipError_t launch_score_passes(const Problem& pb, const void* q, const void* k, const int32_t* cu,
                               void* workspace, hipStream_t s) {
  for (int phase = 1; phase <= 3; ++phase) {
    const hipError_t e = launch_score_phase(pb, phase, q, k, cu, workspace, s);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_finalise_scores(const Problem& pb, const int32_t* cu, const void* workspace,
                                  float* scores_out, hipStream_t s) {
  if (pb.T == 0) return hipSuccess;
  const Workspace w = workspace_layout(pb);
  const double* part_o = (const double*)((const char*)workspace + w.part_o_off);
  hipLaunchKernelGGL(k_finalise, dim3((unsigned)((pb.T + 255) / 256)), dim3(256), 0, s, cu, part_o,
                     pb.Hkv * pb.n_slab, pb.R, pb.T, pb.n_obs, pb.Hq, scores_out);
  return hipGetLastError();
}

}  // namespace up
