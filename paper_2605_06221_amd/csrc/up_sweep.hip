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
// of one sequence, eight waves of 32 keys each.  A wave keeps its keys of the
// current kv head in registers as MFMA operands (8 k-steps) and sweeps all
// query rows of that head's GQA group; the rows stream through LDS in units of
// 128 (coalesced 128-bit loads, padded rows, read back in operand layout),
// shared by the eight waves.  v_mfma_f32_32x32x16_bf16: bf16 products are exact
// in fp32 and accumulate in fp32.
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

constexpr int kUnit = 128;           // query rows per LDS staging unit (4 MFMA row tiles)
constexpr int kQRow = 272;           // LDS bytes per query row: 256 + 16 pad (conflict-free b128 reads)
constexpr int kSweepWaves = 8;
constexpr int kSweepThreads = kSweepWaves * 64;

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

// LDS of one work-group (< 80 KB so that two work-groups share a CU).  The staged query
// rows are dead once the sweep is over, so the selection state reuses their space; the
// per-wave statistics (pass 1) and the per-row constants (pass 2) share another region.
struct SweepSmem {
  union {
    __align__(16) unsigned char q[2][kUnit * kQRow];   // staged query rows (bf16), double-buffered
    struct {
      double o64[kKeyBlock];                           // pass 2: column sums of the block's keys
      SelectSmem sel;
    } tail;
  };
  union {
    float2 wstat[kSweepWaves][kUnit];                  // pass 1: per-wave (reference, sum) per staged row
    __align__(16) float2 cst[2][kUnit];                // pass 2: (negative reference, 1/sum) per staged row
  };
  __align__(16) int rowpos[2][kUnit];                  // local position of each staged row, -1 = no such row
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
  const int key_base = kblock * kKeyBlock + wave * 32;     // first local key of this wave
  const float c = a.c;
  const int rs0 = rowslot_base(c0, r, a.n_obs);

  // ---- key operands of one kv head: one 32-key tile, lane = (key l32, k-slice half)
  bf16x8 kf[8];
  auto load_keys = [&](int g) {
    // keys past the end of the sequence re-read the last key (finite values): pass 1 masks
    // them (such a block is always an edge block), pass 2 never emits their scores
    const int key = imin(key_base + l32, N - 1);
    const char* kp = a.k + (long long)(c0 + key) * a.k_stride_b + (long long)g * 256 + half * 16;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) kf[kk] = as_bf16x8(*(const u32x4*)(kp + kk * 32));
  };

  // ---- staging of one unit of query rows: 2048 pieces of 16 bytes (128 rows x 16), 4 per
  // thread, moved in two rounds of 2.  Thread t owns column t%16 of rows t/16 + 32*i.
  const bool whole_heads = (n_eff % kUnit) == 0;     // a unit never straddles two heads
  const int my_row = tid >> 4;
  const char* q_seq = a.q + (long long)(c0 + first_q) * a.q_stride_b + (tid & 15) * 16;
  u32x4 pre_q[2];
  auto fetch_round = [&](int f, int round) {
    const int g = f / n_units;
    const int u = f - g * n_units;
    if (whole_heads) {
      const int per_head = n_eff / kUnit;
      const int hh = u / per_head;
      const int jj0 = (u - hh * per_head) * kUnit;
      const char* base = q_seq + (long long)(g * a.Gq + hh) * 256 + (long long)(jj0 + my_row) * a.q_stride_b;
#pragma unroll
      for (int i = 0; i < 2; ++i)
        pre_q[i] = *(const u32x4*)(base + (long long)((round * 2 + i) * 32) * a.q_stride_b);
    } else {
      // general case: one division per piece; rows past the end re-read the last row
      // (finite values; their results are discarded through the per-row constants)
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int rho = imin(u * kUnit + my_row + (round * 2 + i) * 32, rows_total - 1);
        int hh, jj;
        divmod((unsigned)rho, (unsigned)n_eff, magic, hh, jj);
        pre_q[i] = *(const u32x4*)(q_seq + (long long)jj * a.q_stride_b + (long long)(g * a.Gq + hh) * 256);
      }
    }
  };
  auto stash_round = [&](int buf, int round) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
      *(u32x4*)(&sm.q[buf][(my_row + (round * 2 + i) * 32) * kQRow + (tid & 15) * 16]) = pre_q[i];
  };
  // per-row constants of a unit: threads 0..127 take one row each
  auto stage_meta = [&](int f, int buf) {
    if (tid < kUnit) {
      const int g = f / n_units;
      const int u = f - g * n_units;
      const int rho = u * kUnit + tid;
      float2 cst = make_float2(-INFINITY, 0.0f);   // no such row: weight exactly zero
      int pos = -1;
      if (rho < rows_total) {
        int hh, jj;
        divmod((unsigned)rho, (unsigned)n_eff, magic, hh, jj);
        pos = first_q + jj;
        if (PASS == 2) cst = a.stat_fin[(size_t)(g * a.Gq + hh) * a.row_slots + rs0 + jj];
      }
      if (PASS == 2) sm.cst[buf][tid] = cst;
      sm.rowpos[buf][tid] = pos;
    }
  };

  double col64 = 0.0;   // pass 2: running column sum of this lane's key

  // ---- one phase = one 32x32 tile: row tile rt of the staged unit against the wave's keys.
  // A phase has a matrix half (8 MFMAs) and a vector half (softmax arithmetic on the 16
  // results per lane).  In program order, two MFMAs of phase rt+1 are followed by a quarter
  // of the vector half of phase rt, four times over, with scheduling barriers in between so
  // that the order (and the register footprint) stays as written: the matrix pipe works on
  // the MFMAs while the wave issues the vector instructions behind them.
  u32x4 qv[8];                         // operand fragments of the row tile whose MFMAs are being issued
  auto load_rows = [&](int buf, int rt) {
    const unsigned char* qrow = &sm.q[buf][(rt * 32 + l32) * kQRow + half * 16];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) qv[kk] = *(const u32x4*)(qrow + kk * 32);
  };
  auto mfma_part = [&](f32x16& acc, int part) {
    if (part == 0) {
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[e] = 0.0f;
    }
#pragma unroll
    for (int kk = 2 * part; kk < 2 * part + 2; ++kk) {
      if (PASS == 1)   // S^T: rows of the result are keys, columns are query rows
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], as_bf16x8(qv[kk]), acc, 0, 0, 0);
      else             // S: rows are query rows, columns are keys
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(qv[kk]), kf[kk], acc, 0, 0, 0);
    }
  };
  float p1_ref = 0.0f, p1_negref = 0.0f, p1_l0 = 0.0f, p1_l1 = 0.0f;   // pass 1 phase state
  float p2_cs0 = 0.0f, p2_cs1 = 0.0f;                                    // pass 2 phase state
  auto valu_part = [&](int buf, int rt, f32x16& acc, int part) {
    if (PASS == 1) {
      // element e = key 8*(e/4) + 4*half + e%4 of the wave's tile, query row rt*32 + l32
      if (part == 0) {
        if (EDGE) {
          const int rp = sm.rowpos[buf][rt * 32 + l32];
#pragma unroll
          for (int e = 0; e < 16; ++e)
            if (key_base + 8 * (e >> 2) + 4 * half + (e & 3) > rp) acc[e] = -INFINITY;
        }
        float m = fmaxf(acc[0], acc[1]);
#pragma unroll
        for (int e = 2; e < 16; ++e) m = fmaxf(m, acc[e]);
        p1_ref = m * c;                          // reference in log2 units
        p1_negref = (EDGE && m == -INFINITY) ? 0.0f : -p1_ref;
        p1_l0 = 0.0f;
        p1_l1 = 0.0f;
      } else if (part < 3) {
#pragma unroll
        for (int e = 8 * (part - 1); e < 8 * part; e += 2) {
          p1_l0 += exp2_hw(fmaf(acc[e], c, p1_negref));
          p1_l1 += exp2_hw(fmaf(acc[e + 1], c, p1_negref));
        }
      } else {
        // merge the two lane halves (same row, the tile's other 16 keys)
        const float ref = p1_ref;
        const float l = p1_l0 + p1_l1;           // 0 when every key was masked (exp2(-inf))
        const float ref_o = __shfl_xor(ref, 32);
        const float l_o = __shfl_xor(l, 32);
        const float mm = fmaxf(ref, ref_o);
        float s_a = l * exp2_hw(ref - mm);
        float s_b = l_o * exp2_hw(ref_o - mm);
        if (EDGE) {
          if (ref == -INFINITY) s_a = 0.0f;
          if (ref_o == -INFINITY) s_b = 0.0f;
        }
        if (half == 0) sm.wstat[wave][rt * 32 + l32] = make_float2(mm, s_a + s_b);
      }
    } else {
      // element e = query row rt*32 + 8*(e/4) + 4*half + e%4, key l32 of the wave's tile; part = e/4
      if (part == 0) { p2_cs0 = 0.0f; p2_cs1 = 0.0f; }
      const int row0 = rt * 32 + 8 * part + 4 * half;
      const f32x4 cs01 = *(const f32x4*)(&sm.cst[buf][row0]);       // rows row0, row0+1
      const f32x4 cs23 = *(const f32x4*)(&sm.cst[buf][row0 + 2]);   // rows row0+2, row0+3
      const float negm[4] = {cs01[0], cs01[2], cs23[0], cs23[2]};
      const float wr[4] = {cs01[1], cs01[3], cs23[1], cs23[3]};
      float x[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        x[i] = fmaf(acc[part * 4 + i], c, negm[i]);
        if (EDGE && key_base + l32 > sm.rowpos[buf][row0 + i]) x[i] = -INFINITY;
      }
      p2_cs0 = fmaf(exp2_hw(x[0]), wr[0], p2_cs0);
      p2_cs1 = fmaf(exp2_hw(x[1]), wr[1], p2_cs1);
      p2_cs0 = fmaf(exp2_hw(x[2]), wr[2], p2_cs0);
      p2_cs1 = fmaf(exp2_hw(x[3]), wr[3], p2_cs1);
      if (part == 3) col64 += (double)(p2_cs0 + p2_cs1);
    }
  };
  // keeps memory accesses (IR level) and all instructions (scheduler) on their side of this point
  // (the running sums pass through the asm statement, so the arithmetic that feeds them
  // cannot be sunk below it either)
  auto pin_order = [&]() {
    if (PASS == 1) asm volatile("" : "+v"(p1_l0), "+v"(p1_l1), "+v"(p1_negref) : : "memory");
    else asm volatile("" : "+v"(p2_cs0), "+v"(p2_cs1) : : "memory");
    __builtin_amdgcn_sched_barrier(0);
  };
  // matrix half of the next row tile (into acc_m) next to the vector half of row tile rt_v (on acc_v)
  auto overlapped = [&](int buf, f32x16& acc_m, int rt_v, f32x16& acc_v) {
#pragma unroll
    for (int part = 0; part < 4; ++part) {
      mfma_part(acc_m, part);
      valu_part(buf, rt_v, acc_v, part);
      pin_order();
    }
  };

  fetch_round(0, 0);
  stash_round(0, 0);
  fetch_round(0, 1);
  stash_round(0, 1);
  stage_meta(0, 0);
  __syncthreads();

  int f = 0;
  for (int g = 0; g < a.Hkv; ++g) {
    load_keys(g);
    for (int u = 0; u < n_units; ++u, ++f) {
      const int buf = f & 1;
      const bool more = f + 1 < n_flat;
      f32x16 accA, accB;

      if (more) fetch_round(f + 1, 0);
      load_rows(buf, 0);
#pragma unroll
      for (int part = 0; part < 4; ++part) mfma_part(accA, part);
      pin_order();
      load_rows(buf, 1);
      overlapped(buf, accB, 0, accA);
      if (more) { stash_round(buf ^ 1, 0); fetch_round(f + 1, 1); }
      load_rows(buf, 2);
      overlapped(buf, accA, 1, accB);
      load_rows(buf, 3);
      overlapped(buf, accB, 2, accA);
#pragma unroll
      for (int part = 0; part < 4; ++part) { valu_part(buf, 3, accB, part); pin_order(); }
      if (more) { stash_round(buf ^ 1, 1); stage_meta(f + 1, buf ^ 1); }
      __syncthreads();

      if (PASS == 1) {
        if (tid < kUnit) {
          // merge the eight waves' statistics of one staged row, write the key block's partial
          const int rho = u * kUnit + tid;
          if (rho < rows_total) {
            float2 st[kSweepWaves];
#pragma unroll
            for (int w2 = 0; w2 < kSweepWaves; ++w2) st[w2] = sm.wstat[w2][tid];
            float mm = st[0].x;
#pragma unroll
            for (int w2 = 1; w2 < kSweepWaves; ++w2) mm = fmaxf(mm, st[w2].x);
            float l = 0.0f;
#pragma unroll
            for (int w2 = 0; w2 < kSweepWaves; ++w2)
              if (st[w2].x != -INFINITY) l += st[w2].y * exp2_hw(st[w2].x - mm);
            int hh, jj;
            divmod((unsigned)rho, (unsigned)n_eff, magic, hh, jj);
            a.stat_part[(size_t)slot * (a.Hq * a.n_obs) + (size_t)(g * a.Gq + hh) * a.n_obs + jj] =
                make_float2(mm, l);
          }
        }
        __syncthreads();   // the statistics buffer is written again by the next unit
      }
    }
  }

  if (PASS == 2) {
    // (the loop's last barrier has passed: the staged rows are dead and their space is reused)
    // the two lane halves hold the same key over different rows: add them (fixed order)
    const double other = __shfl_xor(col64, 32);
    if (half == 0) sm.tail.o64[wave * 32 + l32] = col64 + other;
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
    float sc = 0.0f;
    if (tid < kKeyBlock) {
      const int key = kblock * kKeyBlock + tid;
      if (key < N) {
        const double o = sm.tail.o64[tid] / (double)(n_eff * a.Hq);
        sc = o < 0x1p-64 ? 0.0f : (float)o;
        if (a.scores_out != nullptr) a.scores_out[c0 + key] = sc;
      }
      if (a.do_select) sm.tail.sel.score[tid] = sc;
    }
    if (!a.do_select) return;
    __syncthreads();
    // the block-local top-k and the gather, one selection block after the other
    const int G = a.sel.G;
    const int nb = imin(kKeyBlock / G, ceil_div(N - kblock * kKeyBlock, G));
    for (int b = 0; b < nb; ++b)
      select_block(a.sel, sm.tail.sel, r, c0, N, kblock * (kKeyBlock / G) + b, &sm.tail.sel.score[b * G]);
  }
}

// Merge the per-key-block softmax statistics of every (sequence, window row, head):
// final reference = max of the block references, sum rescaled to it.  A work-group
// handles 32 consecutive window rows of one head (coalesced along the rows); the 32
// threads that share a row each take 16 key blocks per round, all loads in flight.
__global__ __launch_bounds__(1024) void k_combine(const int32_t* __restrict__ cu,
                                                  const float2* __restrict__ stat_part,
                                                  float2* __restrict__ stat_fin, int R, int Hq,
                                                  int n_obs, int row_slots) {
  __shared__ float sh_m[32][33];
  __shared__ double sh_l[32][33];
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
  double L = 0.0;
  for (int b0 = ty * 16; b0 < n_blocks; b0 += 512) {
    float2 v[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
      v[i] = b0 + i < n_blocks ? p[(size_t)(b0 + i) * stride] : make_float2(-INFINITY, 0.0f);
    float mc = v[0].x;
#pragma unroll
    for (int i = 1; i < 16; ++i) mc = fmaxf(mc, v[i].x);
    if (mc != -INFINITY) {
      double Lc = 0.0;
#pragma unroll
      for (int i = 0; i < 16; ++i)
        if (v[i].x != -INFINITY) Lc += (double)(v[i].y * exp2f(v[i].x - mc));
      const float mn = fmaxf(m, mc);
      L = (m == -INFINITY ? 0.0 : L * exp2((double)m - (double)mn)) + Lc * exp2((double)mc - (double)mn);
      m = mn;
    }
  }
  sh_m[ty][tx] = m;
  sh_l[ty][tx] = L;
  __syncthreads();
  if (ty == 0 && live) {
    float mm = -INFINITY;
    for (int i = 0; i < 32; ++i) mm = fmaxf(mm, sh_m[i][tx]);
    double tot = 0.0;
    for (int i = 0; i < 32; ++i)
      if (sh_m[i][tx] != -INFINITY) tot += sh_l[i][tx] * exp2((double)sh_m[i][tx] - (double)mm);
    stat_fin[(size_t)h * row_slots + u] = make_float2(-mm, (float)(1.0 / tot));
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
  hipLaunchKernelGGL(k_combine, dim3((unsigned)((pb.row_slots + 31) / 32), (unsigned)pb.Hq), dim3(1024),
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
