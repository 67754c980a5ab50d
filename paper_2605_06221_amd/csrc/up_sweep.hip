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
// Work decomposition ("key-stationary"): one work-group = 256 or 512 consecutive
// keys of one sequence, eight waves of 32 or 64 keys each (KT = 1 or 2 key tiles
// per wave; the larger block halves the per-key cost of staging, merging and LDS
// reads and is used when it still yields enough work-groups).  A wave keeps its
// keys of the current kv head in registers as MFMA operands and sweeps all
// query rows of that head's GQA group; the rows stream through LDS in units of
// 128 (coalesced 128-bit loads, padded rows, read back in operand layout),
// shared by the eight waves.  v_mfma_f32_32x32x16_bf16: bf16 products are exact
// in fp32 and accumulate in fp32.
//
// Because a pass-2 work-group ends with the final scores of its consecutive
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

// LDS of one work-group.  The staged query rows are dead once the sweep is over, so the
// selection state reuses their space.  Small per-unit tables live in rings: a unit's vector
// work trails its matrix work by one phase and crosses the unit barrier, so the tables of
// three units can be live at once.
struct SweepSmem {
  union {
    __align__(16) unsigned char q[2][kUnit * kQRow];   // staged query rows (bf16), double-buffered
    struct {
      double o64[kMaxKeyBlock];                        // pass 2: column sums of the block's keys
      SelectSmem sel;
    } tail;
  };
  union {
    float2 wstat[3][kSweepWaves][kUnit];               // pass 1: per-wave (reference, sum) per staged row
    __align__(16) float2 cst[4][kUnit];                // pass 2: (negative reference, 1/sum) per staged row
  };
  __align__(16) int rowpos[4][kUnit];                  // local position of each staged row, -1 = no such row
};

// Position of a staging unit inside the sweep: kv head g, unit u of that head's rows and,
// when units never straddle query heads, the query head hh inside the group and the first
// window row jj0 of the unit.  Advanced without divisions.
struct UnitCursor {
  int g, u, hh, jj0;
  __device__ __forceinline__ void advance(int n_units, int n_eff) {
    ++u;
    jj0 += kUnit;
    if (jj0 >= n_eff) { jj0 = 0; ++hh; }
    if (u == n_units) { u = 0; ++g; hh = 0; jj0 = 0; }
  }
};

template <int PASS, bool EDGE, int KT>
__device__ __forceinline__ void sweep_block(const SweepArgs& a, SweepSmem& sm, int r, int c0, int N,
                                            int kblock, int slot) {
  constexpr int KB = 256 * KT;                              // keys per work-group
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int l32 = lane & 31, half = lane >> 5;
  const int n_eff = imin(a.n_obs, N);
  const int first_q = N - n_eff;
  const int rows_total = n_eff * a.Gq;
  const int n_units = (rows_total + kUnit - 1) / kUnit;
  const int n_flat = a.Hkv * n_units;
  const unsigned magic = 0xFFFFFFFFu / (unsigned)n_eff;
  const int key_base = kblock * KB + wave * 32 * KT;       // first local key of this wave
  const float c = a.c;
  const int rs0 = rowslot_base(c0, r, a.n_obs);
  const bool whole_heads = (n_eff % kUnit) == 0;           // a unit never straddles two query heads

  // ---- key operands of one kv head: KT tiles of 32 keys, lane = (key l32, k-slice half).
  // Keys past the end of the sequence re-read the last key (finite values): pass 1 masks
  // them (such a block is always an edge block), pass 2 never emits their scores.
  bf16x8 kf[KT][8];
  const char* k_lane[KT];
#pragma unroll
  for (int t = 0; t < KT; ++t)
    k_lane[t] = a.k + (long long)(c0 + imin(key_base + 32 * t + l32, N - 1)) * a.k_stride_b + half * 16;
  auto load_keys = [&](int g) {
#pragma unroll
    for (int t = 0; t < KT; ++t)
#pragma unroll
      for (int kk = 0; kk < 8; ++kk)
        kf[t][kk] = as_bf16x8(*(const u32x4*)(k_lane[t] + (long long)g * 256 + kk * 32));
  };
  // pulls the two cache lines of every key row of head g towards the CU well before
  // load_keys(g) needs them (the values are only summed so that the loads stay alive)
  int touched = 0;
  auto touch_keys = [&](int g) {
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      const char* row = k_lane[t] - half * 16 + (long long)g * 256;
      touched += *(const int*)(row + half * 128);
    }
  };

  // ---- staging of one unit of query rows: 2048 pieces of 16 bytes (128 rows x 16), 4 per
  // thread: column t%16 of rows t/16 + 32*i.  Fetched into registers right after a unit
  // barrier, written to LDS just before the next one.
  const int my_row = tid >> 4;
  const char* q_seq = a.q + (long long)(c0 + first_q) * a.q_stride_b + (tid & 15) * 16;
  const long long my_row_off = (long long)my_row * a.q_stride_b;
  u32x4 pre_q[4];
  auto fetch_unit = [&](const UnitCursor& uc) {
    if (whole_heads) {
      const char* base = q_seq + (long long)(uc.g * a.Gq + uc.hh) * 256 + (long long)uc.jj0 * a.q_stride_b + my_row_off;
#pragma unroll
      for (int i = 0; i < 4; ++i) pre_q[i] = *(const u32x4*)(base + (long long)(i * 32) * a.q_stride_b);
    } else {
      // general case: one division per piece; rows past the end re-read the last row
      // (finite values; their results are discarded through the per-row constants)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int rho = imin(uc.u * kUnit + my_row + i * 32, rows_total - 1);
        int hh, jj;
        divmod((unsigned)rho, (unsigned)n_eff, magic, hh, jj);
        pre_q[i] = *(const u32x4*)(q_seq + (long long)jj * a.q_stride_b + (long long)(uc.g * a.Gq + hh) * 256);
      }
    }
  };
  auto stash_unit = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      *(u32x4*)(&sm.q[buf][(my_row + i * 32) * kQRow + (tid & 15) * 16]) = pre_q[i];
  };
  // row of a unit -> (query head inside the group, window row), or false if there is no such row
  auto unit_row = [&](const UnitCursor& uc, int row, int& hh, int& jj) -> bool {
    const int rho = uc.u * kUnit + row;
    if (whole_heads) { hh = uc.hh; jj = uc.jj0 + row; return true; }
    if (rho >= rows_total) { hh = 0; jj = 0; return false; }
    divmod((unsigned)rho, (unsigned)n_eff, magic, hh, jj);
    return true;
  };
  // per-row tables of a unit: threads 0..127 take one row each
  auto stage_meta = [&](const UnitCursor& uc, int ring) {
    if (tid < kUnit) {
      float2 cst = make_float2(-INFINITY, 0.0f);   // no such row: weight exactly zero
      int pos = -1, hh, jj;
      if (unit_row(uc, tid, hh, jj)) {
        pos = first_q + jj;
        if (PASS == 2) cst = a.stat_fin[(size_t)(uc.g * a.Gq + hh) * a.row_slots + rs0 + jj];
      }
      if (PASS == 2) sm.cst[ring][tid] = cst;
      sm.rowpos[ring][tid] = pos;
    }
  };

  double col64[KT];   // pass 2: running column sums of this lane's keys
#pragma unroll
  for (int t = 0; t < KT; ++t) col64[t] = 0.0;

  // ---- one phase = row tile rt of the staged unit against the wave's KT key tiles.
  // A phase has a matrix half (8 MFMAs per key tile) and a vector half (softmax arithmetic on
  // the 16 results per lane and tile).  In program order, the MFMAs of one k-step are followed
  // by the LDS read that refills the operand register just consumed with the next phase's
  // rows, and by an eighth of the vector half of the previous phase; scheduling barriers keep
  // that order (and the register footprint) as written, so no LDS latency is exposed and a
  // dependent MFMA is never the next instruction after its predecessor.
  u32x4 qv[8];                         // operand fragments: row tile of the phase being issued / the next one
  auto load_rows_slice = [&](int buf, int rt, int kk) {
    qv[kk] = *(const u32x4*)(&sm.q[buf][(rt * 32 + l32) * kQRow + half * 16 + kk * 32]);
  };
  auto mfma_slice = [&](f32x16 (&acc)[KT], int kk) {
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      if (kk == 0) {
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.0f;
      }
      if (PASS == 1)   // S^T: rows of the result are keys, columns are query rows
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t][kk], as_bf16x8(qv[kk]), acc[t], 0, 0, 0);
      else             // S: rows are query rows, columns are keys
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(qv[kk]), kf[t][kk], acc[t], 0, 0, 0);
    }
  };
  // pass 1 phase state: partial maxima, reference, running sums, lane-half exchange
  float p1_m0 = 0.0f, p1_m1 = 0.0f, p1_ref = 0.0f, p1_negref = 0.0f, p1_l0 = 0.0f, p1_l1 = 0.0f;
  float p1_ref_o = 0.0f, p1_l_o = 0.0f;
  float p2_cs[KT][2];                   // pass 2 phase state
  // vector slice `sl` (0..7) of the phase (unit with table ring slots ring4 / ring3, row tile rt)
  auto valu_slice = [&](int ring4, int ring3, int rt, f32x16 (&acc)[KT], int sl) {
    if (PASS == 1) {
      // element e of tile t = key 32*t + 8*(e/4) + 4*half + e%4 of the wave's keys, query row rt*32 + l32
      if (sl == 0) {
        if (EDGE) {
          const int rp = sm.rowpos[ring4][rt * 32 + l32];
#pragma unroll
          for (int t = 0; t < KT; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e)
              if (key_base + 32 * t + 8 * (e >> 2) + 4 * half + (e & 3) > rp) acc[t][e] = -INFINITY;
        }
        p1_m0 = fmaxf(fmaxf(acc[0][0], acc[0][1]), fmaxf(acc[0][2], acc[0][3]));
        p1_m1 = fmaxf(fmaxf(acc[0][4], acc[0][5]), fmaxf(acc[0][6], acc[0][7]));
        if (KT == 2) {
          p1_m0 = fmaxf(p1_m0, fmaxf(fmaxf(acc[KT - 1][0], acc[KT - 1][1]), fmaxf(acc[KT - 1][2], acc[KT - 1][3])));
          p1_m1 = fmaxf(p1_m1, fmaxf(fmaxf(acc[KT - 1][4], acc[KT - 1][5]), fmaxf(acc[KT - 1][6], acc[KT - 1][7])));
        }
      } else if (sl == 1) {
#pragma unroll
        for (int t = 0; t < KT; ++t) {
          p1_m0 = fmaxf(p1_m0, fmaxf(fmaxf(acc[t][8], acc[t][9]), fmaxf(acc[t][10], acc[t][11])));
          p1_m1 = fmaxf(p1_m1, fmaxf(fmaxf(acc[t][12], acc[t][13]), fmaxf(acc[t][14], acc[t][15])));
        }
        const float m = fmaxf(p1_m0, p1_m1);
        p1_ref = m * c;                          // reference in log2 units
        p1_negref = (EDGE && m == -INFINITY) ? 0.0f : -p1_ref;
        p1_l0 = 0.0f;
        p1_l1 = 0.0f;
      } else if (sl < 6) {
        const int e0 = 4 * (sl - 2);
#pragma unroll
        for (int t = 0; t < KT; ++t) {
          p1_l0 += exp2_hw(fmaf(acc[t][e0], c, p1_negref));
          p1_l1 += exp2_hw(fmaf(acc[t][e0 + 1], c, p1_negref));
          p1_l0 += exp2_hw(fmaf(acc[t][e0 + 2], c, p1_negref));
          p1_l1 += exp2_hw(fmaf(acc[t][e0 + 3], c, p1_negref));
        }
      } else if (sl == 6) {
        // exchange with the other lane half (same row, the other keys of the tiles)
        p1_l0 += p1_l1;                          // 0 when every key was masked (exp2(-inf))
        p1_ref_o = __shfl_xor(p1_ref, 32);
        p1_l_o = __shfl_xor(p1_l0, 32);
      } else {
        const float mm = fmaxf(p1_ref, p1_ref_o);
        float s_a = p1_l0 * exp2_hw(p1_ref - mm);
        float s_b = p1_l_o * exp2_hw(p1_ref_o - mm);
        if (EDGE) {
          if (p1_ref == -INFINITY) s_a = 0.0f;
          if (p1_ref_o == -INFINITY) s_b = 0.0f;
        }
        if (half == 0) sm.wstat[ring3][wave][rt * 32 + l32] = make_float2(mm, s_a + s_b);
      }
    } else {
      // element e of tile t = query row rt*32 + 8*(e/4) + 4*half + e%4, key 32*t + l32;
      // slice sl handles e = 2*sl, 2*sl + 1 (two consecutive rows: one 16-byte table read)
      if (sl == 0) {
#pragma unroll
        for (int t = 0; t < KT; ++t) { p2_cs[t][0] = 0.0f; p2_cs[t][1] = 0.0f; }
      }
      const int row0 = rt * 32 + 8 * (sl >> 1) + 4 * half + 2 * (sl & 1);
      const f32x4 cs = *(const f32x4*)(&sm.cst[ring4][row0]);   // (negref, w) of rows row0, row0+1
      int rp0 = 0, rp1 = 0;
      if (EDGE) { rp0 = sm.rowpos[ring4][row0]; rp1 = sm.rowpos[ring4][row0 + 1]; }
#pragma unroll
      for (int t = 0; t < KT; ++t) {
        float x0 = fmaf(acc[t][2 * sl], c, cs[0]);
        float x1 = fmaf(acc[t][2 * sl + 1], c, cs[2]);
        if (EDGE) {
          if (key_base + 32 * t + l32 > rp0) x0 = -INFINITY;
          if (key_base + 32 * t + l32 > rp1) x1 = -INFINITY;
        }
        p2_cs[t][0] = fmaf(exp2_hw(x0), cs[1], p2_cs[t][0]);
        p2_cs[t][1] = fmaf(exp2_hw(x1), cs[3], p2_cs[t][1]);
      }
      if (sl == 7) {
#pragma unroll
        for (int t = 0; t < KT; ++t) col64[t] += (double)(p2_cs[t][0] + p2_cs[t][1]);
      }
    }
  };
  // keeps memory accesses (IR level) and all instructions (scheduler) on their side of this
  // point; the running values pass through the asm statement, so the arithmetic that feeds
  // them cannot be sunk below it either
  auto pin_order = [&]() {
    if (PASS == 1)
      asm volatile("" : "+v"(p1_l0), "+v"(p1_l1), "+v"(p1_negref), "+v"(p1_m0), "+v"(p1_m1) : : "memory");
    else
      asm volatile("" : "+v"(p2_cs[0][0]), "+v"(p2_cs[0][1]), "+v"(p2_cs[KT - 1][0]), "+v"(p2_cs[KT - 1][1]) : : "memory");
    __builtin_amdgcn_sched_barrier(0);
  };
  // matrix half of a phase into acc_m, refilling the operand registers from (buf_n, rt_n),
  // next to the vector half of the previous phase (acc_v; tables ring4_v / ring3_v, row tile rt_v)
  auto overlapped = [&](f32x16 (&acc_m)[KT], int buf_n, int rt_n, bool refill, bool with_valu, int ring4_v,
                        int ring3_v, int rt_v, f32x16 (&acc_v)[KT]) {
#pragma unroll
    for (int sl = 0; sl < 8; ++sl) {
      mfma_slice(acc_m, sl);
      if (refill) load_rows_slice(buf_n, rt_n, sl);
      if (with_valu) valu_slice(ring4_v, ring3_v, rt_v, acc_v, sl);
      pin_order();
    }
  };
  // pass 1: merge the eight waves' statistics of the 128 rows of unit `uc` (ring slot ring3)
  // and write the key block's partial.  One wave does it (the waves take turns), two rows per lane.
  auto merge_unit = [&](const UnitCursor& uc, int ring3) {
#pragma unroll
    for (int rr = 0; rr < 2; ++rr) {
      const int row = lane + 64 * rr;
      float2 st[kSweepWaves];
#pragma unroll
      for (int w2 = 0; w2 < kSweepWaves; ++w2) st[w2] = sm.wstat[ring3][w2][row];
      float mm = st[0].x;
#pragma unroll
      for (int w2 = 1; w2 < kSweepWaves; ++w2) mm = fmaxf(mm, st[w2].x);
      float l = 0.0f;
#pragma unroll
      for (int w2 = 0; w2 < kSweepWaves; ++w2)
        l += st[w2].x == -INFINITY ? 0.0f : st[w2].y * exp2_hw(st[w2].x - mm);
      int hh, jj;
      if (unit_row(uc, row, hh, jj))
        a.stat_part[(size_t)slot * (a.Hq * a.n_obs) + (size_t)(uc.g * a.Gq + hh) * a.n_obs + jj] = make_float2(mm, l);
    }
  };

  // ---- prologue: unit 0 staged and visible, unit 1 in flight, first rows in registers
  UnitCursor cur{0, 0, 0, 0};      // unit whose matrix work is being issued
  UnitCursor prev = cur;           // the unit before it (its last vector half is still pending)
  UnitCursor nxt = cur;            // unit being staged for the next iteration
  fetch_unit(cur);
  stash_unit(0);
  stage_meta(cur, 0);
  load_keys(0);
  __syncthreads();
  nxt.advance(n_units, n_eff);
  if (n_flat > 1) fetch_unit(nxt);
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) load_rows_slice(0, 0, kk);

  f32x16 accA[KT], accB[KT];
  for (int f = 0; f < n_flat; ++f) {
    const int buf = f & 1;
    const bool more = f + 1 < n_flat;
    const bool head_ends = more && cur.u == n_units - 1;   // the next unit belongs to the next kv head
    const int r4 = f & 3, r3 = f % 3;
    const int pr4 = (f + 3) & 3, pr3 = (f + 2) % 3;         // ring slots of unit f-1

    if (head_ends) touch_keys(cur.g + 1);   // needed four phases from now
    // phase 0 of unit f next to the last vector half of unit f-1
    overlapped(accA, buf, 1, true, f > 0, pr4, pr3, 3, accB);
    overlapped(accB, buf, 2, true, true, r4, r3, 0, accA);
    overlapped(accA, buf, 3, true, true, r4, r3, 1, accB);
    if (more) { stash_unit(buf ^ 1); stage_meta(nxt, (f + 1) & 3); }
    __syncthreads();     // unit f+1 is visible; every read of unit f's rows has completed
    if (PASS == 1 && f > 0 && wave == (f & (kSweepWaves - 1))) merge_unit(prev, pr3);
    const int next_g = cur.g + 1;
    prev = cur;
    cur = nxt;
    if (f + 2 < n_flat) { nxt.advance(n_units, n_eff); fetch_unit(nxt); }
    // last phase of unit f; the operand registers are refilled with the first rows of unit f+1
    overlapped(accB, buf ^ 1, 0, more, true, r4, r3, 2, accA);
    if (head_ends) load_keys(next_g);       // this head's last MFMA has been issued
  }
  // the last vector half, then (pass 1) the statistics of the last unit
#pragma unroll
  for (int sl = 0; sl < 8; ++sl) { valu_slice((n_flat + 3) & 3, (n_flat + 2) % 3, 3, accB, sl); pin_order(); }
  __syncthreads();
  if (PASS == 1 && wave == 0) merge_unit(prev, (n_flat + 2) % 3);

  if (PASS == 2) {
    // (a barrier has passed since the last read of the staged rows: their space is reused)
    // the two lane halves hold the same keys over different rows: add them (fixed order)
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      const double other = __shfl_xor(col64[t], 32);
      if (half == 0) sm.tail.o64[wave * 32 * KT + 32 * t + l32] = col64[t] + other;
    }
  }
  if (touched == 0x7fffffff) sm.rowpos[0][0] = touched;   // never true for real data; keeps the touch loads
}

template <int PASS, int KT>
__global__ __launch_bounds__(kSweepThreads) void k_sweep(SweepArgs a) {
  constexpr int KB = 256 * KT;
  __shared__ SweepSmem sm;
  const int slot = blockIdx.x;
  const int r = locate_slot(a.cu, a.R, KB, slot);
  const int c0 = a.cu[r];
  const int N = a.cu[r + 1] - c0;
  const int kblock = slot - slot_base(c0, r, KB);
  if (kblock * KB >= N) return;
  const int n_eff = imin(a.n_obs, N);
  // causal masking and the ragged end only matter where keys reach the query window
  const bool edge = (kblock + 1) * KB - 1 > N - n_eff;
  if (edge) sweep_block<PASS, true, KT>(a, sm, r, c0, N, kblock, slot);
  else sweep_block<PASS, false, KT>(a, sm, r, c0, N, kblock, slot);

  if (PASS == 2) {
    __syncthreads();
    const int tid = threadIdx.x;
    float sc = 0.0f;
    if (tid < KB) {
      const int key = kblock * KB + tid;
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
    const int nb = imin(KB / G, ceil_div(N - kblock * KB, G));
    for (int b = 0; b < nb; ++b)
      select_block(a.sel, sm.tail.sel, r, c0, N, kblock * (KB / G) + b, &sm.tail.sel.score[b * G]);
  }
}

// Merge the per-key-block softmax statistics of every (sequence, window row, head):
// final reference = max of the block references, sum rescaled to it.  A work-group
// handles 32 consecutive window rows of one head (coalesced along the rows); the 32
// threads that share a row each take 16 key blocks per round, all loads in flight.
__global__ __launch_bounds__(1024) void k_combine(const int32_t* __restrict__ cu,
                                                  const float2* __restrict__ stat_part,
                                                  float2* __restrict__ stat_fin, int R, int Hq,
                                                  int n_obs, int row_slots, int key_block) {
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
      n_blocks = ceil_div(N, key_block);
      p = stat_part + (size_t)slot_base(c0, r, key_block) * stride + (size_t)h * n_obs + jj;
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
  if (pb.key_block == 512)
    hipLaunchKernelGGL((k_sweep<1, 2>), dim3((unsigned)pb.key_block_slots), dim3(kSweepThreads), 0, s, a);
  else
    hipLaunchKernelGGL((k_sweep<1, 1>), dim3((unsigned)pb.key_block_slots), dim3(kSweepThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_merge_stats(const Problem& pb, const int32_t* cu, void* workspace, hipStream_t s) {
  if (pb.T == 0) return hipSuccess;
  const SweepArgs a = make_sweep_args(pb, nullptr, nullptr, cu, workspace);
  hipLaunchKernelGGL(k_combine, dim3((unsigned)((pb.row_slots + 31) / 32), (unsigned)pb.Hq), dim3(1024),
                     0, s, cu, a.stat_part, a.stat_fin, pb.R, pb.Hq, pb.n_obs, pb.row_slots, pb.key_block);
  return hipGetLastError();
}

hipError_t launch_column_sums(const Problem& pb, const void* q, const void* k, const int32_t* cu,
                              void* workspace, float* scores_out, const SelectArgs* sel,
                              hipStream_t s) {
  if (pb.T == 0) return hipSuccess;
  SweepArgs a = make_sweep_args(pb, q, k, cu, workspace);
  a.scores_out = scores_out;
  if (sel != nullptr) { a.sel = *sel; a.do_select = 1; }
  if (pb.key_block == 512)
    hipLaunchKernelGGL((k_sweep<2, 2>), dim3((unsigned)pb.key_block_slots), dim3(kSweepThreads), 0, s, a);
  else
    hipLaunchKernelGGL((k_sweep<2, 1>), dim3((unsigned)pb.key_block_slots), dim3(kSweepThreads), 0, s, a);
  return hipGetLastError();
}

}  // namespace up
