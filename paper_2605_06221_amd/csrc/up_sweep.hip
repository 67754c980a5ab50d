// Token-importance scoring (Eq. 2-3) on the gfx950 matrix cores, with the
// block-local selection attached to the second pass.
//
// The softmax of a query row is normalised over *all* visible keys, so the
// Q.K^T product runs twice:
//
//   pass 1 (row statistics)  S^T = K Q^T tiles: a lane owns one query row and
//           16 of its wave's 32 keys; it takes the row maximum and the sum of
//           exponentials over those keys.  Lane halves and the waves of the
//           work-group are merged, giving one (reference, sum) pair per row and
//           key block; k_combine merges the key blocks of a sequence.
//   pass 2 (column sums)  S = Q K^T tiles: a lane owns one key and 16 query
//           rows per tile; it applies each row's final (reference, 1/sum) and
//           adds the normalised weights (fp32 inside a tile, fp64 across tiles).
//           A wave sees every row of every head it sweeps for its keys, so no
//           atomics are needed and the summation order is fixed.
//
// Work decomposition ("key-stationary"): one work-group = 512 or 256 consecutive
// keys of one sequence, NW = 16 or 8 waves of 32 keys each.  A wave keeps its
// keys of the current kv head in registers as MFMA operands and sweeps all
// query rows of that head's GQA group; the rows stream through LDS in units of
// 128 (coalesced 128-bit loads, padded rows, read back in operand layout),
// shared by all waves.  Sixteen waves put four on every SIMD, which covers the
// LDS, barrier and dependency latencies of one another; the program order
// inside a wave is the plain one (operands, 8 MFMAs, vector work on the 16
// results).  v_mfma_f32_32x32x16_bf16: bf16 products are exact in fp32 and
// accumulate in fp32; fp32 operands take v_mfma_f32_32x32x2_f32.
//
// When a batch has too few key blocks to fill the chip, `split` work-groups
// share a key block, each sweeping Hkv / split kv heads.  Pass 1 is unaffected
// (its statistics are per head); pass 2 then leaves partial column sums in the
// workspace and k_finish adds them, forms the scores and selects.
//
// With split == 1 a pass-2 work-group ends with the final scores of its
// consecutive tokens: it owns whole selection blocks (G divides 256) and goes
// straight on to their block-local top-k.  The gather of the kept rows is a
// launch of its own.
//
// Tokens that follow earlier context (chunked prefill): the keys of a sequence are then its
// earlier tokens' keys followed by its own (`cu_k` differs from `cu`), window row j sits at
// key position P + j (P earlier tokens), pass 1 runs over all keys, pass 2 only over key blocks
// that hold keys of the tokens -- with a launch geometry of its own, since these are far fewer --
// and k_finish picks each token's column sum at key P + i.
//
// Logits are handled in log2 units: x = s_raw * c + negref, c = scale*log2(e),
// so the exponential is a bare v_exp_f32.
#include <type_traits>

#include "up_common.h"
#include "up_copy.h"
#include "up_kernels.h"
#include "up_select.h"

namespace up {

constexpr int kUnit = 128;           // query rows per LDS staging unit (4 MFMA row tiles)
// bytes of one head row (D elements) in global memory, and in LDS with a 16-byte pad that makes
// the 128-bit operand reads conflict-free
template <bool F32, int D> constexpr int kHeadRowBytes = D * (F32 ? 4 : 2);
template <bool F32, int D> constexpr int kQRow = kHeadRowBytes<F32, D> + 16;
// pass 1 leaves one pair of statistics per lane half of every wave when LDS has room for it
// (head rows of up to 256 bytes), which spares the tiles a lane exchange; otherwise one per wave
template <bool F32, int D> constexpr bool kHalfStats = kHeadRowBytes<F32, D> <= 256;

typedef float f32x16 __attribute__((ext_vector_type(16)));

struct SweepArgs {
  const char* q;
  const char* k;
  const int32_t* cu;     // token offsets (queries, scores)
  const int32_t* cu_k;   // key offsets (== cu when no sequence has earlier context)
  const int32_t* block_table;   // paged keys: physical block of every logical KV block, or nullptr
  long long table_stride;       // entries per sequence in block_table
  int kv_block;                 // tokens per KV block
  float2* stat_part;   // [key_block_slots][Hq * n_obs]  (reference in log2 units, sum)
  float2* stat_fin;    // [Hq][row_slots]                 (negative reference, 1/sum)
  float* scores_out;   // pass 2: optional
  double* colsum_out;  // pass 2 through k_finish: optional, the raw column sums (a rank's share, Eq. 15)
  double* o_part;      // pass 2, via_finish: [pass-2 slots][split][keys per block] partial column sums
  long long q_stride_b, k_stride_b;   // bytes between tokens
  float c;             // scale * log2(e)
  int R, T, Hq, Hkv, Gq, n_obs, row_slots;
  int split;           // work-groups per key block in this pass; each sweeps Hkv / split kv heads
  int spare2;          // pass 2 numbers its key blocks by the tokens: slots per sequence beyond N / KB
  int via_finish;      // pass 2 ends with the partial column sums; k_finish forms scores and selects
  int do_select;       // pass 2: run the block-local top-k
  int skip_forced;     // sequences kept whole whatever their scores (N <= sinks + window; never set with earlier
                       // context) are not scored: the caller selects and wants no scores
  int n_sink;
  SelectArgs sel;
  GatherArgs gather;   // the kernel that selects also copies its kept rows (hidden == nullptr: no)
};

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ __forceinline__ float exp2_hw(float x) { return __builtin_amdgcn_exp2f(x); }

// value of another lane through the data-parallel-primitive path (no LDS traffic);
// CTRL: 0xB1 = lane^1, 0x4E = lane^2 (inside quads), 0x141 = mirror inside groups of 8
template <int CTRL>
__device__ __forceinline__ float dpp(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

// x -> (x / d, x % d) with a precomputed magic = 0xFFFFFFFF / d  (x < 2^31).
__device__ __forceinline__ void divmod(unsigned x, unsigned d, unsigned magic, int& qo, int& ro) {
  unsigned qq = __umulhi(x, magic);
  unsigned rr = x - qq * d;
  if (rr >= d) { ++qq; rr -= d; }
  qo = (int)qq;
  ro = (int)rr;
}

// LDS of one work-group of NW waves.  The staged query rows are dead once the sweep is over,
// so the selection state reuses their space.  The per-unit tables are double-buffered like
// the rows: the tables of unit f+1 are written while unit f is being read.
template <int NW, bool F32, int D>
struct SweepSmem {
  union {
    __align__(16) unsigned char q[2][kUnit * kQRow<F32, D>];   // staged query rows, double-buffered
    struct {
      double o64[32 * NW];                             // pass 2: column sums of the block's keys
      SelectSmem sel;
    } tail;
  };
  union {
    // pass 1: (reference, sum) per staged row from every wave, or from each lane half of every wave
    float2 wstat[2][NW * (kHalfStats<F32, D> ? 2 : 1)][kUnit];
    __align__(16) float2 cst[2][kUnit];                // pass 2: (negative reference, 1/sum) per staged row
  };
  __align__(16) int rowpos[2][kUnit];                  // local position of each staged row, -1 = no such row
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

template <int PASS, bool EDGE, int NW, bool F32, int D>
__device__ __forceinline__ void sweep_block(const SweepArgs& a, SweepSmem<NW, F32, D>& sm, int r, int c0, int N,
                                            int ck0, int Lk, int kblock, int slot, int g0, int n_heads) {
  constexpr int KB = 32 * NW;                               // keys per work-group
  constexpr int THREADS = 64 * NW;
  constexpr int SRCB = kHeadRowBytes<F32, D>;               // bytes of a head row in global memory
  constexpr int ROWB = kQRow<F32, D>;                       // ... and in LDS
  constexpr bool HS = kHalfStats<F32, D>;
  constexpr int PPR = SRCB / 16;                            // 16-byte pieces per row
  constexpr int PIECES = kUnit * PPR / THREADS;             // pieces of a unit per thread
  constexpr int ROWSTEP = THREADS / PPR;                    // rows between a thread's pieces
  static_assert(THREADS % PPR == 0 && (kUnit * PPR) % THREADS == 0 && PIECES >= 1, "staging split");
  static_assert(sizeof(SweepSmem<NW, F32, D>) <= 160 * 1024, "LDS of one CU");
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int l32 = lane & 31, half = lane >> 5;
  // N tokens (queries) at packed rows c0.., Lk >= N keys at packed key rows ck0..; the tokens are
  // the last N positions of the Lk
  const int n_eff = imin(a.n_obs, N);
  const int first_q = N - n_eff;                   // first window row among the tokens
  const int first_pos = Lk - n_eff;                // ... and its position among the keys
  const int rows_total = n_eff * a.Gq;
  const int n_units = (rows_total + kUnit - 1) / kUnit;
  const int n_flat = n_heads * n_units;            // this work-group sweeps kv heads g0 .. g0 + n_heads - 1
  const unsigned magic = 0xFFFFFFFFu / (unsigned)n_eff;
  const int key_base = kblock * KB + wave * 32;            // first local key of this wave
  const float c = a.c;
  const int rs0 = rowslot_base(c0, r, a.n_obs);
  const bool whole_heads = (n_eff % kUnit) == 0;           // a unit never straddles two query heads

  // ---- key operands of one kv head: 32 keys, lane = (key l32, half of the contraction).
  // bf16: MFMA step kk contracts elements 16*kk .. 16*kk+15, lane half h supplies 8*h .. 8*h+7 of
  // them (one 128-bit register group per step).  fp32 (v_mfma_f32_32x32x2_f32, two elements per
  // step): step t contracts elements t and D/2+t, so that a lane half owns D/2 consecutive
  // elements and loads them with 128-bit accesses; queries use the same order.
  // Keys past the end of the sequence re-read the last key (finite values): pass 1 masks
  // them (such a block is always an edge block), pass 2 never emits their scores.
  constexpr int KREG = SRCB / 32;                 // 128-bit register groups of a lane's half row
  constexpr int HOFF = F32 ? SRCB / 2 : 16;       // byte offset of the second lane half
  constexpr int KSTEP = F32 ? 16 : 32;            // bytes between a lane's register groups
  u32x4 kf[KREG];
  // (paged keys: key i of the sequence lives in row block_table[r][i / B] * B + i % B of the cache)
  const int k_idx = imin(key_base + l32, Lk - 1);
  const long long k_row = a.block_table == nullptr
                              ? (long long)ck0 + k_idx
                              : (long long)a.block_table[(long long)r * a.table_stride + k_idx / a.kv_block] * a.kv_block +
                                    k_idx % a.kv_block;
  const char* k_lane = a.k + k_row * a.k_stride_b + half * HOFF;
  auto load_keys = [&](int g) {
#pragma unroll
    for (int kk = 0; kk < KREG; ++kk)
      kf[kk] = *(const u32x4*)(k_lane + (long long)g * SRCB + kk * KSTEP);
  };

  // ---- staging of one unit of query rows: 128 rows x PPR pieces of 16 bytes, PIECES per thread:
  // piece t%PPR of rows t/PPR + ROWSTEP*i.  Fetched into registers at the start of the
  // previous unit's matrix work, written to LDS just before the barrier that ends it.
  const int my_row = tid / PPR, my_col = tid % PPR;
  const char* q_seq = a.q + (long long)(c0 + first_q) * a.q_stride_b + my_col * 16;
  const long long my_row_off = (long long)my_row * a.q_stride_b;
  u32x4 pre_q[PIECES];
  auto fetch_unit = [&](const UnitCursor& uc) {
    if (whole_heads) {
      const char* base = q_seq + (long long)(uc.g * a.Gq + uc.hh) * SRCB + (long long)uc.jj0 * a.q_stride_b + my_row_off;
#pragma unroll
      for (int i = 0; i < PIECES; ++i) pre_q[i] = *(const u32x4*)(base + (long long)(i * ROWSTEP) * a.q_stride_b);
    } else {
      // general case: one division per piece; rows past the end re-read the last row
      // (finite values; their results are discarded through the per-row constants)
#pragma unroll
      for (int i = 0; i < PIECES; ++i) {
        const int rho = imin(uc.u * kUnit + my_row + i * ROWSTEP, rows_total - 1);
        int hh, jj;
        divmod((unsigned)rho, (unsigned)n_eff, magic, hh, jj);
        pre_q[i] = *(const u32x4*)(q_seq + (long long)jj * a.q_stride_b + (long long)(uc.g * a.Gq + hh) * SRCB);
      }
    }
  };
  auto stash_unit = [&](int buf) {
#pragma unroll
    for (int i = 0; i < PIECES; ++i)
      *(u32x4*)(&sm.q[buf][(my_row + i * ROWSTEP) * ROWB + my_col * 16]) = pre_q[i];
  };
  // row of a unit -> (query head inside the group, window row), or false if there is no such row
  auto unit_row = [&](const UnitCursor& uc, int row, int& hh, int& jj) -> bool {
    const int rho = uc.u * kUnit + row;
    if (whole_heads) { hh = uc.hh; jj = uc.jj0 + row; return true; }
    if (rho >= rows_total) { hh = 0; jj = 0; return false; }
    divmod((unsigned)rho, (unsigned)n_eff, magic, hh, jj);
    return true;
  };
  // per-row tables of a unit: threads 0..127 take one row each; fetched with the rows, written with them
  float2 pre_cst = make_float2(-INFINITY, 0.0f);
  int pre_pos = -1;
  // (every thread issues the load -- threads 128.. repeat rows 0..127, a unit's missing rows read
  // row 0 -- and nothing looks at the value before stash_meta: the load's latency stays behind
  // the unit's matrix work, and the number of loads in flight is the same on every path, so the
  // wait for the key operands, which are older, does not have to cover them)
  auto fetch_meta = [&](const UnitCursor& uc) {
    int hh, jj;
    const bool have = unit_row(uc, tid & (kUnit - 1), hh, jj);
    pre_pos = have ? first_pos + jj : -1;
    if (PASS == 2) pre_cst = a.stat_fin[(size_t)(uc.g * a.Gq + hh) * a.row_slots + rs0 + jj];
  };
  auto stash_meta = [&](int tb) {
    if (tid < kUnit) {
      // no such row: weight exactly zero
      if (PASS == 2) sm.cst[tb][tid] = pre_pos >= 0 ? pre_cst : make_float2(-INFINITY, 0.0f);
      sm.rowpos[tb][tid] = pre_pos;
    }
  };

  double col64 = 0.0;   // pass 2: running column sum of this lane's key

  // ---- one tile = 32 staged rows (row tile rt of buffer buf, tables tb) against the wave's 32 keys;
  // MASK: some (row, key) pairs of the tile are not visible (key after the row, or past the end)
  // (reload: this is the kv head's last tile; once its MFMAs are issued the key registers are free
  // and the next head's keys are fetched under this tile's vector work)
  auto tile = [&](auto mask_tag, int buf, int tb, int rt, bool reload, int next_g) {
    constexpr bool MASK = decltype(mask_tag)::value;
    u32x4 qv[KREG];
#pragma unroll
    for (int kk = 0; kk < KREG; ++kk)
      qv[kk] = *(const u32x4*)(&sm.q[buf][(rt * 32 + l32) * ROWB + half * HOFF + kk * KSTEP]);
    f32x16 acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.0f;
    // pass 1 computes S^T (rows of the result are keys, columns are query rows), pass 2 S
    if (F32) {
      auto step = [&](unsigned kbits, unsigned qbits) {
        const float kx = __builtin_bit_cast(float, kbits), qx = __builtin_bit_cast(float, qbits);
        acc = PASS == 1 ? __builtin_amdgcn_mfma_f32_32x32x2f32(kx, qx, acc, 0, 0, 0)
                        : __builtin_amdgcn_mfma_f32_32x32x2f32(qx, kx, acc, 0, 0, 0);
      };
#pragma unroll
      for (int kk = 0; kk < KREG; ++kk) {
        const u32x4 k4 = kf[kk], q4 = qv[kk];
        step(k4.x, q4.x);
        step(k4.y, q4.y);
        step(k4.z, q4.z);
        step(k4.w, q4.w);
      }
    } else {
#pragma unroll
      for (int kk = 0; kk < KREG; ++kk)
        acc = PASS == 1 ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(kf[kk]), as_bf16x8(qv[kk]), acc, 0, 0, 0)
                        : __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(qv[kk]), as_bf16x8(kf[kk]), acc, 0, 0, 0);
    }
    if (reload) load_keys(next_g);
    if (PASS == 1) {
      // element e = key 8*(e/4) + 4*half + e%4 of the wave's keys, query row rt*32 + l32
      if (MASK) {
        const int rp = sm.rowpos[tb][rt * 32 + l32];
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (key_base + 8 * (e >> 2) + 4 * half + (e & 3) > rp) acc[e] = -INFINITY;
      }
      float m0 = fmaxf(fmaxf(acc[0], acc[1]), fmaxf(acc[2], acc[3]));
      float m1 = fmaxf(fmaxf(acc[4], acc[5]), fmaxf(acc[6], acc[7]));
      m0 = fmaxf(m0, fmaxf(fmaxf(acc[8], acc[9]), fmaxf(acc[10], acc[11])));
      m1 = fmaxf(m1, fmaxf(fmaxf(acc[12], acc[13]), fmaxf(acc[14], acc[15])));
      const float m = fmaxf(m0, m1);
      const float ref = m * c;                          // reference in log2 units
      const float negref = (MASK && m == -INFINITY) ? 0.0f : -ref;
      float l0 = 0.0f, l1 = 0.0f;
#pragma unroll
      for (int e = 0; e < 16; e += 2) {
        l0 += exp2_hw(fmaf(acc[e], c, negref));
        l1 += exp2_hw(fmaf(acc[e + 1], c, negref));
      }
      l0 += l1;                                         // 0 when every key was masked (exp2(-inf))
      if (HS) {
        // each lane half leaves its own pair (the same row over its 16 keys); the unit merge adds them
        sm.wstat[tb][2 * wave + half][rt * 32 + l32] = make_float2(ref, l0);
      } else {
        // the other lane half holds the same row over the other 16 keys
        const float ref_o = __shfl_xor(ref, 32);
        const float l_o = __shfl_xor(l0, 32);
        const float mm = fmaxf(ref, ref_o);
        float s_a = l0 * exp2_hw(ref - mm);
        float s_b = l_o * exp2_hw(ref_o - mm);
        if (MASK) {
          if (ref == -INFINITY) s_a = 0.0f;
          if (ref_o == -INFINITY) s_b = 0.0f;
        }
        if (half == 0) sm.wstat[tb][wave][rt * 32 + l32] = make_float2(mm, s_a + s_b);
      }
    } else {
      // element e = query row rt*32 + 8*(e/4) + 4*half + e%4, key l32
      float cs0 = 0.0f, cs1 = 0.0f;
#pragma unroll
      for (int e = 0; e < 16; e += 2) {
        const int row0 = rt * 32 + 8 * (e >> 2) + 4 * half + (e & 3);
        const f32x4 cs = *(const f32x4*)(&sm.cst[tb][row0]);   // (negref, w) of rows row0, row0+1
        float x0 = fmaf(acc[e], c, cs[0]);
        float x1 = fmaf(acc[e + 1], c, cs[2]);
        if (MASK) {
          if (key_base + l32 > sm.rowpos[tb][row0]) x0 = -INFINITY;
          if (key_base + l32 > sm.rowpos[tb][row0 + 1]) x1 = -INFINITY;
        }
        cs0 = fmaf(exp2_hw(x0), cs[1], cs0);
        cs1 = fmaf(exp2_hw(x1), cs[3], cs1);
      }
      col64 += (double)(cs0 + cs1);
    }
  };

  // pass 1: merge the statistics of the 128 rows of unit `uc` (tables tb) and write the key
  // block's partial.  Every wave takes 128/NW rows; the partials of a row (one per wave, or one per
  // lane half of every wave) sit PPL per lane on neighbouring lanes and are reduced with lane
  // permutes in a fixed order.  The two halves (LDS reads; arithmetic and store) are issued a tile
  // apart inside the next unit's matrix work, where their latency disappears.
  constexpr int RPW = kUnit / NW;                 // rows per wave: 8 or 16
  constexpr int LPR = 64 / RPW;                   // lanes per row: 8 or 4
  constexpr int PPL = (HS ? 2 * NW : NW) / LPR;   // partials per lane: 2 or 4
  float2 mp[PPL];
#pragma unroll
  for (int i = 0; i < PPL; ++i) mp[i] = make_float2(0.0f, 0.0f);
  auto merge_load = [&](int tb) {
    const int row = wave * RPW + lane / LPR;
    const int sub = lane % LPR;
#pragma unroll
    for (int i = 0; i < PPL; ++i) mp[i] = sm.wstat[tb][sub + LPR * i][row];
  };
  auto merge_finish = [&](const UnitCursor& uc) {
    const int row = wave * RPW + lane / LPR;
    const int sub = lane % LPR;
    float mm = mp[0].x;
#pragma unroll
    for (int i = 1; i < PPL; ++i) mm = fmaxf(mm, mp[i].x);
    mm = fmaxf(mm, dpp<0xB1>(mm));
    mm = fmaxf(mm, dpp<0x4E>(mm));
    if (LPR == 8) mm = fmaxf(mm, dpp<0x141>(mm));
    float l = 0.0f;
#pragma unroll
    for (int i = 0; i < PPL; ++i) l += mp[i].x == -INFINITY ? 0.0f : mp[i].y * exp2_hw(mp[i].x - mm);
    l += dpp<0xB1>(l);
    l += dpp<0x4E>(l);
    if (LPR == 8) l += dpp<0x141>(l);
    int hh, jj;
    if (sub == 0 && unit_row(uc, row, hh, jj))
      a.stat_part[(size_t)slot * (a.Hq * a.n_obs) + (size_t)(uc.g * a.Gq + hh) * a.n_obs + jj] = make_float2(mm, l);
  };

  // ---- prologue: unit 0 staged and visible
  UnitCursor cur{g0, 0, 0, 0};     // unit being processed
  UnitCursor nxt = cur;            // unit being staged
  UnitCursor prev = cur;           // unit whose statistics are still to be merged (pass 1)
  fetch_unit(cur);
  fetch_meta(cur);
  load_keys(g0);
  stash_unit(0);
  stash_meta(0);
  __syncthreads();
  if (n_flat > 1) nxt.advance(n_units, n_eff);

  for (int f = 0; f < n_flat; ++f) {
    const int buf = f & 1;
    const bool more = f + 1 < n_flat;
    const bool head_ends = more && cur.u == n_units - 1;   // the next unit belongs to the next kv head
    // rows and tables of the next unit: in flight during this unit's matrix work (after the
    // last unit the cursor stays where it is and the loads repeat: the same loads on every path)
    fetch_unit(nxt);
    fetch_meta(nxt);
#pragma unroll
    for (int rt = 0; rt < 4; ++rt) {
      // pass 1: the previous unit's statistics are merged in passing (its table slot is free
      // for unit f+1 only after the barrier below, which every wave reaches after its merge)
      if (PASS == 1 && f > 0 && rt == 1) merge_load(buf ^ 1);
      if (PASS == 1 && f > 0 && rt == 2) merge_finish(prev);
      const bool reload = head_ends && rt == 3;
      if (!EDGE) {
        tile(std::false_type{}, buf, buf, rt, reload, cur.g + 1);
      } else {
        // the wave's 32 keys against the tile's rows: all visible, none visible, or mixed.  When a
        // unit holds consecutive window rows of one head the row positions of a tile are a known
        // range; otherwise any tile of a wave whose keys reach the window is treated as mixed.
        bool none = false, mixed;
        if (whole_heads) {
          const int r_lo = first_pos + cur.jj0 + 32 * rt;
          none = key_base > r_lo + 31;
          mixed = key_base + 31 > r_lo;
        } else {
          mixed = key_base + 31 > first_pos;
        }
        if (none) {
          if (PASS == 1) {
            if (HS) sm.wstat[buf][2 * wave + half][rt * 32 + l32] = make_float2(-INFINITY, 0.0f);
            else if (half == 0) sm.wstat[buf][wave][rt * 32 + l32] = make_float2(-INFINITY, 0.0f);
          }
          if (reload) load_keys(cur.g + 1);
        } else if (mixed) {
          tile(std::true_type{}, buf, buf, rt, reload, cur.g + 1);
        } else {
          tile(std::false_type{}, buf, buf, rt, reload, cur.g + 1);
        }
      }
      // tiles stay apart: neither the compiler nor the scheduler may pull the next tile's table
      // reads across (they would all be live at once)
      asm volatile("" : "+v"(col64) : : "memory");
      __builtin_amdgcn_sched_barrier(0);
    }
    if (more) { stash_unit(buf ^ 1); stash_meta(buf ^ 1); }
    __syncthreads();     // unit f+1 is visible; every read of unit f's rows and tables has completed
    prev = cur;
    cur = nxt;
    if (f + 2 < n_flat) nxt.advance(n_units, n_eff);
  }

  if (PASS == 1) {   // statistics of the last unit (its barrier has passed)
    merge_load((n_flat - 1) & 1);
    merge_finish(prev);
  }
  if (PASS == 2) {
    // (a barrier has passed since the last read of the staged rows: their space is reused)
    // the two lane halves hold the same keys over different rows: add them (fixed order)
    const double other = __shfl_xor(col64, 32);
    if (half == 0) sm.tail.o64[wave * 32 + l32] = col64 + other;
  }
}

template <int PASS, int NW, bool F32, int D>
__global__ __launch_bounds__(64 * NW) void k_sweep(SweepArgs a) {
  constexpr int KB = 32 * NW;
  __shared__ SweepSmem<NW, F32, D> sm;
  const int slot = blockIdx.x / a.split, part = blockIdx.x % a.split;
  // pass 1 numbers the key blocks of all keys; pass 2 only those that hold keys of the tokens
  // (column sums are not wanted for the earlier context), starting with the block of the first one
  const int r = PASS == 1 ? locate_slot(a.cu_k, a.R, KB, slot) : locate_slot(a.cu, a.R, KB, slot, a.spare2);
  const int ck0 = a.cu_k[r];
  const int Lk = a.cu_k[r + 1] - ck0;
  const int c0 = a.cu[r];
  const int N = a.cu[r + 1] - c0;
  const int kblock = PASS == 1 ? slot - slot_base(ck0, r, KB)
                               : (Lk - N) / KB + slot - slot_base(c0, r, KB, a.spare2);
  if (kblock * KB >= Lk || N == 0) return;
  const int n_eff = imin(a.n_obs, N);
  // a sequence of which every token is a sink or in the window (a decode row, a short request) is
  // kept whole whatever its scores: when only the selection is wanted it is not scored at all
  const bool unscored = a.skip_forced && N <= a.n_sink + a.n_obs;
  if (unscored && (PASS == 1 || a.via_finish)) return;
  // causal masking and the ragged end only matter where keys reach the query window
  const bool edge = (kblock + 1) * KB - 1 > Lk - n_eff;
  const int n_heads = a.Hkv / a.split;
  if (!unscored) {
    if (edge) sweep_block<PASS, true, NW, F32, D>(a, sm, r, c0, N, ck0, Lk, kblock, slot, part * n_heads, n_heads);
    else sweep_block<PASS, false, NW, F32, D>(a, sm, r, c0, N, ck0, Lk, kblock, slot, part * n_heads, n_heads);
  }

  if (PASS == 2) {
    __syncthreads();
    const int tid = threadIdx.x;
    if (a.via_finish) {
      // the key block's heads are shared by `split` work-groups, or its keys are not aligned with
      // the tokens' selection blocks: each work-group leaves its partial sums in the workspace and
      // k_finish adds them up (in a fixed order) after this kernel has ended
      if (tid < KB) a.o_part[((size_t)slot * a.split + part) * KB + tid] = sm.tail.o64[tid];
      return;
    }
    float sc = 0.0f;
    if (tid < KB) {
      const int key = kblock * KB + tid;
      if (key < N && !unscored) {
        const double o = sm.tail.o64[tid] / (double)(n_eff * a.Hq);
        sc = o < 0x1p-64 ? 0.0f : (float)o;
        if (a.scores_out != nullptr) a.scores_out[c0 + key] = sc;
      }
      if (a.do_select) sm.tail.sel.score[tid] = sc;
    }
    if (!a.do_select) return;
    __syncthreads();
    // the block-local top-k, one selection block after the other
    const int G = a.sel.G;
    const int g_first = kblock * (KB / G);
    const int nb = imin(KB / G, ceil_div(N - kblock * KB, G));
    const bool gather = a.gather.hidden != nullptr;
    int list_base = -1, list_n = 0;
    if (gather) {      // where the key block's kept rows start in the output, and how many there are
      SeqGeom sg{N, G, a.sel.n_obs, sinks_of(a.sel.cu_k, a.sel.n_sink, r, N), (double)a.sel.ratio[r]};
      const int before = kept_before(sg, g_first);
      list_base = a.sel.new_cu[r] + before;
      list_n = kept_before(sg, g_first + nb) - before;
    }
    for (int b = 0; b < nb; ++b)
      select_block(a.sel, sm.tail.sel, r, c0, N, g_first + b, &sm.tail.sel.score[b * G], list_base);
    if (!gather) return;
    // the key block's kept rows (Eq. 7), dealt to the waves (select_block ends with a barrier)
    const int wave = tid >> 6, lane = tid & 63;
    for (int i = wave; i < list_n; i += NW) {
      const long long row = sm.tail.sel.kept_rows[i];
      copy_row_wave(a.gather.hidden + row * a.gather.stride_bytes,
                    a.gather.hidden_out + (long long)(list_base + i) * a.gather.stride_bytes, a.gather.row_bytes, lane);
      if (a.gather.pos != nullptr && lane == 0) a.gather.pos_out[list_base + i] = a.gather.pos[row];
    }
  }
}

// When the kv heads of a key block were shared by several work-groups (split > 1), or the
// tokens follow earlier context: one work-group per selection block adds the parts' column
// sums in a fixed order, forms the scores (mean, floor) and runs the block-local top-k.
__global__ __launch_bounds__(256) void k_finish(SweepArgs a, int key_block) {   // (pass 2's key block)
  __shared__ SelectSmem sm;
  const int G = a.sel.G;
  const int slot = blockIdx.x;
  const int r = locate_slot(a.cu, a.R, G, slot);
  const int c0 = a.cu[r];
  const int N = a.cu[r + 1] - c0;
  const int g = slot - slot_base(c0, r, G);
  if (g * G >= N) return;   // slack slot (also every slot of an empty sequence)
  const int tid = threadIdx.x;
  const int tok = g * G + tid;
  if (tid < G) {
    float sc = 0.0f;
    if (tok < N && !(a.skip_forced && N <= a.n_sink + a.n_obs)) {      // (an unscored sequence left no sums)
      const int ck0 = a.cu_k[r];
      const int earlier = (a.cu_k[r + 1] - ck0) - N;
      const int key = earlier + tok;                       // the token's place among the sequence's keys
      const int kblock = key / key_block;
      const int slot2 = slot_base(c0, r, key_block, a.spare2) + kblock - earlier / key_block;
      const double* part0 = a.o_part + (size_t)slot2 * a.split * key_block + (key - kblock * key_block);
      double sum = 0.0;
      for (int pp = 0; pp < a.split; ++pp) sum += part0[(size_t)pp * key_block];
      if (a.colsum_out != nullptr) a.colsum_out[c0 + tok] = sum;
      const double o = sum / (double)(imin(a.n_obs, N) * a.Hq);
      sc = o < 0x1p-64 ? 0.0f : (float)o;
      if (a.scores_out != nullptr) a.scores_out[c0 + tok] = sc;
    }
    sm.score[tid] = sc;
  }
  if (!a.do_select) return;
  __syncthreads();
  const bool gather = a.gather.hidden != nullptr;
  int list_base = -1, list_n = 0;
  if (gather) {      // where the block's kept rows go in the output, and how many there are
    SeqGeom sg{N, G, a.sel.n_obs, sinks_of(a.sel.cu_k, a.sel.n_sink, r, N), (double)a.sel.ratio[r]};
    list_base = a.sel.new_cu[r] + kept_before(sg, g);
    list_n = block_kept(sg, g);
  }
  select_block(a.sel, sm, r, c0, N, g, sm.score, list_base);
  if (!gather) return;
  const int wave = tid >> 6, lane = tid & 63;      // four waves (select_block ends with a barrier)
  for (int i = wave; i < list_n; i += 4) {
    const long long row = sm.kept_rows[i];
    copy_row_wave(a.gather.hidden + row * a.gather.stride_bytes,
                  a.gather.hidden_out + (long long)(list_base + i) * a.gather.stride_bytes, a.gather.row_bytes, lane);
    if (a.gather.pos != nullptr && lane == 0) a.gather.pos_out[list_base + i] = a.gather.pos[row];
  }
}

// Merge the per-key-block softmax statistics of every (sequence, window row, head):
// final reference = max of the block references, sum rescaled to it.  A work-group
// handles 32 consecutive window rows of one head (coalesced along the rows); the LPR
// threads that share a row each take 16 key blocks per round, all loads in flight
// (LPR = 32 for long sequences, 8 when no sequence has more than 128 key blocks).
// Row slots are laid out with slack between sequences; a work-group without a live row
// ends at once.  In the fused call the first work-group also does the plan (kept totals per
// sequence and their prefix), which nothing needs before the kernel after this one: one launch
// and its gap less than with k_plan.
struct PlanInCombine {
  const float* ratio;      // nullptr: no plan here
  int32_t* new_cu;
  const int32_t* cu_k_sel; // key-side offsets for the sinks (nullptr without earlier context)
  int G, n_sink;
};
template <int LPR>
__global__ __launch_bounds__(32 * LPR) void k_combine(const int32_t* __restrict__ cu,
                                                      const int32_t* __restrict__ cu_k,
                                                      const float2* __restrict__ stat_part,
                                                      float2* __restrict__ stat_fin, int R, int Hq,
                                                      int n_obs, int row_slots, int key_block,
                                                      int heads_per_group, PlanInCombine plan) {
  __shared__ float sh_m[LPR][33];
  __shared__ double sh_l[LPR][33];
  if (plan.ratio != nullptr && blockIdx.x == 0 && blockIdx.y == 0) {
    __shared__ int wave_tot[16];
    __shared__ int carry;
    plan_scan<32 * LPR>(cu, plan.cu_k_sel, plan.ratio, R, plan.G, n_obs, plan.n_sink, plan.new_cu, wave_tot, &carry);
  }
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const int u = blockIdx.x * 32 + tx;
  bool live = u < row_slots;
  int n_blocks = 0;
  const float2* p_row = stat_part;
  const size_t stride = (size_t)Hq * n_obs;
  if (live) {
    const int r = locate_rowslot(cu, R, n_obs, u);
    const int c0 = cu[r];
    const int N = cu[r + 1] - c0;
    const int jj = u - rowslot_base(c0, r, n_obs);
    live = jj < imin(n_obs, N);
    if (live) {
      const int ck0 = cu_k[r];
      n_blocks = ceil_div(cu_k[r + 1] - ck0, key_block);
      p_row = stat_part + (size_t)slot_base(ck0, r, key_block) * stride + jj;
    }
  }
  if (__syncthreads_or(live) == 0) return;
  // the work-group's heads one after the other: the look-up of the row's sequence above (a chain of
  // dependent loads) is paid once for all of them
  for (int h = blockIdx.y * heads_per_group; h < (blockIdx.y + 1) * heads_per_group; ++h) {
    const float2* p = p_row + (size_t)h * n_obs;
    float m = -INFINITY;
    double L = 0.0;
    for (int b0 = ty * 16; b0 < n_blocks; b0 += 16 * LPR) {
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
      for (int i = 0; i < LPR; ++i) mm = fmaxf(mm, sh_m[i][tx]);
      double tot = 0.0;
      for (int i = 0; i < LPR; ++i)
        if (sh_m[i][tx] != -INFINITY) tot += sh_l[i][tx] * exp2((double)sh_m[i][tx] - (double)mm);
      stat_fin[(size_t)h * row_slots + u] = make_float2(-mm, (float)(1.0 / tot));
    }
    __syncthreads();      // the shared arrays are reused by the next head
  }
}

// Row normalisers handed in (the natural log of the row's sum of exponentials, as an attention
// kernel returns it) instead of pass 1 and the merge: the pair pass 2 reads is (-hi, 2^(hi - L))
// with L = lse * log2(e) in double and hi = L rounded to float, so that the weight
// 2^(x - hi) * 2^(hi - L) is exact to float rounding.  One thread per (window row, head); the
// first work-group also does the plan when asked, as in k_combine.
__global__ __launch_bounds__(256) void k_lse_stats(const int32_t* __restrict__ cu, const float* __restrict__ lse,
                                                   long long lse_stride, float2* __restrict__ stat_fin, int R,
                                                   int Hq, int n_obs, int row_slots, PlanInCombine plan) {
  if (plan.ratio != nullptr && blockIdx.x == 0 && blockIdx.y == 0) {
    __shared__ int wave_tot[16];
    __shared__ int carry;
    plan_scan<256>(cu, plan.cu_k_sel, plan.ratio, R, plan.G, n_obs, plan.n_sink, plan.new_cu, wave_tot, &carry);
  }
  const int u = blockIdx.x * 256 + threadIdx.x;
  const int h = blockIdx.y;
  if (u >= row_slots || h >= Hq) return;
  const int r = locate_rowslot(cu, R, n_obs, u);
  const int c0 = cu[r];
  const int N = cu[r + 1] - c0;
  const int n_eff = imin(n_obs, N);
  const int jj = u - rowslot_base(c0, r, n_obs);
  if (jj >= n_eff) return;
  const double L = (double)lse[(long long)h * lse_stride + c0 + (N - n_eff) + jj] * 1.4426950408889634074;
  const float hi = (float)L;
  stat_fin[(size_t)h * row_slots + u] = make_float2(-hi, (float)exp2((double)hi - L));
}

hipError_t launch_lse_stats(const Problem& pb, const int32_t* cu, const int32_t* cu_k, const float* lse,
                            long long lse_stride, void* workspace, const float* plan_ratio, int32_t* plan_new_cu,
                            hipStream_t s) {
  if (pb.T == 0)
    return plan_ratio != nullptr ? launch_plan(pb, cu, cu_k, plan_ratio, plan_new_cu, s) : hipSuccess;
  const Workspace w = workspace_layout(pb);
  const PlanInCombine plan{plan_ratio, plan_new_cu, cu_k, pb.G, pb.n_sink};
  hipLaunchKernelGGL(k_lse_stats, dim3((unsigned)((pb.row_slots + 255) / 256), (unsigned)pb.Hq), dim3(256), 0, s, cu,
                     lse, lse_stride, (float2*)((char*)workspace + w.stat_fin_off), pb.R, pb.Hq, pb.n_obs,
                     pb.row_slots, plan);
  return hipGetLastError();
}

// Scores from the ranks' partial column sums (Eq. 15, then the means of Eq. 3 and the floor):
// the parts are added in rank order, so every rank that runs this gets the same bits.
__global__ __launch_bounds__(256) void k_scores_from_partials(const double* __restrict__ partials, int num_parts,
                                                              long long part_stride, const int32_t* __restrict__ cu,
                                                              int R, int T, int n_obs, int total_q_heads,
                                                              float* __restrict__ scores) {
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t >= T) return;
  const int r = locate_token(cu, R, t);
  const int N = cu[r + 1] - cu[r];
  double sum = 0.0;
  for (int pp = 0; pp < num_parts; ++pp) sum += partials[(long long)pp * part_stride + t];
  const double o = sum / (double)((long long)imin(n_obs, N) * total_q_heads);
  scores[t] = o < 0x1p-64 ? 0.0f : (float)o;
}

hipError_t launch_scores_from_partials(const double* partials, int num_parts, long long part_stride,
                                       const int32_t* cu, int R, int T, int n_obs, int total_q_heads,
                                       float* scores, hipStream_t s) {
  if (T == 0) return hipSuccess;
  hipLaunchKernelGGL(k_scores_from_partials, dim3((unsigned)((T + 255) / 256)), dim3(256), 0, s, partials, num_parts,
                     part_stride, cu, R, T, n_obs, total_q_heads, scores);
  return hipGetLastError();
}

static SweepArgs make_sweep_args(const Problem& pb, const void* q, const void* k, const int32_t* cu,
                                 const int32_t* cu_k, void* workspace, const PagedKeys* paged = nullptr) {
  const Workspace w = workspace_layout(pb);
  char* ws = (char*)workspace;
  SweepArgs a{};
  a.q = (const char*)q; a.k = (const char*)k; a.cu = cu; a.cu_k = cu_k != nullptr ? cu_k : cu;
  if (paged != nullptr) { a.block_table = paged->block_table; a.table_stride = paged->table_stride; a.kv_block = paged->kv_block; }
  a.stat_part = (float2*)(ws + w.stat_part_off);
  a.stat_fin = (float2*)(ws + w.stat_fin_off);
  a.scores_out = nullptr;
  a.o_part = (double*)(ws + w.o_part_off);
  a.n_sink = pb.n_sink;
  a.split = pb.split;              // (pass 2 overwrites it)
  a.spare2 = pb.spare2;
  a.via_finish = pb.via_finish;
  const int eb = pb.qk_is_f32 ? 4 : 2;
  a.q_stride_b = pb.q_stride * eb; a.k_stride_b = pb.k_stride * eb;
  a.c = pb.scale * 1.44269504088896340736f;
  a.R = pb.R; a.T = pb.T; a.Hq = pb.Hq; a.Hkv = pb.Hkv; a.Gq = pb.Gq; a.n_obs = pb.n_obs;
  a.row_slots = pb.row_slots;
  a.do_select = 0;
  return a;
}

// One instantiation per (operand type, head dimension, waves per work-group) that is offered:
// 16 waves (512 keys) only where a wave's registers hold its operands within 128 VGPRs, i.e. for
// head rows of up to 256 bytes in bf16.
template <int PASS>
static hipError_t launch_sweep(const Problem& pb, const SweepArgs& a, hipStream_t s) {
  const dim3 grid(PASS == 1 ? (unsigned)(pb.key_block_slots * pb.split) : (unsigned)(pb.key_block_slots2 * pb.split2));
  const bool wide = (PASS == 1 ? pb.key_block : pb.key_block2) == 512;
#define UP_SWEEP(NW_, F32_, D_) hipLaunchKernelGGL((k_sweep<PASS, NW_, F32_, D_>), grid, dim3(64 * NW_), 0, s, a)
  if (pb.qk_is_f32) {
    if (wide) return hipErrorInvalidValue;
    if (pb.head_dim == 64) UP_SWEEP(8, true, 64);
    else if (pb.head_dim == 128) UP_SWEEP(8, true, 128);
    else return hipErrorInvalidValue;
  } else if (pb.head_dim == 64) {
    if (wide) UP_SWEEP(16, false, 64); else UP_SWEEP(8, false, 64);
  } else if (pb.head_dim == 128) {
    if (wide) UP_SWEEP(16, false, 128); else UP_SWEEP(8, false, 128);
  } else if (pb.head_dim == 256) {
    if (wide) return hipErrorInvalidValue;
    UP_SWEEP(8, false, 256);
  } else {
    return hipErrorInvalidValue;
  }
#undef UP_SWEEP
  return hipGetLastError();
}

hipError_t launch_row_stats(const Problem& pb, const void* q, const void* k, const int32_t* cu,
                            const int32_t* cu_k, const PagedKeys* paged, void* workspace, hipStream_t s,
                            bool skip_forced) {
  if (pb.T == 0) return hipSuccess;
  SweepArgs a = make_sweep_args(pb, q, k, cu, cu_k, workspace, paged);
  a.skip_forced = skip_forced && !pb.has_ctx;
  return launch_sweep<1>(pb, a, s);
}

hipError_t launch_merge_stats(const Problem& pb, const int32_t* cu, const int32_t* cu_k, void* workspace,
                              const float* plan_ratio, int32_t* plan_new_cu, hipStream_t s) {
  if (pb.T == 0) {
    // nothing to merge; the plan still has to say so (new_cu = 0 everywhere)
    return plan_ratio != nullptr ? launch_plan(pb, cu, cu_k, plan_ratio, plan_new_cu, s) : hipSuccess;
  }
  const PlanInCombine plan{plan_ratio, plan_new_cu, cu_k, pb.G, pb.n_sink};
  const SweepArgs a = make_sweep_args(pb, nullptr, nullptr, cu, cu_k, workspace);
  // a work-group takes 32 row slots x heads_per_group heads: with many (mostly short) sequences the
  // grid is large and much of a work-group's time is the look-up of its rows' sequence, so up to four
  // heads share one as long as the grid keeps eight work-groups per CU (more heads per work-group
  // were slower: the work-groups with live rows then run their heads one after the other)
  const int row_groups = (pb.row_slots + 31) / 32;
  int hpg = 1;
  while (hpg < 4 && pb.Hq % (2 * hpg) == 0 && (long long)row_groups * (pb.Hq / (2 * hpg)) >= 2048) hpg *= 2;
  const dim3 grid((unsigned)row_groups, (unsigned)(pb.Hq / hpg));
  if (pb.max_key_blocks > 128)
    hipLaunchKernelGGL(k_combine<32>, grid, dim3(1024), 0, s, cu, a.cu_k, a.stat_part, a.stat_fin, pb.R, pb.Hq,
                       pb.n_obs, pb.row_slots, pb.key_block, hpg, plan);
  else
    hipLaunchKernelGGL(k_combine<8>, grid, dim3(256), 0, s, cu, a.cu_k, a.stat_part, a.stat_fin, pb.R, pb.Hq,
                       pb.n_obs, pb.row_slots, pb.key_block, hpg, plan);
  return hipGetLastError();
}

hipError_t launch_column_sums(const Problem& pb, const void* q, const void* k, const int32_t* cu,
                              const int32_t* cu_k, const PagedKeys* paged, void* workspace, float* scores_out,
                              const SelectArgs* sel, hipStream_t s, double* colsum_out, bool skip_forced,
                              const GatherArgs* gather) {
  if (pb.T == 0) return hipSuccess;
  SweepArgs a = make_sweep_args(pb, q, k, cu, cu_k, workspace, paged);
  a.split = pb.split2;
  a.scores_out = scores_out;
  a.colsum_out = colsum_out;
  if (colsum_out != nullptr) a.via_finish = 1;
  a.skip_forced = skip_forced && sel != nullptr && scores_out == nullptr && colsum_out == nullptr && !pb.has_ctx;
  if (gather != nullptr && sel != nullptr) a.gather = *gather;
  if (sel != nullptr) { a.sel = *sel; a.do_select = 1; }
  else { a.sel.G = pb.G; a.sel.cu_k = nullptr; }
  const hipError_t e = launch_sweep<2>(pb, a, s);
  if (e != hipSuccess) return e;
  if (a.via_finish)
    hipLaunchKernelGGL(k_finish, dim3((unsigned)(pb.T / pb.G + pb.R)), dim3(256), 0, s, a, pb.key_block2);
  return hipGetLastError();
}

}  // namespace up
