// C ABI of the UniPrefill operator library: argument validation, closed-form
// planning, and kernel sequencing.  Every check happens on the host before the
// first launch; nothing here allocates, synchronises or copies.
#include "../../include/uniprefill.h"

#include <math.h>

#include <atomic>

#include "up_common.h"
#include "up_kernels.h"
#include "up_select.h"

using namespace up;

// ---- host-only pieces of the launch plumbing (this file holds no device code apart from the
// static scratch array: everything in it also builds with a plain C++ compiler, which is how the
// argument checks and the geometry are run under the address and undefined-behaviour sanitizers)
namespace up {

Workspace workspace_layout(const Problem& pb) {
  auto al = [](size_t x) { return (x + 255) & ~(size_t)255; };
  Workspace w;
  size_t off = 0;
  // block-level top-p selection: flags and offsets per selection block, totals per sequence.
  // First in the buffer: their place depends on T, G and R only, not on the scoring geometry.
  const size_t sel_slots = (size_t)(pb.T / pb.G + pb.R);
  w.tp_keep_off = off;
  off = al(off + sel_slots * sizeof(int32_t));
  w.tp_off_off = off;
  off = al(off + sel_slots * sizeof(int32_t));
  w.tp_seq_off = off;
  off = al(off + (size_t)(pb.R + 1) * sizeof(int32_t));
  w.tp_mass_off = off;
  off = al(off + sel_slots * sizeof(float));
  w.tp_rank_off = off;
  off = al(off + sel_slots * sizeof(int32_t));
  w.tp_sorted_off = off;
  off = al(off + sel_slots * sizeof(float));
  w.tp_total = off;
  w.stat_part_off = off;
  off = al(off + (size_t)pb.key_block_slots * pb.Hq * pb.n_obs * 2 * sizeof(float));
  w.stat_fin_off = off;
  off = al(off + (size_t)pb.row_slots * pb.Hq * 2 * sizeof(float));
  w.o_part_off = off;
  // (always there: a call that wants the raw column sums goes through k_finish whatever the split)
  off = al(off + (size_t)pb.key_block_slots2 * pb.split2 * pb.key_block2 * sizeof(double));
  w.total = off;
  return w;
}

GatherArgs make_gather_args(const Problem& pb, const void* hidden, const int32_t* pos, void* hidden_out,
                            int32_t* pos_out) {
  return GatherArgs{(const char*)hidden, (char*)hidden_out, pos, pos_out, (long long)pb.d * pb.hidden_elem_bytes,
                    pb.h_stride * pb.hidden_elem_bytes};
}

SelectArgs make_select_args(const Problem& pb, const float* scores, const int32_t* cu, const int32_t* cu_k,
                            const float* ratio, const int32_t* new_cu, int32_t* kept_idx) {
  SelectArgs a;
  a.scores = scores; a.cu = cu; a.cu_k = cu_k; a.ratio = ratio; a.new_cu = new_cu; a.kept_idx = kept_idx;
  a.R = pb.R; a.T = pb.T; a.G = pb.G; a.n_obs = pb.n_obs; a.n_sink = pb.n_sink;
  return a;
}

}  // namespace up

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int elem_bytes(int dt) { return dt == UP_BF16 ? 2 : 4; }

// head rows of 512 bytes (fp32 operands, or 256 bf16 elements) only fit the 8-wave work-group
bool narrow_only(const Problem& pb) { return pb.qk_is_f32 || pb.head_dim > 128; }

// Checks that need only the parameter block.
int check_params(const up_params* p, bool need_qk, bool need_hidden, Problem* pb) {
  if (p == nullptr) return UP_ERR_NULL;
  if (p->num_seqs < 0 || p->total_tokens < 0) return UP_ERR_SHAPE;
  if (p->block_size != 32 && p->block_size != 64 && p->block_size != 128) return UP_ERR_RANGE;
  if (p->n_obs < 1 || p->n_obs > kMaxNObs || p->n_sink < 0) return UP_ERR_RANGE;
  Problem q{};
  q.R = p->num_seqs; q.T = p->total_tokens; q.Tk = q.T;
  q.G = p->block_size; q.n_obs = p->n_obs; q.n_sink = p->n_sink;
  q.Hq = p->num_q_heads; q.Hkv = p->num_kv_heads; q.d = p->hidden_dim;
  q.q_stride = p->q_row_stride; q.k_stride = p->k_row_stride; q.h_stride = p->hidden_row_stride;
  q.Gq = 1;
  if (need_qk) {
    if (p->head_dim != 64 && p->head_dim != 128 && p->head_dim != 256) return UP_ERR_UNSUPPORTED;
    if (p->head_dim == 256 && p->qk_dtype == UP_F32) return UP_ERR_UNSUPPORTED;
    if (p->num_q_heads < 1 || p->num_kv_heads < 1) return UP_ERR_SHAPE;
    if (p->num_q_heads % p->num_kv_heads != 0) return UP_ERR_UNSUPPORTED;
    if (p->num_q_heads / p->num_kv_heads > 64) return UP_ERR_UNSUPPORTED;
    if (p->qk_dtype != UP_BF16 && p->qk_dtype != UP_F32) return UP_ERR_UNSUPPORTED;
    if (!(p->softmax_scale >= 0.0f) || isinf(p->softmax_scale)) return UP_ERR_RANGE;
    if (p->q_row_stride < (int64_t)p->num_q_heads * p->head_dim ||
        p->k_row_stride < (int64_t)p->num_kv_heads * p->head_dim)
      return UP_ERR_SHAPE;
    const int eb = elem_bytes(p->qk_dtype);
    if ((p->q_row_stride * eb) % 16 != 0 || (p->k_row_stride * eb) % 16 != 0) return UP_ERR_ALIGN;
    q.Gq = p->num_q_heads / p->num_kv_heads;
    q.qk_is_f32 = p->qk_dtype == UP_F32;
    q.head_dim = p->head_dim;
    q.scale = p->softmax_scale > 0.0f ? p->softmax_scale : 1.0f / sqrtf((float)p->head_dim);
  }
  if (need_hidden) {
    if (p->hidden_dim < 1) return UP_ERR_SHAPE;
    if (p->hidden_dtype != UP_BF16 && p->hidden_dtype != UP_F32) return UP_ERR_UNSUPPORTED;
    if (p->hidden_row_stride < p->hidden_dim) return UP_ERR_SHAPE;
    q.hidden_elem_bytes = elem_bytes(p->hidden_dtype);
    if (((int64_t)p->hidden_dim * q.hidden_elem_bytes) % 16 != 0 ||
        (p->hidden_row_stride * q.hidden_elem_bytes) % 16 != 0)
      return UP_ERR_ALIGN;
  }
  // launch geometry of the scoring sweeps: provisional until choose_geometry has seen the lengths
  q.key_block = narrow_only(q) ? 256 : 512;
  q.key_block_slots = q.T / q.key_block + q.R;
  q.split = 1;
  q.key_block2 = q.key_block; q.split2 = 1; q.spare2 = 1; q.key_block_slots2 = q.key_block_slots;
  q.via_finish = 0;
  q.max_key_blocks = q.key_block_slots;
  const long long rs = (long long)q.R * q.n_obs;
  q.row_slots = rs < q.T ? (int)rs : q.T;
  *pb = q;
  return UP_OK;
}

int check_cu(const up_params* p, const int32_t* cu_host) {
  if (cu_host == nullptr) return UP_ERR_NULL;
  if (cu_host[0] != 0) return UP_ERR_SHAPE;
  for (int r = 0; r < p->num_seqs; ++r)
    if (cu_host[r + 1] < cu_host[r]) return UP_ERR_SHAPE;
  if (cu_host[p->num_seqs] != p->total_tokens) return UP_ERR_SHAPE;
  return UP_OK;
}

// Key-side offsets of tokens that follow earlier context: every sequence has at least as many
// keys as tokens.
int check_cu_k(const up_params* p, const int32_t* cu_host, const int32_t* cu_k_host) {
  if (cu_k_host == nullptr) return UP_ERR_NULL;
  if (cu_k_host[0] != 0) return UP_ERR_SHAPE;
  for (int r = 0; r < p->num_seqs; ++r)
    if (cu_k_host[r + 1] - cu_k_host[r] < cu_host[r + 1] - cu_host[r]) return UP_ERR_SHAPE;
  return UP_OK;
}

int check_ratio(const up_params* p, const float* ratio_host) {
  if (p->num_seqs == 0) return UP_OK;       // an empty array may be NULL
  if (ratio_host == nullptr) return UP_ERR_NULL;
  for (int r = 0; r < p->num_seqs; ++r)
    if (!(ratio_host[r] > 0.0f && ratio_host[r] <= 1.0f)) return UP_ERR_RANGE;
  return UP_OK;
}

// Launch geometry of the scoring sweeps from the sequence lengths.  A work-group owns one key
// block (512 keys with 16 waves; 256 with 8 waves for head rows of 512 bytes, or when even a full head
// split leaves most of the chip idle) and `split` work-groups share a key block, each sweeping
// Hkv / split kv heads.  The split grows (powers of two dividing Hkv) until the launch has about
// one work-group per CU; launches of a few rounds are split further (below).
//   live(kb)  key blocks of kb keys that have work in this pass
//   grid(kb)  slots of the launch (the live ones plus the spares that sit between them)
struct PassGeometry { int kb, split; };
template <class Live, class Grid>
PassGeometry pass_geometry(const Problem& pb, long long units_per_head, Live live, Grid grid) {
  constexpr int kCUs = 256, kEnough = 224;
  int kb = narrow_only(pb) ? 256 : 512;
  long long nb = live(kb);
  int split = 1;
  auto can_double = [&]() { return 2 * split <= pb.Hkv && pb.Hkv % (2 * split) == 0; };
  while (nb * split < kEnough && can_double()) split *= 2;
  if (nb * split < kEnough && kb == 512) {
    kb = 256;
    nb = live(kb);
  }
  // A launch of a few rounds balances better with shorter work-groups (their durations differ:
  // edge blocks, ragged sequences): keep halving the heads per work-group up to about six rounds,
  // as long as a work-group still sweeps eight staging units or more.
  // The spare slots exit at once, but they sit between the live work-groups, and a grid of more
  // than one work-group per CU then runs as two rounds even when the live ones alone would fit in
  // one.  So it is the grid that is compared with the CU count (one sequence: its spares come
  // last and do no harm).
  const long long slots = pb.R == 1 ? nb : grid(kb);
  if (slots * split > kCUs)
    while (can_double() && nb * split < 6 * kCUs && (pb.Hkv / (2 * split)) * units_per_head >= 8) split *= 2;
  return PassGeometry{kb, split};
}

void choose_geometry(Problem* pb, const int32_t* cu, const int32_t* cu_k = nullptr) {
  const int32_t* ck = cu_k != nullptr ? cu_k : cu;     // pass 1 sweeps every key
  pb->has_ctx = cu_k != nullptr;
  pb->Tk = ck[pb->R];
  int longest_n = 0, longest_k = 0;
  for (int r = 0; r < pb->R; ++r) {
    longest_n = cu[r + 1] - cu[r] > longest_n ? cu[r + 1] - cu[r] : longest_n;
    longest_k = ck[r + 1] - ck[r] > longest_k ? ck[r + 1] - ck[r] : longest_k;
  }
  const long long units_per_head = ((long long)(longest_n < pb->n_obs ? longest_n : pb->n_obs) * pb->Gq + 127) / 128;
  const PassGeometry g1 = pass_geometry(
      *pb, units_per_head,
      [&](int kb) {
        long long n = 0;
        for (int r = 0; r < pb->R; ++r)
          if (cu[r + 1] > cu[r]) n += (ck[r + 1] - ck[r] + kb - 1) / kb;
        return n;
      },
      [&](int kb) { return (long long)pb->Tk / kb + pb->R; });
  pb->key_block = g1.kb;
  pb->split = g1.split;
  pb->key_block_slots = pb->Tk / g1.kb + pb->R;
  pb->max_key_blocks = (longest_k + g1.kb - 1) / g1.kb;
  if (!pb->has_ctx) {
    pb->key_block2 = g1.kb;
    pb->split2 = g1.split;
    pb->spare2 = 1;
    pb->key_block_slots2 = pb->key_block_slots;
  } else {
    // pass 2 sweeps only the key blocks that hold keys of the tokens: from the block of the
    // first token's key (not aligned with the tokens: one more slot per sequence) to the last
    pb->spare2 = 2;
    const PassGeometry g2 = pass_geometry(
        *pb, units_per_head,
        [&](int kb) {
          long long n = 0;
          for (int r = 0; r < pb->R; ++r) {
            const int N = cu[r + 1] - cu[r], L = ck[r + 1] - ck[r];
            if (N > 0) n += (L + kb - 1) / kb - (L - N) / kb;
          }
          return n;
        },
        [&](int kb) { return (long long)pb->T / kb + 2 * pb->R; });
    pb->key_block2 = g2.kb;
    pb->split2 = g2.split;
    pb->key_block_slots2 = pb->T / g2.kb + 2 * pb->R;
  }
  pb->via_finish = pb->split2 > 1 || pb->has_ctx;
}

long long host_total_kept(const Problem& pb, const int32_t* cu, const int32_t* cu_k, const float* ratio,
                          int32_t* new_cu_out) {
  long long total = 0;
  if (new_cu_out) new_cu_out[0] = 0;
  for (int r = 0; r < pb.R; ++r) {
    const int N = cu[r + 1] - cu[r];
    // sinks are the first A tokens of the sequence so far; earlier context holds some or all of them
    const int earlier = cu_k != nullptr ? (cu_k[r + 1] - cu_k[r]) - N : 0;
    SeqGeom sg{N, pb.G, pb.n_obs, imax(0, pb.n_sink - earlier), (double)ratio[r]};
    total += seq_kept(sg);
    if (new_cu_out) new_cu_out[r + 1] = (int32_t)total;
  }
  return total;
}

// ---- the entry points that exist with and without earlier context share these bodies
// (cu_k_dev / cu_k_host are nullptr for sequences whose keys are their own tokens' keys)

int plan_impl(const up_params* p, const int32_t* cu_host, const int32_t* cu_k_host, bool ctx,
              const float* ratio_host, int32_t* new_cu_host, int64_t* total_kept, size_t* workspace_bytes) {
  Problem pb;
  const bool want_ws = workspace_bytes != nullptr;
  int st = check_params(p, want_ws, false, &pb);
  if (st != UP_OK) return st;
  if ((st = check_cu(p, cu_host)) != UP_OK) return st;
  if (ctx && (st = check_cu_k(p, cu_host, cu_k_host)) != UP_OK) return st;
  if ((st = check_ratio(p, ratio_host)) != UP_OK) return st;
  const long long total = host_total_kept(pb, cu_host, cu_k_host, ratio_host, new_cu_host);
  if (total_kept) *total_kept = total;
  if (want_ws) choose_geometry(&pb, cu_host, cu_k_host);
  if (want_ws) *workspace_bytes = workspace_layout(pb).total;
  return UP_OK;
}

// Where the keys of the tokens' sequences are: packed with the tokens (ctx false), packed by
// their own offsets after earlier context (ctx), or in a paged cache addressed through a block
// table (ctx with paged).
struct KeySide {
  const int32_t* cu_k_dev;
  const int32_t* cu_k_host;
  bool ctx;
  const PagedKeys* paged;
};
const KeySide kOwnKeys{nullptr, nullptr, false, nullptr};

int check_key_side(const up_params* p, const int32_t* cu_host, const KeySide& ks) {
  if (!ks.ctx) return UP_OK;
  if (!ks.cu_k_dev) return UP_ERR_NULL;
  int st = check_cu_k(p, cu_host, ks.cu_k_host);
  if (st != UP_OK) return st;
  if (ks.paged != nullptr) {
    if (ks.paged->block_table == nullptr) return UP_ERR_NULL;
    if (ks.paged->kv_block < 1 || ks.paged->table_stride < 0) return UP_ERR_RANGE;
    for (int r = 0; r < p->num_seqs; ++r) {
      const long long blocks = ((long long)(ks.cu_k_host[r + 1] - ks.cu_k_host[r]) + ks.paged->kv_block - 1) / ks.paged->kv_block;
      if (blocks > ks.paged->table_stride) return UP_ERR_SHAPE;     // a row of the table is too short
    }
  }
  return UP_OK;
}

// key side of the entries that take it as optional arguments (both offset pointers or neither;
// a block table only with them)
int optional_key_side(const int32_t* cu_k_dev, const int32_t* cu_k_host, const PagedKeys* paged, KeySide* ks) {
  if ((cu_k_dev == nullptr) != (cu_k_host == nullptr)) return UP_ERR_NULL;
  const bool ctx = cu_k_host != nullptr;
  if (!ctx && paged->block_table != nullptr) return UP_ERR_NULL;      // a block table needs the key counts
  *ks = KeySide{cu_k_dev, cu_k_host, ctx, paged->block_table != nullptr ? paged : nullptr};
  return UP_OK;
}

int score_impl(const up_params* p, const void* q, const void* k, const int32_t* cu_dev,
               const int32_t* cu_host, const KeySide& ks, float* scores_out, void* workspace,
               size_t workspace_bytes, void* stream, const float* lse = nullptr, long long lse_stride = 0,
               double* colsum_out = nullptr) {
  const int32_t* cu_k_dev = ks.cu_k_dev;
  const int32_t* cu_k_host = ks.cu_k_host;
  Problem pb;
  int st = check_params(p, true, false, &pb);
  if (st != UP_OK) return st;
  if (!cu_dev || (pb.T > 0 && (!q || !k || (!scores_out && !colsum_out)))) return UP_ERR_NULL;
  if ((st = check_cu(p, cu_host)) != UP_OK) return st;
  if ((st = check_key_side(p, cu_host, ks)) != UP_OK) return st;
  if (lse != nullptr && lse_stride < pb.T) return UP_ERR_SHAPE;      // the heads of lse would overlap
  if (!aligned16(q) || !aligned16(k)) return UP_ERR_ALIGN;
  choose_geometry(&pb, cu_host, cu_k_host);
  if (pb.T > 0 && (workspace == nullptr || workspace_bytes < workspace_layout(pb).total)) return UP_ERR_WORKSPACE;
  if (pb.T > 0 && (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return UP_ERR_ALIGN;
  hipStream_t s = (hipStream_t)stream;
  if (lse != nullptr) {      // the rows' normalisers are given: no pass 1, no merge
    if (launch_lse_stats(pb, cu_dev, cu_k_dev, lse, lse_stride, workspace, nullptr, nullptr, s) != hipSuccess)
      return UP_ERR_HIP;
  } else {
    if (launch_row_stats(pb, q, k, cu_dev, cu_k_dev, ks.paged, workspace, s) != hipSuccess) return UP_ERR_HIP;
    if (launch_merge_stats(pb, cu_dev, cu_k_dev, workspace, nullptr, nullptr, s) != hipSuccess) return UP_ERR_HIP;
  }
  if (launch_column_sums(pb, q, k, cu_dev, cu_k_dev, ks.paged, workspace, scores_out, nullptr, s, colsum_out) !=
      hipSuccess)
    return UP_ERR_HIP;
  return UP_OK;
}

int select_impl(const up_params* p, const float* scores, const int32_t* cu_dev, const int32_t* cu_host,
                const int32_t* cu_k_dev, const int32_t* cu_k_host, bool ctx, const float* ratio_dev,
                const float* ratio_host, int32_t* kept_idx, int32_t* new_cu_dev, void* stream) {
  Problem pb;
  int st = check_params(p, false, false, &pb);
  if (st != UP_OK) return st;
  if (!cu_dev || (pb.R > 0 && !ratio_dev) || !new_cu_dev || (ctx && !cu_k_dev) || (pb.T > 0 && (!scores || !kept_idx)))
    return UP_ERR_NULL;
  if ((st = check_cu(p, cu_host)) != UP_OK) return st;
  if (ctx && (st = check_cu_k(p, cu_host, cu_k_host)) != UP_OK) return st;
  if ((st = check_ratio(p, ratio_host)) != UP_OK) return st;
  hipStream_t s = (hipStream_t)stream;
  if (launch_plan(pb, cu_dev, cu_k_dev, ratio_dev, new_cu_dev, s) != hipSuccess) return UP_ERR_HIP;
  const SelectArgs sa = make_select_args(pb, scores, cu_dev, cu_k_dev, ratio_dev, new_cu_dev, kept_idx);
  if (launch_select(pb, sa, s) != hipSuccess) return UP_ERR_HIP;
  return UP_OK;
}

int fused_impl(const up_params* p, const void* q, const void* k, const void* hidden, const int32_t* pos,
               const int32_t* cu_dev, const int32_t* cu_host, const KeySide& ks, const float* ratio_dev,
               const float* ratio_host, void* hidden_out, int32_t* pos_out, int32_t* kept_idx,
               int32_t* new_cu_dev, float* scores_out, void* workspace, size_t workspace_bytes,
               int phase_mask, void* stream, const float* lse = nullptr, long long lse_stride = 0) {
  const int32_t* cu_k_dev = ks.cu_k_dev;
  const int32_t* cu_k_host = ks.cu_k_host;
  Problem pb;
  int st = check_params(p, true, true, &pb);
  if (st != UP_OK) return st;
  // (a batch without tokens touches none of the per-token arrays: they may be NULL then)
  if (!cu_dev || (pb.R > 0 && !ratio_dev) || !new_cu_dev ||
      (pb.T > 0 && (!q || !k || !hidden || !hidden_out || !kept_idx)))
    return UP_ERR_NULL;
  if (pb.T > 0 && (pos == nullptr) != (pos_out == nullptr)) return UP_ERR_NULL;
  if ((st = check_cu(p, cu_host)) != UP_OK) return st;
  if ((st = check_key_side(p, cu_host, ks)) != UP_OK) return st;
  if ((st = check_ratio(p, ratio_host)) != UP_OK) return st;
  if (lse != nullptr && lse_stride < pb.T) return UP_ERR_SHAPE;      // the heads of lse would overlap
  if (!aligned16(q) || !aligned16(k) || !aligned16(hidden) || !aligned16(hidden_out))
    return UP_ERR_ALIGN;
  choose_geometry(&pb, cu_host, cu_k_host);
  const Workspace w = workspace_layout(pb);
  if (pb.T > 0 && (workspace == nullptr || workspace_bytes < w.total)) return UP_ERR_WORKSPACE;
  if (pb.T > 0 && (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return UP_ERR_ALIGN;
  if (phase_mask & ~(UP_PHASE_ALL | UP_PHASE_GATHER_IN_SELECT)) return UP_ERR_RANGE;
  hipStream_t s = (hipStream_t)stream;
  if (pb.T == 0) {      // no token: only the offsets (all zero) are written
    if ((phase_mask & UP_PHASE_PLAN) && launch_plan(pb, cu_dev, cu_k_dev, ratio_dev, new_cu_dev, s) != hipSuccess)
      return UP_ERR_HIP;
    return UP_OK;
  }
  if (lse != nullptr) {
    // the rows' normalisers are given: no pass 1, no merge; the plan rides in the conversion
    if (launch_lse_stats(pb, cu_dev, cu_k_dev, lse, lse_stride, workspace, ratio_dev, new_cu_dev, s) != hipSuccess)
      return UP_ERR_HIP;
    phase_mask &= ~(UP_PHASE_PLAN | UP_PHASE_ROW_STATS | UP_PHASE_MERGE_STATS);
  }
  // the plan rides in the merge kernel when both are asked for (one launch less)
  const bool plan_in_merge = (phase_mask & UP_PHASE_PLAN) && (phase_mask & UP_PHASE_MERGE_STATS);
  if ((phase_mask & UP_PHASE_PLAN) && !plan_in_merge &&
      launch_plan(pb, cu_dev, cu_k_dev, ratio_dev, new_cu_dev, s) != hipSuccess)
    return UP_ERR_HIP;
  // sequences that are kept whole (every token a sink or in the window: decode rows, short requests)
  // are not scored when the caller wants no scores
  const bool skip_forced = scores_out == nullptr;
  if ((phase_mask & UP_PHASE_ROW_STATS) &&
      launch_row_stats(pb, q, k, cu_dev, cu_k_dev, ks.paged, workspace, s, skip_forced) != hipSuccess)
    return UP_ERR_HIP;
  if ((phase_mask & UP_PHASE_MERGE_STATS) &&
      launch_merge_stats(pb, cu_dev, cu_k_dev, workspace, plan_in_merge ? ratio_dev : nullptr,
                         plan_in_merge ? new_cu_dev : nullptr, s) != hipSuccess)
    return UP_ERR_HIP;
  if (phase_mask & UP_PHASE_SWEEP_SELECT) {
    const SelectArgs sa = make_select_args(pb, nullptr, cu_dev, cu_k_dev, ratio_dev, new_cu_dev, kept_idx);
    // (UP_PHASE_GATHER_IN_SELECT: the kernel that selects also copies its rows -- kept for measurement)
    const GatherArgs ga = make_gather_args(pb, hidden, pos, hidden_out, pos_out);
    if (launch_column_sums(pb, q, k, cu_dev, cu_k_dev, ks.paged, workspace, scores_out, &sa, s, nullptr, skip_forced,
                           (phase_mask & UP_PHASE_GATHER_IN_SELECT) ? &ga : nullptr) != hipSuccess)
      return UP_ERR_HIP;
  }
  if ((phase_mask & UP_PHASE_GATHER) && !((phase_mask & UP_PHASE_GATHER_IN_SELECT) && (phase_mask & UP_PHASE_SWEEP_SELECT))) {
    // one wave per kept row: measured faster than gathering inside the scoring kernel, whose
    // work-groups all reach their gather at the same moment
    const long long total_kept = host_total_kept(pb, cu_host, cu_k_host, ratio_host, nullptr);
    if (launch_compact(pb, hidden, pos, kept_idx, total_kept, hidden_out, pos_out, s) != hipSuccess)
      return UP_ERR_HIP;
  }
  return UP_OK;
}

int select_top_p_impl(const up_params* p, const float* scores, const int32_t* cu_dev, const int32_t* cu_host,
                      const KeySide& ks, const float* top_p_dev, const float* top_p_host, int32_t* kept_idx,
                      int32_t* new_cu_dev, void* workspace, size_t workspace_bytes, void* stream) {
  Problem pb;
  int st = check_params(p, false, false, &pb);
  if (st != UP_OK) return st;
  if (!cu_dev || (pb.R > 0 && !top_p_dev) || !new_cu_dev || (pb.T > 0 && (!scores || !kept_idx))) return UP_ERR_NULL;
  if ((st = check_cu(p, cu_host)) != UP_OK) return st;
  if ((st = check_key_side(p, cu_host, ks)) != UP_OK) return st;
  if ((st = check_ratio(p, top_p_host)) != UP_OK) return st;
  int max_blocks = 0;
  for (int r = 0; r < p->num_seqs; ++r)
    max_blocks = imax(max_blocks, (cu_host[r + 1] - cu_host[r] + pb.G - 1) / pb.G);
  if (max_blocks > kMaxTopPBlocks) return UP_ERR_UNSUPPORTED;
  if (pb.T == 0) {      // no token: the offsets are all zero (the plan's kernel writes them), no workspace is touched
    if (launch_plan(pb, cu_dev, ks.cu_k_dev, top_p_dev, new_cu_dev, (hipStream_t)stream) != hipSuccess) return UP_ERR_HIP;
    return UP_OK;
  }
  if (workspace == nullptr || workspace_bytes < workspace_layout(pb).tp_total) return UP_ERR_WORKSPACE;
  if (pb.T > 0 && (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return UP_ERR_ALIGN;
  if (launch_top_p(pb, scores, cu_dev, ks.cu_k_dev, top_p_dev, kept_idx, new_cu_dev, workspace, max_blocks,
                   (hipStream_t)stream) != hipSuccess)
    return UP_ERR_HIP;
  return UP_OK;
}

// score -> top-p selection -> gather with the count on the device; every check of the three
// steps happens before the first launch
int fused_top_p_impl(const up_params* p, const void* q, const void* k, const void* hidden, const int32_t* pos,
                     const int32_t* cu_dev, const int32_t* cu_host, const KeySide& ks, const float* top_p_dev,
                     const float* top_p_host, void* hidden_out, int32_t* pos_out, int32_t* kept_idx,
                     int32_t* new_cu_dev, float* scores, void* workspace, size_t workspace_bytes, void* stream,
                     const float* lse = nullptr, long long lse_stride = 0) {
  Problem pb;
  int st = check_params(p, true, true, &pb);
  if (st != UP_OK) return st;
  if (!cu_dev || (pb.R > 0 && !top_p_dev) || !new_cu_dev ||
      (pb.T > 0 && (!q || !k || !hidden || !hidden_out || !kept_idx || !scores)))
    return UP_ERR_NULL;
  if (lse != nullptr && lse_stride < pb.T) return UP_ERR_SHAPE;
  if (pb.T > 0 && (pos == nullptr) != (pos_out == nullptr)) return UP_ERR_NULL;
  if ((st = check_cu(p, cu_host)) != UP_OK) return st;
  if ((st = check_key_side(p, cu_host, ks)) != UP_OK) return st;
  if ((st = check_ratio(p, top_p_host)) != UP_OK) return st;
  for (int r = 0; r < p->num_seqs; ++r)
    if ((cu_host[r + 1] - cu_host[r] + pb.G - 1) / pb.G > kMaxTopPBlocks) return UP_ERR_UNSUPPORTED;
  if (!aligned16(q) || !aligned16(k) || !aligned16(hidden) || !aligned16(hidden_out)) return UP_ERR_ALIGN;
  choose_geometry(&pb, cu_host, ks.cu_k_host);
  if (pb.T > 0 && (workspace == nullptr || workspace_bytes < workspace_layout(pb).total)) return UP_ERR_WORKSPACE;
  if (pb.T > 0 && (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return UP_ERR_ALIGN;
  if ((st = score_impl(p, q, k, cu_dev, cu_host, ks, scores, workspace, workspace_bytes, stream, lse, lse_stride)) != UP_OK)
    return st;
  if ((st = select_top_p_impl(p, scores, cu_dev, cu_host, ks, top_p_dev, top_p_host, kept_idx, new_cu_dev,
                              workspace, workspace_bytes, stream)) != UP_OK)
    return st;
  return uniprefill_compact_counted(p, hidden, pos, kept_idx, new_cu_dev + p->num_seqs, p->total_tokens, hidden_out,
                                    pos_out, stream);
}

// ---- scratch memory of the call that allocates nothing (uniprefill_fused_static): a static
// device array; every GPU holds its own copy at its own address, looked up once per device.
// In host code the array's name is only a handle for hipGetSymbolAddress -- kernels get the
// address that call returns.
static __device__ __align__(256) unsigned char scratch[UNIPREFILL_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return UP_ERR_HIP;
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (ptr == nullptr) {
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return UP_ERR_HIP;
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);     // (a racing first call stores the same address)
  }
  *out = ptr;
  return UP_OK;
}

}  // namespace

extern "C" {

int uniprefill_plan(const up_params* p, const int32_t* cu_seqlens_host, const float* keep_ratio_host,
                    int32_t* new_cu_seqlens_host, int64_t* total_kept, size_t* workspace_bytes) {
  return plan_impl(p, cu_seqlens_host, nullptr, false, keep_ratio_host, new_cu_seqlens_host, total_kept,
                   workspace_bytes);
}

int uniprefill_plan_chunked(const up_params* p, const int32_t* cu_seqlens_host,
                            const int32_t* cu_seqlens_k_host, const float* keep_ratio_host,
                            int32_t* new_cu_seqlens_host, int64_t* total_kept, size_t* workspace_bytes) {
  return plan_impl(p, cu_seqlens_host, cu_seqlens_k_host, true, keep_ratio_host, new_cu_seqlens_host,
                   total_kept, workspace_bytes);
}

int uniprefill_score(const up_params* p, const void* q, const void* k, const int32_t* cu_seqlens_dev,
                     const int32_t* cu_seqlens_host, float* scores_out, void* workspace,
                     size_t workspace_bytes, void* stream) {
  return score_impl(p, q, k, cu_seqlens_dev, cu_seqlens_host, kOwnKeys, scores_out, workspace,
                    workspace_bytes, stream);
}

int uniprefill_score_chunked(const up_params* p, const void* q, const void* k,
                             const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host,
                             const int32_t* cu_seqlens_k_dev, const int32_t* cu_seqlens_k_host,
                             float* scores_out, void* workspace, size_t workspace_bytes, void* stream) {
  const KeySide ks{cu_seqlens_k_dev, cu_seqlens_k_host, true, nullptr};
  return score_impl(p, q, k, cu_seqlens_dev, cu_seqlens_host, ks, scores_out, workspace, workspace_bytes, stream);
}

int uniprefill_score_paged(const up_params* p, const void* q, const void* k_cache,
                           const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host,
                           const int32_t* cu_seqlens_k_dev, const int32_t* cu_seqlens_k_host,
                           const int32_t* block_table, int64_t block_table_stride, int32_t kv_block_size,
                           float* scores_out, void* workspace, size_t workspace_bytes, void* stream) {
  const PagedKeys paged{block_table, block_table_stride, kv_block_size};
  const KeySide ks{cu_seqlens_k_dev, cu_seqlens_k_host, true, &paged};
  return score_impl(p, q, k_cache, cu_seqlens_dev, cu_seqlens_host, ks, scores_out, workspace, workspace_bytes,
                    stream);
}

int uniprefill_select(const up_params* p, const float* scores, const int32_t* cu_seqlens_dev,
                      const int32_t* cu_seqlens_host, const float* keep_ratio_dev,
                      const float* keep_ratio_host, int32_t* kept_idx, int32_t* new_cu_seqlens_dev,
                      void* stream) {
  return select_impl(p, scores, cu_seqlens_dev, cu_seqlens_host, nullptr, nullptr, false, keep_ratio_dev,
                     keep_ratio_host, kept_idx, new_cu_seqlens_dev, stream);
}

int uniprefill_select_chunked(const up_params* p, const float* scores, const int32_t* cu_seqlens_dev,
                              const int32_t* cu_seqlens_host, const int32_t* cu_seqlens_k_dev,
                              const int32_t* cu_seqlens_k_host, const float* keep_ratio_dev,
                              const float* keep_ratio_host, int32_t* kept_idx,
                              int32_t* new_cu_seqlens_dev, void* stream) {
  return select_impl(p, scores, cu_seqlens_dev, cu_seqlens_host, cu_seqlens_k_dev, cu_seqlens_k_host, true,
                     keep_ratio_dev, keep_ratio_host, kept_idx, new_cu_seqlens_dev, stream);
}

int uniprefill_select_top_p(const up_params* p, const float* scores, const int32_t* cu_seqlens_dev,
                            const int32_t* cu_seqlens_host, const float* top_p_dev,
                            const float* top_p_host, int32_t* kept_idx, int32_t* new_cu_seqlens_dev,
                            void* workspace, size_t workspace_bytes, void* stream) {
  return select_top_p_impl(p, scores, cu_seqlens_dev, cu_seqlens_host, kOwnKeys, top_p_dev, top_p_host, kept_idx,
                           new_cu_seqlens_dev, workspace, workspace_bytes, stream);
}

int uniprefill_select_top_p_chunked(const up_params* p, const float* scores, const int32_t* cu_seqlens_dev,
                                    const int32_t* cu_seqlens_host, const int32_t* cu_seqlens_k_dev,
                                    const int32_t* cu_seqlens_k_host, const float* top_p_dev,
                                    const float* top_p_host, int32_t* kept_idx, int32_t* new_cu_seqlens_dev,
                                    void* workspace, size_t workspace_bytes, void* stream) {
  const KeySide ks{cu_seqlens_k_dev, cu_seqlens_k_host, true, nullptr};
  return select_top_p_impl(p, scores, cu_seqlens_dev, cu_seqlens_host, ks, top_p_dev, top_p_host, kept_idx,
                           new_cu_seqlens_dev, workspace, workspace_bytes, stream);
}

int uniprefill_compact_counted(const up_params* p, const void* hidden, const int32_t* pos,
                               const int32_t* kept_idx, const int32_t* total_kept_dev,
                               int64_t capacity, void* hidden_out, int32_t* pos_out, void* stream) {
  Problem pb;
  int st = check_params(p, false, true, &pb);
  if (st != UP_OK) return st;
  if (capacity < 0 || capacity > p->total_tokens) return UP_ERR_RANGE;
  if (capacity == 0) return UP_OK;      // nothing to copy, nothing launched
  if (!hidden || !kept_idx || !hidden_out || !total_kept_dev) return UP_ERR_NULL;
  if ((pos == nullptr) != (pos_out == nullptr)) return UP_ERR_NULL;
  if (!aligned16(hidden) || !aligned16(hidden_out)) return UP_ERR_ALIGN;
  if (launch_compact_counted(pb, hidden, pos, kept_idx, total_kept_dev, capacity, hidden_out, pos_out,
                             (hipStream_t)stream) != hipSuccess)
    return UP_ERR_HIP;
  return UP_OK;
}

int uniprefill_fused_top_p(const up_params* p, const void* q, const void* k, const void* hidden,
                           const int32_t* pos, const int32_t* cu_seqlens_dev,
                           const int32_t* cu_seqlens_host, const float* top_p_dev,
                           const float* top_p_host, void* hidden_out, int32_t* pos_out,
                           int32_t* kept_idx, int32_t* new_cu_seqlens_dev, float* scores,
                           void* workspace, size_t workspace_bytes, void* stream) {
  return fused_top_p_impl(p, q, k, hidden, pos, cu_seqlens_dev, cu_seqlens_host, kOwnKeys, top_p_dev, top_p_host,
                          hidden_out, pos_out, kept_idx, new_cu_seqlens_dev, scores, workspace, workspace_bytes,
                          stream);
}

int uniprefill_fused_top_p_chunked(const up_params* p, const void* q, const void* k, const void* hidden,
                                   const int32_t* pos, const int32_t* cu_seqlens_dev,
                                   const int32_t* cu_seqlens_host, const int32_t* cu_seqlens_k_dev,
                                   const int32_t* cu_seqlens_k_host, const int32_t* block_table,
                                   int64_t block_table_stride, int32_t kv_block_size, const float* top_p_dev,
                                   const float* top_p_host, void* hidden_out, int32_t* pos_out,
                                   int32_t* kept_idx, int32_t* new_cu_seqlens_dev, float* scores,
                                   void* workspace, size_t workspace_bytes, void* stream) {
  const PagedKeys paged{block_table, block_table_stride, kv_block_size};
  const KeySide ks{cu_seqlens_k_dev, cu_seqlens_k_host, true, block_table != nullptr ? &paged : nullptr};
  return fused_top_p_impl(p, q, k, hidden, pos, cu_seqlens_dev, cu_seqlens_host, ks, top_p_dev, top_p_host,
                          hidden_out, pos_out, kept_idx, new_cu_seqlens_dev, scores, workspace, workspace_bytes,
                          stream);
}

int uniprefill_compact(const up_params* p, const void* hidden, const int32_t* pos,
                       const int32_t* kept_idx, int64_t total_kept, void* hidden_out,
                       int32_t* pos_out, void* stream) {
  Problem pb;
  int st = check_params(p, false, true, &pb);
  if (st != UP_OK) return st;
  if (total_kept < 0 || total_kept > p->total_tokens) return UP_ERR_RANGE;
  if (total_kept == 0) return UP_OK;    // nothing to copy, nothing launched
  if (!hidden || !kept_idx || !hidden_out) return UP_ERR_NULL;
  if ((pos == nullptr) != (pos_out == nullptr)) return UP_ERR_NULL;
  if (!aligned16(hidden) || !aligned16(hidden_out)) return UP_ERR_ALIGN;
  if (launch_compact(pb, hidden, pos, kept_idx, total_kept, hidden_out, pos_out,
                     (hipStream_t)stream) != hipSuccess)
    return UP_ERR_HIP;
  return UP_OK;
}

int uniprefill_scatter(const up_params* p, const void* hidden_compact, const int32_t* kept_idx,
                       int64_t total_kept, void* hidden_full_inout, void* stream) {
  Problem pb;
  int st = check_params(p, false, true, &pb);
  if (st != UP_OK) return st;
  if (total_kept < 0 || total_kept > p->total_tokens) return UP_ERR_RANGE;
  if (total_kept == 0) return UP_OK;    // nothing to copy, nothing launched
  if (!hidden_compact || !kept_idx || !hidden_full_inout) return UP_ERR_NULL;
  if (!aligned16(hidden_compact) || !aligned16(hidden_full_inout)) return UP_ERR_ALIGN;
  if (launch_scatter(pb, hidden_compact, kept_idx, total_kept, hidden_full_inout,
                     (hipStream_t)stream) != hipSuccess)
    return UP_ERR_HIP;
  return UP_OK;
}

int uniprefill_compose_index(const int32_t* outer_idx, int64_t n_outer, const int32_t* inner_idx,
                             const int32_t* n_inner_dev, int64_t n_inner, int32_t* composed_idx,
                             void* stream) {
  if (n_outer < 0 || n_inner < 0 || n_inner > n_outer) return UP_ERR_RANGE;
  if (n_inner == 0) return UP_OK;
  if (!outer_idx || !inner_idx || !composed_idx) return UP_ERR_NULL;
  if (launch_compose(outer_idx, inner_idx, n_inner, n_inner_dev, composed_idx, (hipStream_t)stream) !=
      hipSuccess)
    return UP_ERR_HIP;
  return UP_OK;
}

int uniprefill_keep_mask(const int32_t* kept_idx, int64_t capacity, const int32_t* total_kept_dev,
                         int64_t total_tokens, uint8_t* mask_out, void* stream) {
  if (capacity < 0 || total_tokens < 0 || capacity > total_tokens) return UP_ERR_RANGE;
  if (total_tokens == 0) return UP_OK;
  if (!mask_out || (capacity > 0 && !kept_idx)) return UP_ERR_NULL;
  if (launch_keep_mask(kept_idx, capacity, total_kept_dev, total_tokens, mask_out, (hipStream_t)stream) != hipSuccess)
    return UP_ERR_HIP;
  return UP_OK;
}

int uniprefill_seqused(const int32_t* drop_layers_host, int32_t num_drops, const int32_t* retained_dev,
                       const int32_t* kv_len_dev, const int32_t* orig_len_dev, int32_t num_seqs,
                       int32_t num_layers, int32_t* seqused_out, void* stream) {
  if (num_drops < 0 || num_seqs < 0 || num_layers < 0 || num_layers > 65535) return UP_ERR_RANGE;
  if (num_drops > kMaxDropLayers) return UP_ERR_UNSUPPORTED;
  if (num_drops > 0 && drop_layers_host == nullptr) return UP_ERR_NULL;
  DropLayers drops{};
  drops.n = num_drops;
  for (int k = 0; k < num_drops; ++k) {
    if (drop_layers_host[k] < 0 || (k > 0 && drop_layers_host[k] <= drop_layers_host[k - 1])) return UP_ERR_RANGE;
    drops.layer[k] = drop_layers_host[k];
  }
  if (num_seqs == 0 || num_layers == 0) return UP_OK;
  if ((num_drops > 0 && !retained_dev) || !kv_len_dev || !orig_len_dev || !seqused_out) return UP_ERR_NULL;
  if (launch_seqused(drops, retained_dev, kv_len_dev, orig_len_dev, num_seqs, num_layers, seqused_out,
                     (hipStream_t)stream) != hipSuccess)
    return UP_ERR_HIP;
  return UP_OK;
}

int uniprefill_compact_column(const void* column, int32_t elem_bytes, const int32_t* kept_idx,
                              int64_t capacity, const int32_t* total_kept_dev, void* column_out,
                              void* stream) {
  if (elem_bytes != 4 && elem_bytes != 8) return UP_ERR_UNSUPPORTED;
  if (capacity < 0) return UP_ERR_RANGE;
  if (capacity == 0) return UP_OK;
  if (!column || !kept_idx || !column_out) return UP_ERR_NULL;
  const uintptr_t mask = (uintptr_t)elem_bytes - 1;
  if ((reinterpret_cast<uintptr_t>(column) & mask) || (reinterpret_cast<uintptr_t>(column_out) & mask))
    return UP_ERR_ALIGN;
  if (launch_column(column, elem_bytes, kept_idx, capacity, total_kept_dev, column_out,
                    (hipStream_t)stream) != hipSuccess)
    return UP_ERR_HIP;
  return UP_OK;
}

int uniprefill_slot_mapping(const int32_t* pos_kept, const int32_t* new_cu_seqlens_dev, int32_t num_seqs,
                            const int32_t* block_table, int64_t block_table_stride, int32_t kv_block_size,
                            int64_t capacity, int64_t* slots, void* stream) {
  if (num_seqs < 0 || capacity < 0 || kv_block_size < 1 || block_table_stride < 0) return UP_ERR_RANGE;
  if (capacity == 0 || num_seqs == 0) return UP_OK;
  if (!pos_kept || !new_cu_seqlens_dev || !block_table || !slots) return UP_ERR_NULL;
  if (launch_slot_mapping(pos_kept, new_cu_seqlens_dev, num_seqs, block_table, block_table_stride,
                          kv_block_size, capacity, slots, (hipStream_t)stream) != hipSuccess)
    return UP_ERR_HIP;
  return UP_OK;
}

int uniprefill_fused_phases(const up_params* p, const void* q, const void* k, const void* hidden,
                            const int32_t* pos, const int32_t* cu_seqlens_dev,
                            const int32_t* cu_seqlens_host, const float* keep_ratio_dev,
                            const float* keep_ratio_host, void* hidden_out, int32_t* pos_out,
                            int32_t* kept_idx, int32_t* new_cu_seqlens_dev, float* scores_out,
                            void* workspace, size_t workspace_bytes, int phase_mask, void* stream) {
  return fused_impl(p, q, k, hidden, pos, cu_seqlens_dev, cu_seqlens_host, kOwnKeys,
                    keep_ratio_dev, keep_ratio_host, hidden_out, pos_out, kept_idx, new_cu_seqlens_dev,
                    scores_out, workspace, workspace_bytes, phase_mask, stream);
}

int uniprefill_fused_chunked(const up_params* p, const void* q, const void* k, const void* hidden,
                             const int32_t* pos, const int32_t* cu_seqlens_dev,
                             const int32_t* cu_seqlens_host, const int32_t* cu_seqlens_k_dev,
                             const int32_t* cu_seqlens_k_host, const float* keep_ratio_dev,
                             const float* keep_ratio_host, void* hidden_out, int32_t* pos_out,
                             int32_t* kept_idx, int32_t* new_cu_seqlens_dev, float* scores_out,
                             void* workspace, size_t workspace_bytes, void* stream) {
  const KeySide ks{cu_seqlens_k_dev, cu_seqlens_k_host, true, nullptr};
  return fused_impl(p, q, k, hidden, pos, cu_seqlens_dev, cu_seqlens_host, ks, keep_ratio_dev, keep_ratio_host,
                    hidden_out, pos_out, kept_idx, new_cu_seqlens_dev, scores_out, workspace, workspace_bytes,
                    UP_PHASE_ALL, stream);
}

int uniprefill_fused_lse(const up_params* p, const void* q, const void* k, const float* lse,
                         int64_t lse_row_stride, const void* hidden, const int32_t* pos,
                         const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host,
                         const int32_t* cu_seqlens_k_dev, const int32_t* cu_seqlens_k_host,
                         const int32_t* block_table, int64_t block_table_stride, int32_t kv_block_size,
                         const float* keep_ratio_dev, const float* keep_ratio_host, void* hidden_out,
                         int32_t* pos_out, int32_t* kept_idx, int32_t* new_cu_seqlens_dev,
                         float* scores_out, void* workspace, size_t workspace_bytes, void* stream) {
  if (lse == nullptr) return UP_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(lse) & 3u) != 0) return UP_ERR_ALIGN;
  const PagedKeys paged{block_table, block_table_stride, kv_block_size};
  KeySide ks;
  const int st = optional_key_side(cu_seqlens_k_dev, cu_seqlens_k_host, &paged, &ks);
  if (st != UP_OK) return st;
  return fused_impl(p, q, k, hidden, pos, cu_seqlens_dev, cu_seqlens_host, ks, keep_ratio_dev, keep_ratio_host,
                    hidden_out, pos_out, kept_idx, new_cu_seqlens_dev, scores_out, workspace, workspace_bytes,
                    UP_PHASE_ALL, stream, lse, lse_row_stride);
}

int uniprefill_score_lse(const up_params* p, const void* q, const void* k, const float* lse,
                         int64_t lse_row_stride, const int32_t* cu_seqlens_dev,
                         const int32_t* cu_seqlens_host, const int32_t* cu_seqlens_k_dev,
                         const int32_t* cu_seqlens_k_host, const int32_t* block_table,
                         int64_t block_table_stride, int32_t kv_block_size, float* scores_out,
                         void* workspace, size_t workspace_bytes, void* stream) {
  if (lse == nullptr) return UP_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(lse) & 3u) != 0) return UP_ERR_ALIGN;
  const PagedKeys paged{block_table, block_table_stride, kv_block_size};
  KeySide ks;
  const int st = optional_key_side(cu_seqlens_k_dev, cu_seqlens_k_host, &paged, &ks);
  if (st != UP_OK) return st;
  return score_impl(p, q, k, cu_seqlens_dev, cu_seqlens_host, ks, scores_out, workspace, workspace_bytes, stream,
                    lse, lse_row_stride);
}

int uniprefill_fused_top_p_lse(const up_params* p, const void* q, const void* k, const float* lse,
                               int64_t lse_row_stride, const void* hidden, const int32_t* pos,
                               const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host,
                               const int32_t* cu_seqlens_k_dev, const int32_t* cu_seqlens_k_host,
                               const int32_t* block_table, int64_t block_table_stride,
                               int32_t kv_block_size, const float* top_p_dev, const float* top_p_host,
                               void* hidden_out, int32_t* pos_out, int32_t* kept_idx,
                               int32_t* new_cu_seqlens_dev, float* scores, void* workspace,
                               size_t workspace_bytes, void* stream) {
  if (lse == nullptr) return UP_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(lse) & 3u) != 0) return UP_ERR_ALIGN;
  const PagedKeys paged{block_table, block_table_stride, kv_block_size};
  KeySide ks;
  const int st = optional_key_side(cu_seqlens_k_dev, cu_seqlens_k_host, &paged, &ks);
  if (st != UP_OK) return st;
  return fused_top_p_impl(p, q, k, hidden, pos, cu_seqlens_dev, cu_seqlens_host, ks, top_p_dev, top_p_host,
                          hidden_out, pos_out, kept_idx, new_cu_seqlens_dev, scores, workspace, workspace_bytes,
                          stream, lse, lse_row_stride);
}

int uniprefill_score_partial(const up_params* p, const void* q, const void* k,
                             const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host,
                             const int32_t* cu_seqlens_k_dev, const int32_t* cu_seqlens_k_host,
                             double* colsum_out, void* workspace, size_t workspace_bytes, void* stream) {
  if (p != nullptr && p->total_tokens > 0 && colsum_out == nullptr) return UP_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(colsum_out) & 7u) != 0) return UP_ERR_ALIGN;
  const PagedKeys none{nullptr, 0, 1};
  KeySide ks;
  const int st = optional_key_side(cu_seqlens_k_dev, cu_seqlens_k_host, &none, &ks);
  if (st != UP_OK) return st;
  return score_impl(p, q, k, cu_seqlens_dev, cu_seqlens_host, ks, nullptr, workspace, workspace_bytes, stream,
                    nullptr, 0, colsum_out);
}

int uniprefill_scores_from_partials(const double* partials, int32_t num_parts, int64_t part_stride,
                                    const int32_t* cu_seqlens_dev, int32_t num_seqs, int32_t total_tokens,
                                    int32_t n_obs, int32_t total_q_heads, float* scores_out, void* stream) {
  if (num_parts < 1 || num_seqs < 0 || total_tokens < 0 || n_obs < 1 || total_q_heads < 1 ||
      part_stride < total_tokens)
    return UP_ERR_RANGE;
  if (total_tokens == 0) return UP_OK;
  if (!partials || !cu_seqlens_dev || !scores_out) return UP_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(partials) & 7u) != 0) return UP_ERR_ALIGN;
  if (launch_scores_from_partials(partials, num_parts, part_stride, cu_seqlens_dev, num_seqs, total_tokens, n_obs,
                                  total_q_heads, scores_out, (hipStream_t)stream) != hipSuccess)
    return UP_ERR_HIP;
  return UP_OK;
}

int uniprefill_fused_paged(const up_params* p, const void* q, const void* k_cache, const void* hidden,
                           const int32_t* pos, const int32_t* cu_seqlens_dev,
                           const int32_t* cu_seqlens_host, const int32_t* cu_seqlens_k_dev,
                           const int32_t* cu_seqlens_k_host, const int32_t* block_table,
                           int64_t block_table_stride, int32_t kv_block_size, const float* keep_ratio_dev,
                           const float* keep_ratio_host, void* hidden_out, int32_t* pos_out,
                           int32_t* kept_idx, int32_t* new_cu_seqlens_dev, float* scores_out,
                           void* workspace, size_t workspace_bytes, void* stream) {
  const PagedKeys paged{block_table, block_table_stride, kv_block_size};
  const KeySide ks{cu_seqlens_k_dev, cu_seqlens_k_host, true, &paged};
  return fused_impl(p, q, k_cache, hidden, pos, cu_seqlens_dev, cu_seqlens_host, ks, keep_ratio_dev,
                    keep_ratio_host, hidden_out, pos_out, kept_idx, new_cu_seqlens_dev, scores_out, workspace,
                    workspace_bytes, UP_PHASE_ALL, stream);
}

int uniprefill_fused(const up_params* p, const void* q, const void* k, const void* hidden,
                     const int32_t* pos, const int32_t* cu_seqlens_dev,
                     const int32_t* cu_seqlens_host, const float* keep_ratio_dev,
                     const float* keep_ratio_host, void* hidden_out, int32_t* pos_out,
                     int32_t* kept_idx, int32_t* new_cu_seqlens_dev, float* scores_out,
                     void* workspace, size_t workspace_bytes, void* stream) {
  return uniprefill_fused_phases(p, q, k, hidden, pos, cu_seqlens_dev, cu_seqlens_host,
                                 keep_ratio_dev, keep_ratio_host, hidden_out, pos_out, kept_idx,
                                 new_cu_seqlens_dev, scores_out, workspace, workspace_bytes,
                                 UP_PHASE_ALL, stream);
}

int uniprefill_fused_static(const up_params* p, const void* q, const void* k, const void* hidden,
                            const int32_t* pos, const int32_t* cu_seqlens_dev,
                            const int32_t* cu_seqlens_host, const float* keep_ratio_dev,
                            const float* keep_ratio_host, void* hidden_out, int32_t* pos_out,
                            int32_t* kept_idx, int32_t* new_cu_seqlens_dev, float* scores_out,
                            void* stream) {
  // what the call needs, from the same closed forms as uniprefill_plan (host only)
  size_t need = 0;
  const int st = plan_impl(p, cu_seqlens_host, nullptr, false, keep_ratio_host, nullptr, nullptr, &need);
  if (st != UP_OK) return st;
  if (need > (size_t)UNIPREFILL_STATIC_SCRATCH_BYTES) return UP_ERR_SCRATCH;
  void* ws = nullptr;
  if (p->total_tokens > 0) {      // (a batch without tokens touches no workspace)
    const int sw = static_scratch(&ws);
    if (sw != UP_OK) return sw;
  }
  return fused_impl(p, q, k, hidden, pos, cu_seqlens_dev, cu_seqlens_host, kOwnKeys, keep_ratio_dev, keep_ratio_host,
                    hidden_out, pos_out, kept_idx, new_cu_seqlens_dev, scores_out, ws,
                    (size_t)UNIPREFILL_STATIC_SCRATCH_BYTES, UP_PHASE_ALL, stream);
}

const char* uniprefill_status_string(int status) {
  switch (status) {
    case UP_OK: return "ok";
    case UP_ERR_NULL: return "required pointer is NULL";
    case UP_ERR_SHAPE: return "inconsistent shape or cu_seqlens";
    case UP_ERR_RANGE: return "parameter out of range";
    case UP_ERR_UNSUPPORTED: return "unsupported configuration";
    case UP_ERR_ALIGN: return "pointer or row stride not 16-byte aligned";
    case UP_ERR_WORKSPACE: return "workspace missing or too small";
    case UP_ERR_HIP: return "kernel launch failed";
    case UP_ERR_SCRATCH: return "the library's static scratch buffer is too small for this call";
    default: return "unknown status";
  }
}

}  // extern "C"
