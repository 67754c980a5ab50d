// Launchers of the gfx950 kernels behind the C ABI (internal header).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace up {

struct SelectArgs;

// Static description of one call, derived on the host from up_params.
struct Problem {
  int R, T;
  int Tk;                     // key rows: T, or more when the tokens follow earlier context
  int has_ctx;                // a key-side cu_seqlens is given
  int G, n_obs, n_sink;
  int Hq, Hkv, Gq;            // Gq = query heads per kv head
  int d;
  long long q_stride, k_stride, h_stride;  // elements
  int hidden_elem_bytes;      // 2 (bf16) or 4 (f32)
  int qk_is_f32;
  int head_dim;               // 64, 128 or 256 (256: bf16 only)
  float scale;                // softmax scale (resolved, > 0)
  // pass 1 (row statistics) runs over every key of every sequence
  int key_block;              // keys per work-group: 256 or 512
  int key_block_slots;        // Tk / key_block + R: key blocks of all sequences (an upper bound)
  int split;                  // work-groups per key block: each sweeps Hkv / split kv heads
  // pass 2 (column sums) runs over the tokens' own keys; without earlier context its geometry is
  // that of pass 1
  int key_block2, split2;
  int spare2;                 // slots per sequence beyond N / key_block2: 1, or 2 with earlier context
                              // (the tokens' first key is then not aligned with a key block)
  int key_block_slots2;       // T / key_block2 + spare2 * R
  int via_finish;             // pass 2 leaves column sums in the workspace and k_finish selects
                              // (split2 > 1, or earlier context: tokens and key blocks not aligned)
  int max_key_blocks;         // key blocks of the longest sequence
  int row_slots;              // min(T, R * n_obs): window rows of all sequences
};

// Workspace carve-up (byte offsets, each 256-aligned).
struct Workspace {
  size_t stat_part_off, stat_fin_off, o_part_off, total;
  size_t tp_keep_off, tp_off_off, tp_seq_off, tp_mass_off, tp_rank_off, tp_sorted_off, tp_total;   // top-p selection part (first tp_total bytes)
};
Workspace workspace_layout(const Problem& pb);

// --- copies (Eq. 7 / Eq. 8)
// The gather as a rider of the kernel that selects (hidden == nullptr: it does not ride).  Measured
// slower than the launch of its own on every workload, so the fused call does not use it; it stays
// selectable so that the comparison can be repeated.
struct GatherArgs {
  const char* hidden;
  char* hidden_out;
  const int32_t* pos;      // nullptr: no position ids
  int32_t* pos_out;
  long long row_bytes, stride_bytes;
};
GatherArgs make_gather_args(const Problem& pb, const void* hidden, const int32_t* pos, void* hidden_out,
                            int32_t* pos_out);
hipError_t launch_compact(const Problem& pb, const void* hidden, const int32_t* pos,
                          const int32_t* kept_idx, long long total_kept, void* hidden_out,
                          int32_t* pos_out, hipStream_t s);
hipError_t launch_scatter(const Problem& pb, const void* hidden_compact, const int32_t* kept_idx,
                          long long total_kept, void* hidden_full, hipStream_t s);

// index map of two successive drops: out[t] = outer[inner[t]], t < n (or < count_dev[0] <= n)
hipError_t launch_compose(const int32_t* outer, const int32_t* inner, long long n,
                          const int32_t* count_dev, int32_t* out, hipStream_t s);

// one per-token column of 4- or 8-byte elements: out[t] = column[idx[t]], t < n (and < count_dev[0])
hipError_t launch_column(const void* column, int elem_bytes, const int32_t* idx, long long n,
                         const int32_t* count_dev, void* out, hipStream_t s);

// token keep mask (one byte per token) from the ascending list of kept rows
hipError_t launch_keep_mask(const int32_t* kept_idx, long long capacity, const int32_t* count_dev, long long T,
                            uint8_t* mask, hipStream_t s);

// per-layer KV length during decode (Eq. 17): out[l][r] for l < num_layers
constexpr int kMaxDropLayers = 64;
struct DropLayers { int n; int layer[kMaxDropLayers]; };
hipError_t launch_seqused(const DropLayers& drops, const int32_t* retained, const int32_t* kv_len,
                          const int32_t* orig_len, int R, int num_layers, int32_t* out, hipStream_t s);

// physical KV-cache slots of the retained tokens (Eq. 16); the token count is new_cu[R] on the device
hipError_t launch_slot_mapping(const int32_t* pos_kept, const int32_t* new_cu, int R,
                               const int32_t* block_table, long long table_stride, int kv_block,
                               long long capacity, int64_t* slots, hipStream_t s);

// --- selection
// (cu_k: key-side offsets when the tokens follow earlier context, else nullptr)
hipError_t launch_plan(const Problem& pb, const int32_t* cu, const int32_t* cu_k, const float* ratio,
                       int32_t* new_cu, hipStream_t s);
SelectArgs make_select_args(const Problem& pb, const float* scores, const int32_t* cu, const int32_t* cu_k,
                            const float* ratio, const int32_t* new_cu, int32_t* kept_idx);
hipError_t launch_select(const Problem& pb, const SelectArgs& a, hipStream_t s);

// --- block-level top-p selection (Eq. 4-6); kept_idx needs room for T entries
constexpr int kMaxTopPBlocks = 65536;   // blocks of one sequence that the top-p kernels order (1024 chunks of the running sum)
struct TopPArgs {
  const float* scores;
  const int32_t* cu;
  const int32_t* cu_k;   // key-side offsets when the tokens follow earlier context, else nullptr
  const float* top_p;
  int32_t* kept_idx;
  int32_t* new_cu;
  int32_t* blk_keep;     // [T/G + R] block chosen by the top-p rule
  int32_t* blk_off;      // [T/G + R] kept tokens of the sequence before this block
  int32_t* seq_kept;     // [R] kept tokens per sequence
  float* blk_mass;       // [T/G + R] block masses
  int32_t* blk_rank;     // [T/G + R] place of the block in the descending order of its sequence
  float* blk_sorted;     // [T/G + R] the masses of a sequence's blocks in that order
  int R, T, G, n_obs, n_sink;
};
// (max_blocks: selection blocks of the longest sequence, at most kMaxTopPBlocks)
hipError_t launch_top_p(const Problem& pb, const float* scores, const int32_t* cu, const int32_t* cu_k,
                        const float* top_p, int32_t* kept_idx, int32_t* new_cu, void* workspace, int max_blocks,
                        hipStream_t s);
// gather with the row count on the device (count_dev[0] rows, at most capacity)
hipError_t launch_compact_counted(const Problem& pb, const void* hidden, const int32_t* pos,
                                  const int32_t* kept_idx, const int32_t* count_dev, long long capacity,
                                  void* hidden_out, int32_t* pos_out, hipStream_t s);

// Keys in a paged KV cache: key i of sequence r is row
// block_table[r * table_stride + i / kv_block] * kv_block + i % kv_block of k (the indexing of Eq. 16).
struct PagedKeys {
  const int32_t* block_table;
  long long table_stride;
  int kv_block;
};

// --- scoring (Eq. 2-3)
// pass 1: softmax statistics of every window row per key block (into the workspace)
// (cu_k as above; the kernels take cu itself where it is nullptr)
// (paged: nullptr when the keys are packed by cu / cu_k)
// (skip_forced: sequences that are kept whole whatever their scores are left out -- for a call
// that selects and returns no scores; both passes must agree on it)
hipError_t launch_row_stats(const Problem& pb, const void* q, const void* k, const int32_t* cu,
                            const int32_t* cu_k, const PagedKeys* paged, void* workspace, hipStream_t s,
                            bool skip_forced = false);
// merge of the per-block statistics into one (reference, 1/sum) per row; with plan_ratio given
// the same launch also does what launch_plan does (into plan_new_cu)
hipError_t launch_merge_stats(const Problem& pb, const int32_t* cu, const int32_t* cu_k, void* workspace,
                              const float* plan_ratio, int32_t* plan_new_cu, hipStream_t s);
// instead of the two launches above: the rows' normalisers are given (lse[h * lse_stride + t] =
// natural log of the sum of exponentials of token t's row in head h)
hipError_t launch_lse_stats(const Problem& pb, const int32_t* cu, const int32_t* cu_k, const float* lse,
                            long long lse_stride, void* workspace, const float* plan_ratio, int32_t* plan_new_cu,
                            hipStream_t s);
// pass 2: normalised weights summed per token; optional scores_out; sel != nullptr runs the
// block-local top-k (in the same kernel when every key block has one work-group, otherwise in
// k_finish)
// colsum_out != nullptr: also the raw column sums in double (always through k_finish)
hipError_t launch_column_sums(const Problem& pb, const void* q, const void* k, const int32_t* cu,
                              const int32_t* cu_k, const PagedKeys* paged, void* workspace, float* scores_out,
                              const SelectArgs* sel, hipStream_t s, double* colsum_out = nullptr,
                              bool skip_forced = false, const GatherArgs* gather = nullptr);
// (gather != nullptr, with sel: the kernel that selects -- pass 2 itself or k_finish -- also copies its kept rows)
// scores from the tensor-parallel ranks' partial column sums (Eq. 15): parts added in rank order
hipError_t launch_scores_from_partials(const double* partials, int num_parts, long long part_stride,
                                       const int32_t* cu, int R, int T, int n_obs, int total_q_heads,
                                       float* scores, hipStream_t s);

}  // namespace up
