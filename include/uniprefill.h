/*
 * uniprefill.h -- C ABI of the UniPrefill block-wise token-sparsification operator
 * for AMD MI355X (gfx950).
 *
 * The operator works on a packed continuous-batching batch: R sequences stored
 * back to back with no padding and addressed through cu_seqlens, the token
 * layout the kernel-design paragraph of section "Fused Kernel and vLLM
 * Integration" prescribes.  Sequence r owns packed rows
 * [cu_seqlens[r], cu_seqlens[r+1]).
 *
 * Conventions shared by every entry point
 *   - "dev"  pointers are device (HBM) addresses, "host" pointers are host
 *     addresses.  Unmarked data pointers (q, k, hidden, pos, scores, kept_idx,
 *     workspace, outputs) are device addresses.
 *   - Ownership: the caller owns every buffer.  The library never allocates or
 *     frees device memory, keeps no state between calls, and only enqueues work
 *     on `stream` (a hipStream_t passed as void*, NULL = the null stream).  It
 *     never synchronises and never copies device->host; the host copies of
 *     cu_seqlens / keep_ratio that serving engines already hold are passed in.
 *   - Errors: every entry point returns an up_status.  All argument errors are
 *     found on the host before anything is launched, so an error return means
 *     no kernel ran.  Nothing throws or aborts.
 *       UP_ERR_NULL        a required pointer is NULL
 *       UP_ERR_SHAPE       cu_seqlens[0] != 0, cu_seqlens decreasing, or
 *                          cu_seqlens[R] != total_tokens; negative sizes; a
 *                          sequence with fewer keys than tokens (cu_seqlens_k);
 *                          a block-table row shorter than the sequence's keys
 *       UP_ERR_RANGE       keep ratio not in (0,1] or NaN; block_size not in
 *                          {32,64,128}; n_obs < 1 or > 1024; n_sink < 0;
 *                          total_kept inconsistent with the plan; KV block
 *                          size < 1; drop layers not strictly ascending
 *       UP_ERR_UNSUPPORTED head_dim not in {64,128,256}, or 256 with UP_F32
 *                          operands; num_q_heads % num_kv_heads != 0; more than
 *                          64 query heads per kv head; unknown dtype
 *       UP_ERR_ALIGN       a base pointer is not 16-byte aligned or a row stride
 *                          in bytes is not a multiple of 16
 *       UP_ERR_WORKSPACE   workspace is NULL or smaller than uniprefill_plan says
 *       UP_ERR_HIP         a launch failed (hipGetLastError after the launch)
 *       UP_ERR_SCRATCH     uniprefill_fused_static only: the call needs more scratch
 *                          memory than the library's static buffer holds
 *   - Zero-length sequences are legal and produce nothing; total_tokens == 0 is
 *     legal: the per-token arrays (q, k, hidden, scores, kept_idx, outputs) may
 *     then be NULL, and only new_cu_seqlens_dev is written (all zero).  A copy
 *     of zero rows launches nothing and needs no pointers.
 *   - Layouts: q is [T, num_q_heads, head_dim] with row stride q_row_stride
 *     elements between tokens (heads contiguous inside a row); k likewise with
 *     num_kv_heads and k_row_stride; hidden is [T, hidden_dim] with row stride
 *     hidden_row_stride; compacted outputs are dense with the same row stride
 *     convention (hidden_out uses hidden_row_stride as well).
 *     Query head h reads kv head h / (num_q_heads / num_kv_heads).
 */
#ifndef UNIPREFILL_H
#define UNIPREFILL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  UP_OK = 0,
  UP_ERR_NULL = 1,
  UP_ERR_SHAPE = 2,
  UP_ERR_RANGE = 3,
  UP_ERR_UNSUPPORTED = 4,
  UP_ERR_ALIGN = 5,
  UP_ERR_WORKSPACE = 6,
  UP_ERR_HIP = 7,
  UP_ERR_SCRATCH = 8
} up_status;

typedef enum { UP_BF16 = 0, UP_F32 = 1 } up_dtype;

/* Problem description.  Hyper-parameters follow the paper's notation:
 * G = block_size, n = n_obs (observation window: the last n query positions of
 * each sequence), A = n_sink (attention-sink tokens always retained).  The
 * paper's defaults are G = 64, n = 128, A = 128 (Experimental Setup). */
typedef struct {
  int32_t num_seqs;          /* R */
  int32_t total_tokens;      /* T = cu_seqlens[R] */
  int32_t block_size;        /* G in {32, 64, 128} */
  int32_t n_obs;             /* n >= 1 */
  int32_t n_sink;            /* A >= 0 */
  int32_t num_q_heads;
  int32_t num_kv_heads;
  int32_t head_dim;          /* 64, 128 or 256 (256: UP_BF16 operands only) */
  int32_t hidden_dim;        /* d */
  int64_t q_row_stride;      /* elements between consecutive tokens of q */
  int64_t k_row_stride;      /* elements between consecutive tokens of k */
  int64_t hidden_row_stride; /* elements between consecutive rows of hidden */
  float softmax_scale;       /* 0 => 1/sqrt(head_dim)  (Eq. 2) */
  int32_t qk_dtype;          /* up_dtype of q and k (UP_F32: fp32 products, a slower correctness path) */
  int32_t hidden_dtype;      /* up_dtype of hidden (bit-copied, never computed on) */
} up_params;

/* Host-only, pure, needs no GPU.  Closed-form output layout of the block-local
 * selection: inside every block of G consecutive tokens of a sequence (ragged
 * last block allowed; block partition of "Token Importance Estimation") the
 * operator keeps k_g = max(min(L_g, max(1, ceil(ratio * L_g))), F_g) tokens,
 * L_g the block length and F_g the number of tokens in it that are always
 * retained: the first A and the last n of the sequence ("Top-p Token
 * Selection", last sentence).  ratio is a float widened to double, so the
 * product and the ceiling are exact.
 *   new_cu_seqlens_host [R+1] out (may be NULL): prefix sums of kept counts
 *   total_kept          out (may be NULL)
 *   workspace_bytes     out (may be NULL): bytes the scoring entries need */
int uniprefill_plan(const up_params* p, const int32_t* cu_seqlens_host,
                    const float* keep_ratio_host, int32_t* new_cu_seqlens_host,
                    int64_t* total_kept, size_t* workspace_bytes);

/* Token importance (Eq. 2-3; kernels K1/K2 and the head contraction of K3 in
 * the kernel-design paragraph): for each sequence, query head and each of the
 * last n_eff = min(n, N) query rows, the causal softmax over the whole visible
 * key sequence of scale * <q_j, k_i>; score_i = mean over those rows and over
 * all query heads.  Written as float; means below 2^-64 are written as +0.
 *   q, k           device, qk_dtype; only the last n_eff rows of q per sequence
 *                  are read
 *   scores_out     device float [T]
 *   workspace      device scratch of at least workspace_bytes (from the plan),
 *                  256-byte aligned; contents undefined afterwards */
int uniprefill_score(const up_params* p, const void* q, const void* k,
                     const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host,
                     float* scores_out, void* workspace, size_t workspace_bytes,
                     void* stream);

/* Block-local top-k with forced retention (block partition and retained
 * sinks/window as above; integer ordering key of Eq. 14 with the index word
 * complemented so that equal scores resolve to the lower index).  Emits the
 * kept packed row ids in ascending order and the patched sequence offsets
 * (the compacted stream's query_start_loc, "vLLM scheduler integration").
 *   scores              device float [T]
 *   keep_ratio_dev/host [R] each, same values
 *   kept_idx            device int32 [total_kept]   out
 *   new_cu_seqlens_dev  device int32 [R+1]          out */
int uniprefill_select(const up_params* p, const float* scores,
                      const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host,
                      const float* keep_ratio_dev, const float* keep_ratio_host,
                      int32_t* kept_idx, int32_t* new_cu_seqlens_dev, void* stream);

/* Compaction (Eq. 7: later sublayers run on the retained set only):
 * hidden_out[t] = hidden[kept_idx[t]], pos_out[t] = pos[kept_idx[t]].
 * pos / pos_out may both be NULL.  kept_idx values must lie in [0, T). */
int uniprefill_compact(const up_params* p, const void* hidden, const int32_t* pos,
                       const int32_t* kept_idx, int64_t total_kept, void* hidden_out,
                       int32_t* pos_out, void* stream);

/* Reconstitution (Eq. 8): hidden_full[kept_idx[t]] = hidden_compact[t]; rows not
 * named by kept_idx keep their old state.  kept_idx must not repeat a row. */
int uniprefill_scatter(const up_params* p, const void* hidden_compact,
                       const int32_t* kept_idx, int64_t total_kept,
                       void* hidden_full_inout, void* stream);

/* The whole path in one call: score -> select -> compact, enqueued back to back
 * on `stream` with no host synchronisation (the kernel-design paragraph asks for
 * a chain of kernels on the packed layout with no round trip through the host).
 * Outputs as in the single entries; scores_out may
 * be NULL.  hidden_out needs room for the plan's total_kept rows. */
int uniprefill_fused(const up_params* p, const void* q, const void* k, const void* hidden,
                     const int32_t* pos, const int32_t* cu_seqlens_dev,
                     const int32_t* cu_seqlens_host, const float* keep_ratio_dev,
                     const float* keep_ratio_host, void* hidden_out, int32_t* pos_out,
                     int32_t* kept_idx, int32_t* new_cu_seqlens_dev, float* scores_out,
                     void* workspace, size_t workspace_bytes, void* stream);

/* uniprefill_fused for callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same call, the
 * same kernels and the same results, with the workspace inside the library instead of an
 * argument -- a static device array of UNIPREFILL_STATIC_SCRATCH_BYTES that every GPU the
 * library runs on holds until the process ends.  The call allocates and frees nothing.
 *   - A batch whose workspace (what uniprefill_plan reports) exceeds that size is refused
 *     with UP_ERR_SCRATCH before anything is launched: use uniprefill_fused then.
 *   - `stream` must belong to the current device.  The first call on a device looks the
 *     array's address up (no allocation; not to be made under stream capture); later
 *     calls only enqueue.
 *   - All calls on one GPU share that GPU's array: calls that may overlap there (two
 *     streams, two threads) race and must be serialised by the caller.  Nothing in the
 *     array has to start at zero or survive between calls: every word a kernel reads was
 *     written earlier in the same call. */
#define UNIPREFILL_STATIC_SCRATCH_BYTES (32u << 20)
int uniprefill_fused_static(const up_params* p, const void* q, const void* k, const void* hidden,
                            const int32_t* pos, const int32_t* cu_seqlens_dev,
                            const int32_t* cu_seqlens_host, const float* keep_ratio_dev,
                            const float* keep_ratio_host, void* hidden_out, int32_t* pos_out,
                            int32_t* kept_idx, int32_t* new_cu_seqlens_dev, float* scores_out,
                            void* stream);

/* Block-level top-p selection, the rule of Eq. 4-6: inside each sequence the
 * blocks of G tokens are ordered by their mass (sum of the token scores; packed
 * integer key of Eq. 14 on the 32-bit float mass, block index complemented so
 * that equal masses resolve to the lower block) and the shortest prefix of that
 * order whose cumulative mass reaches top_p of the sequence's total is kept
 * whole; the first A and the last n tokens of a sequence are kept regardless
 * ("Top-p Token Selection"; top-p and expansion kernels of the kernel-design
 * paragraph).  Kept counts depend on the data: kept_idx must have room for
 * total_tokens entries, and the totals stay on the device --
 * new_cu_seqlens_dev[R] is the number of entries written.
 *   Decisions are taken in fixed arithmetic: block mass = double sum of the
 *   float scores in index order, rounded to float; running sum over the ordered
 *   blocks in double, in that order; threshold (double)top_p * total.
 *   top_p_dev/host [R] each, same values, in (0,1]
 *   workspace      device scratch from uniprefill_plan (its first part is used)
 *   UP_ERR_UNSUPPORTED if a sequence has more than 4096 blocks */
int uniprefill_select_top_p(const up_params* p, const float* scores,
                            const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host,
                            const float* top_p_dev, const float* top_p_host, int32_t* kept_idx,
                            int32_t* new_cu_seqlens_dev, void* workspace, size_t workspace_bytes,
                            void* stream);

/* uniprefill_compact with the row count on the device (Eq. 7 after a selection
 * whose size is data-dependent): rows t < total_kept_dev[0] are gathered;
 * capacity (<= total_tokens) bounds the launch and the output buffers. */
int uniprefill_compact_counted(const up_params* p, const void* hidden, const int32_t* pos,
                               const int32_t* kept_idx, const int32_t* total_kept_dev,
                               int64_t capacity, void* hidden_out, int32_t* pos_out, void* stream);

/* score -> block-level top-p selection -> compact in one call, no host
 * synchronisation.  hidden_out, pos_out and kept_idx need room for
 * total_tokens rows / entries; scores (device float [T]) is required. */
int uniprefill_fused_top_p(const up_params* p, const void* q, const void* k, const void* hidden,
                           const int32_t* pos, const int32_t* cu_seqlens_dev,
                           const int32_t* cu_seqlens_host, const float* top_p_dev,
                           const float* top_p_host, void* hidden_out, int32_t* pos_out,
                           int32_t* kept_idx, int32_t* new_cu_seqlens_dev, float* scores,
                           void* workspace, size_t workspace_bytes, void* stream);

/* Index map of two successive drops ("Sparsity Propagation Across All Layers":
 * a token dropped at one layer stays out of all later layers, so retained sets
 * are nested).  outer_idx [n_outer] maps the rows of a compacted stream to packed
 * rows of the original batch; inner_idx selects rows of that compacted stream
 * (a second selection run on it); composed_idx[t] = outer_idx[inner_idx[t]] maps
 * the twice-compacted stream to the original batch, so that one
 * uniprefill_scatter through composed_idx reconstitutes the full sequence (Eq. 8)
 * from the innermost stream.  All three device int32.  Entries t < n_inner are
 * written, or t < n_inner_dev[0] when n_inner_dev is given (then n_inner is the
 * capacity); inner_idx values must lie in [0, n_outer). */
int uniprefill_compose_index(const int32_t* outer_idx, int64_t n_outer, const int32_t* inner_idx,
                             const int32_t* n_inner_dev, int64_t n_inner, int32_t* composed_idx,
                             void* stream);

/* Physical KV-cache slots of the retained tokens after a drop (Eq. 16 of "vLLM
 * scheduler integration"): for token t of the compacted stream, in sequence r
 * (new_cu_seqlens_dev[r] <= t < new_cu_seqlens_dev[r+1]) at logical position
 * p = pos_kept[t],
 *     slots[t] = block_table[r * block_table_stride + p / kv_block_size] * kv_block_size
 *                + p % kv_block_size.
 * All device pointers; slots is int64.  t runs to new_cu_seqlens_dev[num_seqs]
 * (read on the device), at most capacity.  Positions must address existing
 * entries of the sequence's block-table row. */
int uniprefill_slot_mapping(const int32_t* pos_kept, const int32_t* new_cu_seqlens_dev, int32_t num_seqs,
                            const int32_t* block_table, int64_t block_table_stride, int32_t kv_block_size,
                            int64_t capacity, int64_t* slots, void* stream);

/* The kernels behind uniprefill_fused, in stream order.  Measurement aid: a
 * caller that wants to time one kernel enqueues the phases one by one. */
enum {
  UP_PHASE_PLAN = 1,                 /* new_cu_seqlens_dev (a kernel of its own when asked for alone;
                                        together with UP_PHASE_MERGE_STATS it rides in that kernel) */
  UP_PHASE_ROW_STATS = 2,            /* pass 1 of the two-pass softmax: row statistics per key block */
  UP_PHASE_MERGE_STATS = 4,          /* merge of the per-block statistics */
  UP_PHASE_SWEEP_SELECT = 8,         /* pass 2 (normalised weights summed per token) with the
                                        block-local top-k: scores, kept_idx */
  UP_PHASE_GATHER = 16,              /* gather of the kept rows and position ids */
  UP_PHASE_ALL = 31,
  UP_PHASE_GATHER_IN_SELECT = 32     /* with UP_PHASE_SWEEP_SELECT: the kernel that selects also copies its
                                        kept rows (no gather launch).  Measured slower than the launch of
                                        its own on every workload; not part of UP_PHASE_ALL, kept so that
                                        the comparison can be repeated */
};


/* uniprefill_fused restricted to the phases in phase_mask (same arguments,
 * same checks; UP_ERR_RANGE for unknown bits).  A phase reads what the earlier
 * phases left in the workspace and outputs, so the phases of one call sequence
 * must be enqueued in order on one stream with unchanged arguments; enqueuing
 * all five one by one is exactly uniprefill_fused. */
int uniprefill_fused_phases(const up_params* p, const void* q, const void* k, const void* hidden,
                            const int32_t* pos, const int32_t* cu_seqlens_dev,
                            const int32_t* cu_seqlens_host, const float* keep_ratio_dev,
                            const float* keep_ratio_host, void* hidden_out, int32_t* pos_out,
                            int32_t* kept_idx, int32_t* new_cu_seqlens_dev, float* scores_out,
                            void* workspace, size_t workspace_bytes, int phase_mask, void* stream);

/* The token keep mask M in {0,1}^T that the index list stands for (Top-p Token
 * Selection; what the expansion kernel of the kernel-design paragraph leaves):
 * mask_out[t] = 1 if packed row t is among kept_idx[0 .. n), else 0, for every
 * t < total_tokens; n = capacity, or total_kept_dev[0] when that device pointer
 * is given and smaller.  kept_idx must be ascending (as every selection entry
 * point writes it); mask_out is a device array of total_tokens bytes, all of
 * which are written.  capacity > total_tokens: UP_ERR_RANGE. */
int uniprefill_keep_mask(const int32_t* kept_idx, int64_t capacity, const int32_t* total_kept_dev,
                         int64_t total_tokens, uint8_t* mask_out, void* stream);

/* KV length every layer sees during decode (vLLM scheduler integration, Eq. 17):
 * seqused_out[l][r] = s + (kv_len[r] - orig_len[r]) for l < num_layers, r < num_seqs,
 * where s is the length request r retained at the last drop event at a layer
 * strictly before l, or orig_len[r] when there is none.  drop_layers_host holds the
 * layers of the num_drops drop events, strictly ascending and >= 0 (UP_ERR_RANGE
 * otherwise; more than 64 events: UP_ERR_UNSUPPORTED); retained_dev is the drop
 * history [num_drops][num_seqs] on the device (row k = the retained lengths after
 * event k, i.e. the differences of that drop's new_cu_seqlens); kv_len_dev and
 * orig_len_dev are int32 [num_seqs] on the device; seqused_out is int32
 * [num_layers][num_seqs] on the device.  num_layers <= 65535. */
int uniprefill_seqused(const int32_t* drop_layers_host, int32_t num_drops, const int32_t* retained_dev,
                       const int32_t* kv_len_dev, const int32_t* orig_len_dev, int32_t num_seqs,
                       int32_t num_layers, int32_t* seqused_out, void* stream);

/* Compaction of one per-token column (Sparsity Propagation, Eq. 7, for what travels
 * with the hidden states besides the int32 position ids that uniprefill_compact
 * takes: 64-bit position ids, token ids, ...): column_out[t] = column[kept_idx[t]]
 * for t < capacity, and t < total_kept_dev[0] when that device pointer is given
 * (the count of a top-p selection).  column is a device array of total_tokens
 * elements of elem_bytes = 4 or 8 bytes (else UP_ERR_UNSUPPORTED), aligned to its
 * element size (UP_ERR_ALIGN); column_out has room for capacity elements. */
int uniprefill_compact_column(const void* column, int32_t elem_bytes, const int32_t* kept_idx,
                              int64_t capacity, const int32_t* total_kept_dev, void* column_out,
                              void* stream);

/* ---- Tokens that follow earlier context (chunked prefill) -----------------
 *
 * The paper scores whole prompts (Token Importance Estimation, Eq. 2-3) and runs
 * under continuous batching (Fused Kernel and vLLM Integration), where a long
 * prompt arrives in chunks and the keys of its earlier chunks are cached.  These
 * variants take the keys of every sequence as its earlier tokens' keys followed
 * by the keys of its own tokens: k is [Tk, num_kv_heads, head_dim] packed by
 * cu_seqlens_k (int32 [R+1], device and host copies like cu_seqlens;
 * cu_seqlens_k[0] = 0 and every sequence has at least as many keys as tokens,
 * else UP_ERR_SHAPE), while q, hidden, pos, scores and every output stay packed
 * by cu_seqlens over the T = total_tokens tokens.  With P_r earlier tokens, token
 * i of sequence r sits at position P_r + i: window row j (one of the last
 * min(n_obs, N_r) tokens) sees keys 0 .. P_r + j, its softmax runs over all of
 * them, and token i receives the mean weight of key P_r + i -- the scores the
 * tokens would get if the sequence so far were scored in one piece.  Selection
 * blocks start at the sequence's first token; a token is a sink when its position
 * P_r + i is below n_sink.  Everything else (errors, ownership, streams,
 * workspace from the matching plan call) is as for the plain entry points; with
 * cu_seqlens_k equal to cu_seqlens the results are those of the plain ones. */
int uniprefill_plan_chunked(const up_params* p, const int32_t* cu_seqlens_host,
                            const int32_t* cu_seqlens_k_host, const float* keep_ratio_host,
                            int32_t* new_cu_seqlens_host, int64_t* total_kept,
                            size_t* workspace_bytes);
int uniprefill_score_chunked(const up_params* p, const void* q, const void* k,
                             const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host,
                             const int32_t* cu_seqlens_k_dev, const int32_t* cu_seqlens_k_host,
                             float* scores_out, void* workspace, size_t workspace_bytes,
                             void* stream);
int uniprefill_select_chunked(const up_params* p, const float* scores,
                              const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host,
                              const int32_t* cu_seqlens_k_dev, const int32_t* cu_seqlens_k_host,
                              const float* keep_ratio_dev, const float* keep_ratio_host,
                              int32_t* kept_idx, int32_t* new_cu_seqlens_dev, void* stream);
int uniprefill_fused_chunked(const up_params* p, const void* q, const void* k, const void* hidden,
                             const int32_t* pos, const int32_t* cu_seqlens_dev,
                             const int32_t* cu_seqlens_host, const int32_t* cu_seqlens_k_dev,
                             const int32_t* cu_seqlens_k_host, const float* keep_ratio_dev,
                             const float* keep_ratio_host, void* hidden_out, int32_t* pos_out,
                             int32_t* kept_idx, int32_t* new_cu_seqlens_dev, float* scores_out,
                             void* workspace, size_t workspace_bytes, void* stream);

/* The same with the keys in a paged KV cache (vLLM scheduler integration; the
 * indexing of Eq. 16): key i of sequence r is row
 *     block_table[r * block_table_stride + i / kv_block_size] * kv_block_size + i % kv_block_size
 * of k_cache, a device array of rows [num_kv_heads, head_dim] with k_row_stride
 * elements between rows.  cu_seqlens_k still gives the number of keys per
 * sequence (earlier tokens + own tokens) and sizes the workspace through
 * uniprefill_plan_chunked; block_table is int32 on the device, one row of
 * block_table_stride entries per sequence, which must hold at least
 * ceil(keys / kv_block_size) entries (UP_ERR_SHAPE otherwise; kv_block_size < 1:
 * UP_ERR_RANGE).  Its entries must name existing blocks of the cache: they are
 * read on the device and cannot be checked. */
int uniprefill_score_paged(const up_params* p, const void* q, const void* k_cache,
                           const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host,
                           const int32_t* cu_seqlens_k_dev, const int32_t* cu_seqlens_k_host,
                           const int32_t* block_table, int64_t block_table_stride, int32_t kv_block_size,
                           float* scores_out, void* workspace, size_t workspace_bytes, void* stream);
int uniprefill_fused_paged(const up_params* p, const void* q, const void* k_cache, const void* hidden,
                           const int32_t* pos, const int32_t* cu_seqlens_dev,
                           const int32_t* cu_seqlens_host, const int32_t* cu_seqlens_k_dev,
                           const int32_t* cu_seqlens_k_host, const int32_t* block_table,
                           int64_t block_table_stride, int32_t kv_block_size, const float* keep_ratio_dev,
                           const float* keep_ratio_host, void* hidden_out, int32_t* pos_out,
                           int32_t* kept_idx, int32_t* new_cu_seqlens_dev, float* scores_out,
                           void* workspace, size_t workspace_bytes, void* stream);

/* The fused call when the attention layer's own kernel has already normalised
 * the rows: lse[h * lse_row_stride + t] (device, float) is the natural logarithm
 * of the sum of exp(scale * <q_t, k_i>) over the keys token t sees in query head h
 * -- the log-sum-exp that attention kernels return next to their output, laid out
 * [num_q_heads, total_tokens] with lse_row_stride >= total_tokens elements between
 * heads (UP_ERR_SHAPE otherwise).  Only the entries of the window rows are read.
 * The first of the two passes over Q.K^T (Eq. 2's normaliser) and the merge are
 * then not needed: a small conversion kernel (which also does the plan), the
 * second pass with the selection, and the gather.  The weights are
 * exp(scale * <q_j, k_i> - lse) evaluated to float rounding, so with the exact
 * normalisers the results are those of uniprefill_fused.
 * Keys: cu_seqlens_k_dev/_host both NULL (the tokens' own keys), or both given
 * (earlier context, as for uniprefill_fused_chunked) and then optionally a block
 * table (paged cache, as for uniprefill_fused_paged; block_table NULL = packed).
 * Workspace from uniprefill_plan, or uniprefill_plan_chunked when cu_seqlens_k is
 * given. */
int uniprefill_fused_lse(const up_params* p, const void* q, const void* k, const float* lse,
                         int64_t lse_row_stride, const void* hidden, const int32_t* pos,
                         const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host,
                         const int32_t* cu_seqlens_k_dev, const int32_t* cu_seqlens_k_host,
                         const int32_t* block_table, int64_t block_table_stride, int32_t kv_block_size,
                         const float* keep_ratio_dev, const float* keep_ratio_host, void* hidden_out,
                         int32_t* pos_out, int32_t* kept_idx, int32_t* new_cu_seqlens_dev,
                         float* scores_out, void* workspace, size_t workspace_bytes, void* stream);

/* The same source of normalisers for the scores alone, and for the paper's top-p
 * rule end to end (uniprefill_score / uniprefill_fused_top_p with lse and the
 * optional key-side arguments of uniprefill_fused_lse). */
int uniprefill_score_lse(const up_params* p, const void* q, const void* k, const float* lse,
                         int64_t lse_row_stride, const int32_t* cu_seqlens_dev,
                         const int32_t* cu_seqlens_host, const int32_t* cu_seqlens_k_dev,
                         const int32_t* cu_seqlens_k_host, const int32_t* block_table,
                         int64_t block_table_stride, int32_t kv_block_size, float* scores_out,
                         void* workspace, size_t workspace_bytes, void* stream);
int uniprefill_fused_top_p_lse(const up_params* p, const void* q, const void* k, const float* lse,
                               int64_t lse_row_stride, const void* hidden, const int32_t* pos,
                               const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host,
                               const int32_t* cu_seqlens_k_dev, const int32_t* cu_seqlens_k_host,
                               const int32_t* block_table, int64_t block_table_stride,
                               int32_t kv_block_size, const float* top_p_dev, const float* top_p_host,
                               void* hidden_out, int32_t* pos_out, int32_t* kept_idx,
                               int32_t* new_cu_seqlens_dev, float* scores, void* workspace,
                               size_t workspace_bytes, void* stream);

/* One tensor-parallel rank's share (section "Tensor parallelism", Eq. 15).  A rank
 * holds num_q_heads / num_kv_heads of the model's heads (up_params describes the
 * rank's share; q and k may be views into wider rows through the row strides) and
 * leaves, per token, the attention weights summed over the window rows and over
 * its heads -- not divided, not floored -- as doubles: colsum_out [T], device,
 * 8-byte aligned.  cu_seqlens_k_dev/_host: both NULL, or the key-side offsets of
 * tokens after earlier context.  Workspace from uniprefill_plan(_chunked) with
 * the rank's up_params.
 * uniprefill_scores_from_partials then forms the scores from the ranks' sums
 * once they sit side by side on one device (partials[p * part_stride + t], after
 * an all-gather): added in rank order, divided by the window rows min(n_obs, N_r)
 * and by the query heads of all ranks, means below 2^-64 written as +0 -- what
 * uniprefill_score writes on one device, so that uniprefill_select (or the
 * top-p rule) takes the same decision on every rank. */
int uniprefill_score_partial(const up_params* p, const void* q, const void* k,
                             const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host,
                             const int32_t* cu_seqlens_k_dev, const int32_t* cu_seqlens_k_host,
                             double* colsum_out, void* workspace, size_t workspace_bytes, void* stream);
int uniprefill_scores_from_partials(const double* partials, int32_t num_parts, int64_t part_stride,
                                    const int32_t* cu_seqlens_dev, int32_t num_seqs, int32_t total_tokens,
                                    int32_t n_obs, int32_t total_q_heads, float* scores_out, void* stream);

/* The paper's block-level top-p rule (uniprefill_select_top_p, uniprefill_fused_top_p) for
 * tokens that follow earlier context: the sinks are those that fall inside the
 * tokens (position P_r + i below n_sink), and the threshold is p times the mass
 * of the tokens' own blocks.  The fused variant takes the keys packed by
 * cu_seqlens_k (block_table NULL) or in a paged cache (block_table given, as
 * for uniprefill_fused_paged).  Workspace from uniprefill_plan_chunked. */
int uniprefill_select_top_p_chunked(const up_params* p, const float* scores,
                                    const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host,
                                    const int32_t* cu_seqlens_k_dev, const int32_t* cu_seqlens_k_host,
                                    const float* top_p_dev, const float* top_p_host, int32_t* kept_idx,
                                    int32_t* new_cu_seqlens_dev, void* workspace,
                                    size_t workspace_bytes, void* stream);
int uniprefill_fused_top_p_chunked(const up_params* p, const void* q, const void* k, const void* hidden,
                                   const int32_t* pos, const int32_t* cu_seqlens_dev,
                                   const int32_t* cu_seqlens_host, const int32_t* cu_seqlens_k_dev,
                                   const int32_t* cu_seqlens_k_host, const int32_t* block_table,
                                   int64_t block_table_stride, int32_t kv_block_size,
                                   const float* top_p_dev, const float* top_p_host, void* hidden_out,
                                   int32_t* pos_out, int32_t* kept_idx, int32_t* new_cu_seqlens_dev,
                                   float* scores, void* workspace, size_t workspace_bytes, void* stream);

/* Static, never NULL. */
const char* uniprefill_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* UNIPREFILL_H */
