// Launchers of the gfx950 kernels behind the C ABI (internal header).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace up {

// Static description of one call, derived on the host from up_params.
struct Problem {
  int R, T;
  int G, n_obs, n_sink;
  int Hq, Hkv, Gq;            // Gq = query heads per kv head
  int d;
  long long q_stride, k_stride, h_stride;  // elements
  int hidden_elem_bytes;      // 2 (bf16) or 4 (f32)
  int qk_is_f32;
  float scale;                // softmax scale (resolved, > 0)
  // scoring launch shape
  int CK;                     // keys per work-group chunk (multiple of 64)
  int tpw;                    // 16-row query tiles per wave
  int n_slab;                 // row slabs per kv head
  int chunk_slots;            // T / CK + R
  int row_slots;              // min(T, R * n_obs)
};

// Workspace carve-up (byte offsets, each 256-aligned).
struct Workspace {
  size_t stat_part_off, stat_fin_off, part_o_off, total;
};
Workspace workspace_layout(const Problem& pb);

// --- copies (Eq. 7 / Eq. 8)
hipError_t launch_compact(const Problem& pb, const void* hidden, const int32_t* pos,
                          const int32_t* kept_idx, long long total_kept, void* hidden_out,
                          int32_t* pos_out, hipStream_t s);
hipError_t launch_scatter(const Problem& pb, const void* hidden_compact, const int32_t* kept_idx,
                          long long total_kept, void* hidden_full, hipStream_t s);

// --- selection
hipError_t launch_plan(const Problem& pb, const int32_t* cu, const float* ratio, int32_t* new_cu,
                       hipStream_t s);
// scores != nullptr: select on given scores.  Otherwise sum `parts` partial score
// planes [n_parts][T] (double), normalise, floor, optionally write scores_out.
// hidden != nullptr: also gather the kept rows (fused select+compact).
hipError_t launch_select(const Problem& pb, const float* scores, const double* parts, int n_parts,
                         const int32_t* cu, const float* ratio, const int32_t* new_cu,
                         int32_t* kept_idx, float* scores_out, const void* hidden,
                         const int32_t* pos, void* hidden_out, int32_t* pos_out, hipStream_t s);

// --- scoring (Eq. 2-3)
// phase 1: row statistics per key chunk; 2: merge of the chunk statistics; 3: normalised
// column sums (partial score planes in the workspace).
hipError_t launch_score_phase(const Problem& pb, int phase, const void* q, const void* k,
                              const int32_t* cu, void* workspace, hipStream_t s);
hipError_t launch_score_passes(const Problem& pb, const void* q, const void* k, const int32_t* cu,
                               void* workspace, hipStream_t s);
hipError_t launch_finalise_scores(const Problem& pb, const int32_t* cu, const void* workspace,
                                  float* scores_out, hipStream_t s);

}  // namespace up
