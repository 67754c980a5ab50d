// Stand-alone kernels of the selection step: the device-side plan (kept totals
// and their prefix per sequence) and block-local top-k on given scores.
#include "up_common.h"
#include "up_kernels.h"
#include "up_select.h"

namespace up {

// The plan as a kernel of its own (one work-group).
__global__ __launch_bounds__(1024) void k_plan(const int32_t* __restrict__ cu, const int32_t* __restrict__ cu_k,
                                               const float* __restrict__ ratio, int R, int G,
                                               int n_obs, int n_sink, int32_t* __restrict__ new_cu) {
  __shared__ int wave_tot[16];
  __shared__ int carry;
  plan_scan<1024>(cu, cu_k, ratio, R, G, n_obs, n_sink, new_cu, wave_tot, &carry);
}

// One work-group per selection block.
__global__ __launch_bounds__(256) void k_select(SelectArgs a) {
  __shared__ SelectSmem sm;
  const int slot = blockIdx.x;
  const int r = locate_slot(a.cu, a.R, a.G, slot);
  const int c0 = a.cu[r];
  const int N = a.cu[r + 1] - c0;
  const int g = slot - slot_base(c0, r, a.G);
  if (g * a.G >= N) return;   // slack slot (also every slot of an empty sequence)
  select_block(a, sm, r, c0, N, g, a.scores + c0 + g * a.G);
}

hipError_t launch_plan(const Problem& pb, const int32_t* cu, const int32_t* cu_k, const float* ratio,
                       int32_t* new_cu, hipStream_t s) {
  hipLaunchKernelGGL(k_plan, dim3(1), dim3(1024), 0, s, cu, cu_k, ratio, pb.R, pb.G, pb.n_obs, pb.n_sink,
                     new_cu);
  return hipGetLastError();
}

hipError_t launch_select(const Problem& pb, const SelectArgs& a, hipStream_t s) {
  if (pb.T == 0) return hipSuccess;
  const unsigned grid = (unsigned)(pb.T / pb.G + pb.R);
  hipLaunchKernelGGL(k_select, dim3(grid), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace up
