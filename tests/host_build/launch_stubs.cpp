// The kernel launchers of the library, as no-ops: the sanitizer build of the host side never
// launches anything (every test it runs ends in an argument error or an empty batch).
#include "up_common.h"
#include "up_kernels.h"
#include "up_select.h"

namespace up {

hipError_t launch_compact(const Problem&, const void*, const int32_t*, const int32_t*, long long, void*, int32_t*, hipStream_t) { return hipSuccess; }
hipError_t launch_scatter(const Problem&, const void*, const int32_t*, long long, void*, hipStream_t) { return hipSuccess; }
hipError_t launch_compose(const int32_t*, const int32_t*, long long, const int32_t*, int32_t*, hipStream_t) { return hipSuccess; }
hipError_t launch_column(const void*, int, const int32_t*, long long, const int32_t*, void*, hipStream_t) { return hipSuccess; }
hipError_t launch_keep_mask(const int32_t*, long long, const int32_t*, long long, uint8_t*, hipStream_t) { return hipSuccess; }
hipError_t launch_seqused(const DropLayers&, const int32_t*, const int32_t*, const int32_t*, int, int, int32_t*, hipStream_t) { return hipSuccess; }
hipError_t launch_slot_mapping(const int32_t*, const int32_t*, int, const int32_t*, long long, int, long long, int64_t*, hipStream_t) { return hipSuccess; }
hipError_t launch_plan(const Problem&, const int32_t*, const int32_t*, const float*, int32_t*, hipStream_t) { return hipSuccess; }
hipError_t launch_select(const Problem&, const SelectArgs&, hipStream_t) { return hipSuccess; }
hipError_t launch_top_p(const Problem&, const float*, const int32_t*, const int32_t*, const float*, int32_t*, int32_t*, void*, int, hipStream_t) { return hipSuccess; }
hipError_t launch_compact_counted(const Problem&, const void*, const int32_t*, const int32_t*, const int32_t*, long long, void*, int32_t*, hipStream_t) { return hipSuccess; }
hipError_t launch_row_stats(const Problem&, const void*, const void*, const int32_t*, const int32_t*, const PagedKeys*, void*, hipStream_t, bool) { return hipSuccess; }
hipError_t launch_merge_stats(const Problem&, const int32_t*, const int32_t*, void*, const float*, int32_t*, hipStream_t) { return hipSuccess; }
hipError_t launch_lse_stats(const Problem&, const int32_t*, const int32_t*, const float*, long long, void*, const float*, int32_t*, hipStream_t) { return hipSuccess; }
hipError_t launch_column_sums(const Problem&, const void*, const void*, const int32_t*, const int32_t*, const PagedKeys*, void*, float*, const SelectArgs*, hipStream_t, double*, bool, const GatherArgs*) { return hipSuccess; }
hipError_t launch_scores_from_partials(const double*, int, long long, const int32_t*, int, int, int, int, float*, hipStream_t) { return hipSuccess; }

}  // namespace up
