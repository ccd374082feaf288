// Picks the instantiation of the check kernel for the element types of a launch.
#include "evo_internal.h"

namespace evo {

hipError_t launch_check(uint32_t dtype_set, const SegDesc *d_descs, const uint64_t *d_ptrs,
                        uint32_t S, uint32_t total_jobs, uint32_t n_first,
                        Partial *partials, uint32_t *tickets, evo_stats *stats, hipStream_t stream) {
#define EVO_LAUNCH(DTS_)                                                                          \
    return launch_check_for<DTS_>(d_descs, d_ptrs, S, total_jobs, n_first, partials,  \
                                  tickets, stats, stream)
    switch (dtype_set) {
        case 1u << EVO_F32: EVO_LAUNCH(1u << EVO_F32);
        case 1u << EVO_BF16: EVO_LAUNCH(1u << EVO_BF16);
        case 1u << EVO_F16: EVO_LAUNCH(1u << EVO_F16);
        case 1u << EVO_F64: EVO_LAUNCH(1u << EVO_F64);
        case 1u << EVO_I32: EVO_LAUNCH(1u << EVO_I32);
        case 1u << EVO_I64: EVO_LAUNCH(1u << EVO_I64);
        default: EVO_LAUNCH(kAllTypes);
    }
#undef EVO_LAUNCH
}

hipError_t launch_check_inline(uint32_t dtype_set, const InlineTable &tab, uint32_t S,
                               uint32_t total_jobs, uint32_t n_first,
                               Partial *partials, uint32_t *tickets, evo_stats *stats,
                               hipStream_t stream) {
#define EVO_LAUNCH(DTS_)                                                                          \
    return launch_check_inline_for<DTS_>(tab, S, total_jobs, n_first, partials,       \
                                         tickets, stats, stream)
    switch (dtype_set) {
        case 1u << EVO_F32: EVO_LAUNCH(1u << EVO_F32);
        case 1u << EVO_BF16: EVO_LAUNCH(1u << EVO_BF16);
        case 1u << EVO_F16: EVO_LAUNCH(1u << EVO_F16);
        case 1u << EVO_F64: EVO_LAUNCH(1u << EVO_F64);
        case 1u << EVO_I32: EVO_LAUNCH(1u << EVO_I32);
        case 1u << EVO_I64: EVO_LAUNCH(1u << EVO_I64);
        default: EVO_LAUNCH(kAllTypes);
    }
#undef EVO_LAUNCH
}

hipError_t launch_evaluate(uint32_t dtype_set, const InlineTable &tab, uint32_t S, uint32_t total_jobs,
                           uint32_t n_first, Partial *partials,
                           uint32_t *tickets, evo_stats *stats, const FitLaunch &fit,
                           hipStream_t stream) {
#define EVO_LAUNCH(DTS_)                                                                          \
    return launch_evaluate_for<DTS_>(tab, S, total_jobs, n_first, partials, tickets,  \
                                     stats, fit, stream)
    switch (dtype_set) {
        case 1u << EVO_F32: EVO_LAUNCH(1u << EVO_F32);
        case 1u << EVO_BF16: EVO_LAUNCH(1u << EVO_BF16);
        case 1u << EVO_F16: EVO_LAUNCH(1u << EVO_F16);
        case 1u << EVO_F64: EVO_LAUNCH(1u << EVO_F64);
        case 1u << EVO_I32: EVO_LAUNCH(1u << EVO_I32);
        case 1u << EVO_I64: EVO_LAUNCH(1u << EVO_I64);
        default: EVO_LAUNCH(kAllTypes);
    }
#undef EVO_LAUNCH
}

}  // namespace evo
