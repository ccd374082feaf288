// One instantiation of the check kernel: compiled once per element-type set with
// -DEVO_INST_DTS=<bit mask of 1 << evo_dtype> (see build.py).  A launch whose segments all
// have one element type runs the kernel that holds only that type's code, so that its
// register allocation is not the worst case over all types; mixed launches run the one
// instantiated for all of them.
#include "evo_check_device.h"

#ifndef EVO_INST_DTS
#error "compile with -DEVO_INST_DTS=<element-type set>"
#endif

namespace evo {

template hipError_t launch_check_for<EVO_INST_DTS>(const SegDesc *, const uint64_t *, uint32_t, uint32_t,
                                                   uint32_t, Partial *, uint32_t *,
                                                   evo_stats *, hipStream_t);
template hipError_t launch_check_inline_for<EVO_INST_DTS>(const InlineTable &, uint32_t, uint32_t,
                                                          uint32_t, Partial *, uint32_t *,
                                                          evo_stats *, hipStream_t);

template hipError_t launch_evaluate_for<EVO_INST_DTS>(const InlineTable &, uint32_t, uint32_t,
                                                      uint32_t, Partial *, uint32_t *, evo_stats *,
                                                      const FitLaunch &, hipStream_t);

}  // namespace evo
