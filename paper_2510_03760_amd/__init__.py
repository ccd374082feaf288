"""MI355X-native fitness-and-validity evaluation step for LLM-driven kernel evolution
(EvoEngineer, arXiv 2510.03760): a C-ABI HIP library (include/evo.h) and a thin
binding with the same names.  Importing this package loads the library; it raises if
the library has not been built (python -m paper_2510_03760_amd.build)."""
from .binding import (  # noqa: F401
    EVO_BF16, EVO_F16, EVO_F32, EVO_F64, EVO_I32, EVO_I64, EVO_REDUCE_MEAN, EVO_REDUCE_MEDIAN, EvoError, EvoStats, EvoPopSummary, EvoSegment, STATS_DTYPE,
    SUMMARY_DTYPE, Checker, evo_check_batch, evo_check_batch_static, evo_check_cases, evo_check_create,
    evo_check_destroy, evo_check_segmented, evo_check_set_tolerance, evo_check_set_tolerance_class, evo_evaluate, evo_evaluate_segmented, evo_fitness, evo_fitness_ex, evo_select_elite, evo_select_elite_diverse, evo_time_candidates, evo_strerror, lib, lib_path,
)
