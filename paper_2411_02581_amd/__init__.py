"""MI355X-native tunable-radix non-uniform all-to-all (TuNA / TuNA_l^g) for virtual ranks in one
GPU's HBM.  The product is libtuna.so (hand-written HIP for gfx950 behind the C ABI of
include/tuna.h); this package is its thin Python binding."""
from .binding import *  # noqa: F401,F403
from .binding import (EXPORTS, tuna_alltoallv_init, tuna_plan_free, tuna_start, library_path, load, tuna_alltoallv, tuna_alltoallv_hier, tuna_get_stats,
                      tuna_plan_info, tuna_plan_info_t, tuna_plan_phase, tuna_plan_phase_device, tuna_plan_phase_sources, tuna_plain_copy, tuna_phase_stats_t, tuna_release, tuna_select, tuna_predict_ms, tuna_calibrate, tuna_model_constants, tuna_set_option,
                      tuna_set_workspace, tuna_stats_t, tuna_strerror, tuna_t_index, tuna_version,
                      tuna_workspace_bytes)
from .build import build_library  # noqa: F401
