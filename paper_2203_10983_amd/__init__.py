"""MI355X-native BNS-GCN partition step: HIP kernels behind a C ABI plus a thin binding."""
from .binding import (BnsError, Context, adam_update, sample_boundary_noalloc, probe_gather, probe_mfma, NOALLOC_MAX_HALO, EXPORTED, LIB_PATH, PHASES, load_library,  # noqa: F401
                      VIEW_A, VIEW_COL_IDX, VIEW_DZ, VIEW_H, VIEW_KEPT_IDS, VIEW_N_KEPT, VIEW_NNZ,
                      VIEW_REMAP, VIEW_ROW_PTR, VIEW_T_COL_IDX, VIEW_T_ROW_PTR,
                      LAYER_TWO_KERNELS, LAYER_ONE_KERNEL, LAYER_UPDATE_FIRST)
