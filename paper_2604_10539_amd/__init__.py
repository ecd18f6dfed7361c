"""MI355X-native IceCache hot path: HIP kernels behind a C ABI (include/icecache.h) and a thin
ctypes binding.  Importing the package does not load the library; the first call does."""
from .binding import (ICE_GEOMETRY_RAW, ICE_GEOMETRY_TRANSFORMED, ICE_STAGE_ASSIGN, ICE_STAGE_MEANS,  # noqa: F401
                      ICE_STAGE_PAGINATE, ICE_STAGE_SORT, IceConfig, IceError, IceIndex, IceIndexView, ice_attend,
                      ice_attend_noalloc, ice_attend_resident, ice_attend_tokens, ice_build_index, ice_create,
                      ice_debug_assign, ice_debug_peak_mfma, ice_debug_peak_read, ice_debug_rerun_stage,
                      ice_debug_select_fault, ice_destroy, ice_export_geometry, ice_export_index, ice_import_index,
                      ice_insert, ice_insert_batch, ice_last_error, ice_select, ice_select_attend,
                      ice_select_attend_resident, ice_select_hier, ice_select_hier3, ice_build_top_level, ice_export_top_level, ice_selected_tokens, ice_set_geometry,
                      ice_workspace_bytes, lib, make_config)
