"""hyb(c,k) composable-format SpMM for MI355X (gfx950): Python binding of libsptir.so."""
from .binding import (ARRAY_DTYPES, ARRAY_IDS, EXPORTED_SYMBOLS, LIB_PATH, Hyb, Rgms, SddmmPlan, SptirError, load_library,
                      sptir_default_bucket_log2, sptir_gather_offsets_fit_32, sptir_hyb_array, sptir_hyb_build, sptir_hyb_build_ex, sptir_hyb_destroy, sptir_hyb_search,
                      sptir_hyb_info, sptir_launch_plan, sptir_rgms, sptir_rgms_build, sptir_rgms_destroy, sptir_rgms_info,
                      sptir_set_allocator, sptir_release_scratch, sptir_sddmm, sptir_sddmm_csr, sptir_sddmm_default_col_parts, sptir_sddmm_plan_build, sptir_sddmm_plan_destroy,
                      sptir_sddmm_plan_info, sptir_roof_fma, sptir_roof_gather, sptir_spmm, sptir_spmm_csr, sptir_spmm_noalloc, sptir_spmm_timed, sptir_status_string)
