// Matrix-core kernel family (placeholder until the MFMA kernels land).
#include "pv_kernels_common.h"

int pv_mat_run_block(pv_cache *, hipStream_t) { pv_set_error("matrix path not built"); return PV_EINVAL; }
int pv_mat_repack(const pv_model *, const pv_tensor_ref &, int64_t, int64_t, hipStream_t) { pv_set_error("matrix path not built"); return PV_EINVAL; }
size_t pv_mat_part_floats(const pv_model *, int) { return 0; }
