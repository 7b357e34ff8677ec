// Launch functions of the bf16 MFMA kernels (defined in mfma_fwd.hip / mfma_bwd.hip), called by mfma_path.hip.
#pragma once
#include "mfma_common.h"

size_t mfma_cmp_lds_bytes(int hs, int s_max);
int mfma_forward_kernels(const MfmaView &v, int D, const void *q, const void *gates, void *out, float *lse,
                         int32_t *idx, void *out_branch, hipStream_t s);
