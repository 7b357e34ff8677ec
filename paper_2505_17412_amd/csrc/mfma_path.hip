// bf16 MFMA path (placeholder until the kernels land): reports "unsupported" so every problem takes the generic path.
#include "ssa_internal.h"
bool mfma_supported(const ssa_ctx &) { return false; }
size_t mfma_forward_workspace(const ssa_ctx &) { return 0; }
size_t mfma_backward_workspace(const ssa_ctx &) { return 0; }
int mfma_forward(const ssa_ctx &, const void *, const void *, const void *, const void *, void *, float *, int32_t *, void *,
                 void *, size_t) { return SSA_ERR_UNSUPPORTED; }
int mfma_backward(const ssa_ctx &, const void *, const void *, const void *, const void *, const void *, const float *,
                  const int32_t *, const void *, void *, void *, void *, void *, void *, size_t) { return SSA_ERR_UNSUPPORTED; }
