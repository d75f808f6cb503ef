// C ABI: build entry points (placeholder until the build kernels land).
#include "../../include/cagra_hip.h"

extern "C" {
int cagra_exact_search(const float *, int64_t, int32_t, int64_t, cagra_metric, const float *, int64_t, int64_t,
                       int32_t, int32_t, int64_t, uint32_t *, float *, void *, size_t, void *) { return CAGRA_ERR_LAUNCH; }
size_t cagra_exact_search_workspace_bytes(int64_t, int64_t, int32_t) { return 256; }
int cagra_build(const float *, int64_t, int32_t, int64_t, cagra_metric, int32_t, int32_t, uint32_t *, void *, size_t, void *) { return CAGRA_ERR_LAUNCH; }
size_t cagra_build_workspace_bytes(int64_t, int32_t, int32_t, int32_t) { return 256; }
int cagra_optimize(const uint32_t *, int64_t, int32_t, int32_t, uint32_t *, uint32_t *, uint32_t *, uint32_t *, void *, size_t, void *) { return CAGRA_ERR_LAUNCH; }
size_t cagra_optimize_workspace_bytes(int64_t, int32_t, int32_t) { return 256; }
}
