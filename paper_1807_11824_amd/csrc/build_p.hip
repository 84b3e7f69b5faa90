// placeholder until the affinity construction lands
#include "tsne_internal.h"
extern "C" {
int tsne_build_P_workspace_bytes(int32_t, int32_t, int32_t, size_t *) { return TSNE_ESTATE; }
int tsne_build_P(const float *, int32_t, int32_t, float, int32_t, int32_t *, int32_t *, float *, int64_t, int64_t *,
                 int32_t *, float *, int32_t *, void *, size_t, void *) { return TSNE_ESTATE; }
}
