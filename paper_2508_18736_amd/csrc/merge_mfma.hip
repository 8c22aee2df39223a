// MFMA pair search (placeholder until the tiled symmetric kernel lands).
#include "siso_internal.h"

int siso_merge_mfma_supported(const siso_cache *) { return 0; }
int siso_merge_mfma_launch(siso_cache *c, float, int *, long) {
    return siso_fail(c, SISO_EINVAL, "mfma merge path is not available");
}
