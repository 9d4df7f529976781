// Fused single-read A pass (placeholder until the kernel lands): reports that no shape fits, so
// every solver uses the two-pass organisation.
#include "common.h"

namespace lb {

bool fused_shape_ok(const Dims&, const void*, int* variant, int* blocks) {
    *variant = -1;
    *blocks = 0;
    return false;
}

void launch_fused(const Dims&, const Geometry&, const Buffers&, const APassArgs&, hipStream_t) {}

}  // namespace lb
