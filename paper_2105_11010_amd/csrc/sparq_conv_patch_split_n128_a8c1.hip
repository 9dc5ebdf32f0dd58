// Input-patch SPARQ convolution, split-reduction variant (partial sums added with atomics):
// 128 output pixels x 128 output channels per workgroup (2 x 2 wavefronts), 8 patch chunks per lane
// and unit, 64 input channels per unit: all trim variants.
#include "sparq_conv_patch_kernel.h"

namespace sparq {
SPARQ_DECLARE_PATCH(launch_patch_split_n128_a8c1) { return launch_patch_kind<PatchCfg<128, 2, 2, 8, 1, 2, true>>(kind, p, npix_max, s); }
}  // namespace sparq
