// Input-patch SPARQ convolution: 128 output pixels x 64 output channels per workgroup (4 x 1 wavefronts),
// 12 patch chunks per lane and unit, 64 input channels per unit: all trim variants.
#include "sparq_conv_patch_kernel.h"

namespace sparq {
SPARQ_DECLARE_PATCH(launch_patch_n64_a12c1) { return launch_patch_kind<PatchCfg<64, 4, 1, 12, 1, 2>>(kind, p, npix_max, s); }
}  // namespace sparq
