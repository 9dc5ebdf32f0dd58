// Input-patch SPARQ convolution, wave-specialised variant (4 matrix + 4 staging wavefronts, two
// workgroups per CU): 128 output pixels x 64 output channels per workgroup, 4 patch chunks per
// staging lane and unit, 128 input channels per unit: all trim variants.
#include "sparq_conv_patch_kernel.h"

namespace sparq {
SPARQ_DECLARE_PATCH(launch_patch_ws_n64_a4c2) { return launch_patch_kind<PatchCfg<64, 4, 1, 4, 2, 2, true>>(kind, p, npix_max, s); }
}  // namespace sparq
