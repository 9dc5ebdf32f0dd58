// Input-patch SPARQ convolution, wave-specialised variant (4 matrix + 4 staging wavefronts):
// 128 output pixels x 128 output channels per workgroup, 8 patch chunks per staging lane and unit,
// 64 input channels per unit: all trim variants.
#include "sparq_conv_patch_kernel.h"

namespace sparq {
SPARQ_DECLARE_PATCH(launch_patch_ws_n128_a8c1) { return launch_patch_kind<PatchCfg<128, 2, 2, 8, 1, 1, true>>(kind, p, npix_max, s); }
}  // namespace sparq
