// Input-patch SPARQ convolution with 2:4 pruned weights on the sparse matrix instruction (wave-specialised:
// 4 matrix + 4 staging wavefronts): 128 output pixels x 256 output channels per workgroup, every staging shape.
#include "sparq_conv_patch_kernel.h"

namespace sparq {
SPARQ_DECLARE_PATCH(launch_patch_sp_n256_a2c1) { return launch_patch_kind_sparse<PatchCfg<256, 1, 4, 2, 1, 1, true, true>>(kind, p, npix_max, s); }
SPARQ_DECLARE_PATCH(launch_patch_sp_n256_a4c1) { return launch_patch_kind_sparse<PatchCfg<256, 1, 4, 4, 1, 1, true, true>>(kind, p, npix_max, s); }
SPARQ_DECLARE_PATCH(launch_patch_sp_n256_a8c1) { return launch_patch_kind_sparse<PatchCfg<256, 1, 4, 8, 1, 1, true, true>>(kind, p, npix_max, s); }
SPARQ_DECLARE_PATCH(launch_patch_sp_n256_a12c1) { return launch_patch_kind_sparse<PatchCfg<256, 1, 4, 12, 1, 1, true, true>>(kind, p, npix_max, s); }
SPARQ_DECLARE_PATCH(launch_patch_sp_n256_a4c2) { return launch_patch_kind_sparse<PatchCfg<256, 1, 4, 4, 2, 1, true, true>>(kind, p, npix_max, s); }
SPARQ_DECLARE_PATCH(launch_patch_sp_n256_a8c4) { return launch_patch_kind_sparse<PatchCfg<256, 1, 4, 8, 4, 1, true, true>>(kind, p, npix_max, s); }
}  // namespace sparq
