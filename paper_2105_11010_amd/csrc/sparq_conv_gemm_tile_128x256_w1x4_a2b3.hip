// Fused SPARQ conv-GEMM, workgroup tile 128 output pixels x 256 output channels,
// 1 x 4 wavefronts, activation / weight loads 2 / 3 reduction steps ahead: all trim variants.
#include "sparq_conv_gemm_kernel.h"

namespace sparq {
SPARQ_DECLARE_TILE(launch_tile_128x256_w1x4_a2b3) { return launch_kind<TileCfg<128, 256, 1, 4, 2, 3>>(kind, p, s); }
}  // namespace sparq
