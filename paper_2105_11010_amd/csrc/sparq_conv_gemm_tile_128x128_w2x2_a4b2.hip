// Fused SPARQ conv-GEMM, workgroup tile 128 output pixels x 128 output channels,
// 2 x 2 wavefronts, activation / weight loads 4 / 2 reduction steps ahead: all trim variants.
#include "sparq_conv_gemm_kernel.h"

namespace sparq {
SPARQ_DECLARE_TILE(launch_tile_128x128_w2x2_a4b2) { return launch_kind<TileCfg<128, 128, 2, 2, 4, 2>>(kind, p, s); }
}  // namespace sparq
