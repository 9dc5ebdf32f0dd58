// Fused SPARQ conv-GEMM, workgroup tile 128 output pixels x 512 output channels,
// 1 x 4 wavefronts, activation / weight loads 1 / 3 reduction steps ahead: all trim variants.
#include "sparq_conv_gemm_kernel.h"

namespace sparq {
SPARQ_DECLARE_TILE(launch_tile_128x512_w1x4_a1b3) { return launch_kind<TileCfg<128, 512, 1, 4, 1, 3>>(kind, p, s); }
}  // namespace sparq
