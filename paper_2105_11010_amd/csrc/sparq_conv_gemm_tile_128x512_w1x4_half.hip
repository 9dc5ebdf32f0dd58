// Fused SPARQ conv-GEMM, workgroup tile 128 output pixels x 512 output channels,
// 1 x 4 wavefronts, main loop pipelined by half steps (activations requested 3 steps, weights 4 halves ahead): all trim variants.
#include "sparq_conv_gemm_kernel.h"

namespace sparq {
SPARQ_DECLARE_TILE(launch_tile_128x512_w1x4_half) { return launch_kind<TileCfg<128, 512, 1, 4, 3, 4, false, 0, true>>(kind, p, s); }
}  // namespace sparq
