// Machine-ceiling micro-benchmarks (see include/sparq_probe.h): a register-only int8 matrix-instruction
// loop and a streaming copy.  Built into libsparq_probe.so, separate from the method's library.
#include <hip/hip_runtime.h>

#include "../../../include/sparq_probe.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kProbeBlocks = 256, kProbeThreads = 256;

// Each wavefront: a 128 x 64 tile of results (4 x 2 fragments of 32 x 32), two 32-byte reduction halves per
// iteration: 16 matrix instructions per iteration, operands loaded once and kept in registers.
__global__ __launch_bounds__(kProbeThreads) void mfma_i8_loop(const v4i* __restrict__ src, int* __restrict__ sink, int iters) {
    v4i a[2][4], b[2][2];
    for (int k = 0; k < 2; ++k)
        for (int i = 0; i < 4; ++i) {
            a[k][i] = src[(k * 4 + i) * kProbeThreads + threadIdx.x];
            if (i < 2) b[k][i] = src[(8 + k * 2 + i) * kProbeThreads + threadIdx.x];
        }
    v16i c[4][2];
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 2; ++j)
            for (int v = 0; v < 16; ++v) c[i][j][v] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < 2; ++k)
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    c[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[k][i], b[k][j], c[i][j], 0, 0, 0);
    }
    int s = 0;
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 2; ++j)
            for (int v = 0; v < 16; ++v) s += c[i][j][v];
    sink[blockIdx.x * kProbeThreads + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace

extern "C" double sparq_probe_mfma_i8_ops(int32_t iters) {
    // 2 ops per multiply-accumulate x 32*32*32 per instruction x 16 per iteration x 4 wavefronts x workgroups
    return 2.0 * 32768.0 * 16.0 * (double)iters * 4.0 * kProbeBlocks;
}

extern "C" int sparq_probe_mfma_i8(const void* operands, void* sink, int32_t iters, void* stream) {
    if (!operands || !sink || iters <= 0) return 1;
    mfma_i8_loop<<<kProbeBlocks, kProbeThreads, 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<const v4i*>(operands), static_cast<int*>(sink), iters);
    return hipGetLastError() == hipSuccess ? 0 : 4;
}

extern "C" int sparq_probe_copy(const void* src, void* dst, size_t bytes, void* stream) {
    if (!src || !dst || (bytes & 15) || ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15)) return 1;
    if (bytes == 0) return 0;
    const size_t n16 = bytes / 16;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    copy_kernel<<<(unsigned)blocks, 256, 0, static_cast<hipStream_t>(stream)>>>(static_cast<const uint4*>(src),
                                                                                 static_cast<uint4*>(dst), n16);
    return hipGetLastError() == hipSuccess ? 0 : 4;
}
