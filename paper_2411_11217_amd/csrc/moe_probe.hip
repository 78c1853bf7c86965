// Rate probes: measurement helpers, not part of the layer.  The paper's performance model takes
// "profiled" peak rates of the hardware as its inputs (section 4.2); these kernels measure the
// memory-side one in isolation from the layer's own kernels.
#include "moe_internal.h"

namespace moe {
namespace {

// Every block streams a contiguous share of the buffer with 16-byte loads per lane (whole 1 KiB
// stretches per wavefront and instruction) and folds what it read into one word, which is only
// written when it has a value no real buffer produces: the loads cannot be dropped.
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ src, size_t n16, int32_t* __restrict__ sink) {
    const size_t per_block = (n16 + gridDim.x - 1) / gridDim.x;
    const size_t begin = (size_t)blockIdx.x * per_block;
    const size_t end = begin + per_block < n16 ? begin + per_block : n16;
    uint4 acc = {0u, 0u, 0u, 0u};
    size_t i = begin + threadIdx.x;
    for (; i + 3 * 256 < end; i += 4 * 256) {            // four independent loads in flight per lane
        const uint4 a = src[i], b = src[i + 256], c = src[i + 512], d = src[i + 768];
        acc.x ^= a.x ^ b.x ^ c.x ^ d.x;
        acc.y ^= a.y ^ b.y ^ c.y ^ d.y;
        acc.z ^= a.z ^ b.z ^ c.z ^ d.z;
        acc.w ^= a.w ^ b.w ^ c.w ^ d.w;
    }
    for (; i < end; i += 256) {
        const uint4 a = src[i];
        acc.x ^= a.x; acc.y ^= a.y; acc.z ^= a.z; acc.w ^= a.w;
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x5eedf00du && sink) atomicOr(sink, 1);
}

}  // namespace
}  // namespace moe

extern "C" int moe_probe_stream_read(const void* src, size_t bytes, int32_t blocks, int32_t* sink, void* stream) {
    if (!src || bytes == 0 || bytes % 16 != 0 || blocks < 1 || blocks > 65536) return MOE_ERR_INVALID_ARG;
    if (((uintptr_t)src & 15) != 0) return MOE_ERR_INVALID_ARG;
    hipLaunchKernelGGL(moe::stream_read_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (const uint4*)src, bytes / 16, sink);
    MOE_HIP_TRY(hipGetLastError());
    return MOE_OK;
}
