// Plain copy kernel of known size: the yardstick for hardware byte counters.
#include "common.h"

namespace remoe {

namespace {

__global__ __launch_bounds__(256) void copy_probe_kernel(u32x4_t *__restrict__ dst, const u32x4_t *__restrict__ src, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace

remoe_status launch_copy_probe(void *dst, const void *src, size_t bytes, hipStream_t stream)
{
    const size_t n16 = bytes / 16;
    if (n16 == 0) return REMOE_OK;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(copy_probe_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, static_cast<u32x4_t *>(dst),
                       static_cast<const u32x4_t *>(src), n16);
    return check_hip(hipGetLastError(), "copy_probe_kernel launch");
}

}  // namespace remoe
