// tkv_probe_stream_read: a plain 128-bit streaming read of a device buffer, the speed-of-light probe that
// the decode kernel (a read-only scan of the packed pool) is reported against beside the published HBM peak.
// It computes nothing of the method.
#include <hip/hip_runtime.h>

#include "tkv_internal.h"

namespace {

__global__ __launch_bounds__(256) void tkv_probe_read_kernel(const uint4 *__restrict__ buf, size_t n, uint32_t *sink)
{
    size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    uint32_t acc = 0;
    for (; i < n; i += stride) {
        const uint4 v = buf[i];
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    // keeps the loads alive; a lane's xor of its share hits this value once in 2^32
    if (acc == 0x5a17c0deu && sink) atomicOr(sink, 1u);
}

} // namespace

int tkv_launch_probe_read(const void *buf, size_t bytes, uint32_t *sink, void *stream)
{
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return TKV_ERR_HIP;
    const size_t n = bytes / 16;
    hipLaunchKernelGGL(tkv_probe_read_kernel, dim3((unsigned)(cus * 8)), dim3(256), 0, (hipStream_t)stream,
                       (const uint4 *)buf, n, sink);
    return hipGetLastError() == hipSuccess ? TKV_OK : TKV_ERR_HIP;
}
