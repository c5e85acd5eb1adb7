// asnn_device_copy: a plain streaming copy used as the bandwidth yardstick
// (what fraction of a device copy the activation sustains) and as the kernel
// of known traffic against which hardware byte counters are calibrated.
#include "asnn_common.h"

namespace asnn {
namespace {
__global__ __launch_bounds__(256) void copy_kernel(const float4 *__restrict__ in, float4 *__restrict__ out, size_t n4) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) out[i] = in[i];
}
}  // namespace
}  // namespace asnn

extern "C" int asnn_device_copy(void *dst, const void *src, size_t bytes, void *stream) {
    if (!dst || !src) return ASNN_ERR_NULL;
    if (bytes == 0) return ASNN_OK;
    if ((bytes & 15u) != 0 || ((uintptr_t)dst & 15u) != 0 || ((uintptr_t)src & 15u) != 0) return ASNN_ERR_SIZE;
    const size_t n4 = bytes / 16;
    const unsigned blocks = asnn::blocks_for(n4, 256 * 4, 256 * 32);
    hipLaunchKernelGGL(asnn::copy_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const float4 *>(src), static_cast<float4 *>(dst), n4);
    ASNN_HIP_TRY(hipGetLastError());
    return ASNN_OK;
}
