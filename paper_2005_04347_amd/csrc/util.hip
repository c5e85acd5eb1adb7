// Bandwidth yardsticks: kernels of known traffic that do none of the method's arithmetic.  The
// benchmark times them beside the activation (what a plain copy, a plain streaming read and a
// random row gather of the activation's own shape sustain on this device), and the copy doubles
// as the kernel of known traffic against which hardware byte counters are calibrated.
#include "asnn_common.h"

namespace asnn {
namespace {
__global__ __launch_bounds__(256) void copy_kernel(const float4 *__restrict__ in, float4 *__restrict__ out, size_t n4) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) out[i] = in[i];
}

// Streaming read: every thread keeps four 16-byte loads in flight and folds what it reads into one
// number, which is stored only if it has a value that sums of ordinary data do not take (the store
// keeps the loads alive without adding write traffic).
__global__ __launch_bounds__(256) void read_kernel(const float4 *__restrict__ in, size_t n4, float *sink) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    float acc = 0.0f;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i + 3 * stride < n4; i += 4 * stride) {
        const float4 a = in[i], b = in[i + stride], c = in[i + 2 * stride], d = in[i + 3 * stride];
        acc += (a.x + a.y + a.z + a.w) + (b.x + b.y + b.z + b.w) + (c.x + c.y + c.z + c.w) + (d.x + d.y + d.z + d.w);
    }
    for (; i < n4; i += stride) {
        const float4 a = in[i];
        acc += a.x + a.y + a.z + a.w;
    }
    if (acc == -1.2345678e30f) sink[0] = acc;
}

__device__ inline uint32_t mix32(uint32_t x) {
    x ^= x >> 15; x *= 0x2c1b3c6du; x ^= x >> 12; x *= 0x297a2d39u; x ^= x >> 15;
    return x;
}

// Random row gather in the launch shape of a level of the activation: one single-wavefront block
// per (row being computed, tile of batch columns), block index row-major, each wavefront loading
// the same tile of `gathers` pseudo-random source rows (eight loads in flight), the 64 lanes
// covering the tile with VEC floats each.  All tiles of one row pick the same source rows, as the
// connections of a node do.  Only the additions that keep the loads alive are done.  With STORE
// every wavefront also writes its tile of row item_row of `out` (out[rows of the launch][row_floats]),
// as a level writes the rows it computes; without, `out` is the sink of a read-only kernel.
template <int VEC, bool STORE>
__global__ __launch_bounds__(kWave) void gather_rows_kernel(const float *__restrict__ buf, uint32_t n_rows, int row_floats,
                                                             int tiles, int gathers, uint32_t seed, float *out) {
    const uint32_t item_row = blockIdx.x / (uint32_t)tiles;
    const int tile = (int)(blockIdx.x % (uint32_t)tiles);
    const float *base = buf + (size_t)tile * (kWave * VEC) + threadIdx.x * VEC;
    float acc[VEC];
#pragma unroll
    for (int j = 0; j < VEC; ++j) acc[j] = 0.0f;
    for (int k0 = 0; k0 < gathers; k0 += 8) {
        float v[8][VEC];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
#pragma unroll
            for (int j = 0; j < VEC; ++j) v[k][j] = 0.0f;
            if (k0 + k < gathers) {          // wave-uniform: the last round loads only what is left
                const uint32_t h = mix32((item_row * 0x9e3779b1u) ^ ((uint32_t)(k0 + k) * 0x85ebca77u) ^ seed);
                const uint32_t r = __umulhi(h, n_rows);
                const float *p = base + (size_t)r * (size_t)row_floats;
                if constexpr (VEC == 2) { const float2 t = *reinterpret_cast<const float2 *>(p); v[k][0] = t.x; v[k][1] = t.y; }
                else { v[k][0] = *p; }
            }
        }
#pragma unroll
        for (int k = 0; k < 8; ++k)
#pragma unroll
            for (int j = 0; j < VEC; ++j) acc[j] += v[k][j];
    }
    if constexpr (STORE) {
        float *q = out + (size_t)item_row * (size_t)row_floats + (size_t)tile * (kWave * VEC) + threadIdx.x * VEC;
        if constexpr (VEC == 2) *reinterpret_cast<float2 *>(q) = make_float2(acc[0], acc[1]);
        else *q = acc[0];
    } else {
        float all = 0.0f;
#pragma unroll
        for (int j = 0; j < VEC; ++j) all += acc[j];
        if (all == -1.2345678e30f) out[0] = all;
    }
}

int launch_gather(const float *buf, int32_t n_rows, int32_t row_floats, int32_t rows_per_launch, int32_t gathers,
                  uint32_t seed, float *out, bool store, hipStream_t s) {
    if (!buf || !out) return ASNN_ERR_NULL;
    if (n_rows <= 0 || row_floats <= 0 || rows_per_launch <= 0 || gathers <= 0) return ASNN_ERR_SIZE;
    if (row_floats % kWave != 0 || ((uintptr_t)buf & 7u) != 0 || (store && ((uintptr_t)out & 7u) != 0)) return ASNN_ERR_SIZE;
    const int vec = row_floats % (2 * kWave) == 0 ? 2 : 1;
    const int tiles = row_floats / (kWave * vec);
    const long long blocks = (long long)rows_per_launch * tiles;
    if (blocks > 0x7fffffffLL) return ASNN_ERR_SIZE;
    const dim3 grid((unsigned)blocks), block(kWave);
    if (vec == 2 && store)
        hipLaunchKernelGGL((gather_rows_kernel<2, true>), grid, block, 0, s, buf, (uint32_t)n_rows, row_floats, tiles, gathers, seed, out);
    else if (vec == 2)
        hipLaunchKernelGGL((gather_rows_kernel<2, false>), grid, block, 0, s, buf, (uint32_t)n_rows, row_floats, tiles, gathers, seed, out);
    else if (store)
        hipLaunchKernelGGL((gather_rows_kernel<1, true>), grid, block, 0, s, buf, (uint32_t)n_rows, row_floats, tiles, gathers, seed, out);
    else
        hipLaunchKernelGGL((gather_rows_kernel<1, false>), grid, block, 0, s, buf, (uint32_t)n_rows, row_floats, tiles, gathers, seed, out);
    ASNN_HIP_TRY(hipGetLastError());
    return ASNN_OK;
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

extern "C" int asnn_device_read(const void *src, size_t bytes, float *sink, void *stream) {
    if (!src || !sink) return ASNN_ERR_NULL;
    if (bytes == 0) return ASNN_OK;
    if ((bytes & 15u) != 0 || ((uintptr_t)src & 15u) != 0) return ASNN_ERR_SIZE;
    const size_t n4 = bytes / 16;
    const unsigned blocks = asnn::blocks_for(n4, 256 * 4, 256 * 32);
    hipLaunchKernelGGL(asnn::read_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const float4 *>(src), n4, sink);
    ASNN_HIP_TRY(hipGetLastError());
    return ASNN_OK;
}

extern "C" int asnn_device_gather(const float *buf, int32_t n_rows, int32_t row_floats, int32_t rows_per_launch,
                                  int32_t gathers, uint32_t seed, float *sink, void *stream) {
    return asnn::launch_gather(buf, n_rows, row_floats, rows_per_launch, gathers, seed, sink, false,
                               static_cast<hipStream_t>(stream));
}

extern "C" int asnn_device_gather_store(const float *buf, int32_t n_rows, int32_t row_floats, int32_t rows_per_launch,
                                        int32_t gathers, uint32_t seed, float *out, void *stream) {
    return asnn::launch_gather(buf, n_rows, row_floats, rows_per_launch, gathers, seed, out, true,
                               static_cast<hipStream_t>(stream));
}
