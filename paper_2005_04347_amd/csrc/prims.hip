// Device-wide integer primitives used by the preprocess (levels, pack):
// exclusive prefix sum and a stable LSD radix sort of (key, value) pairs.
// Both are deterministic: the same input always gives the same output.
#include "asnn_common.h"

namespace asnn {

// ------------------------------------------------------------------ scan
constexpr int kScanThreads = 256;
constexpr int kScanItems = 8;
constexpr int kScanTile = kScanThreads * kScanItems;   // 2048 values per block

// Exclusive scan of one value per thread across a 256-thread block; returns
// the exclusive prefix of this thread and the block total through *total.
__device__ inline int block_exclusive_scan(int x, int *total) {
    __shared__ int wave_sums[kScanThreads / kWave];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    int incl = x;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        int y = __shfl_up(incl, d, kWave);
        if (lane >= d) incl += y;
    }
    if (lane == kWave - 1) wave_sums[wave] = incl;
    __syncthreads();
    int wave_prefix = 0, tot = 0;
#pragma unroll
    for (int k = 0; k < kScanThreads / kWave; ++k) {
        int s = wave_sums[k];
        if (k < wave) wave_prefix += s;
        tot += s;
    }
    __syncthreads();
    *total = tot;
    return wave_prefix + incl - x;
}

__global__ __launch_bounds__(kScanThreads) void scan_reduce_kernel(const int32_t *__restrict__ in,
                                                                     int32_t *__restrict__ block_sums, size_t n) {
    const size_t base = (size_t)blockIdx.x * kScanTile + (size_t)threadIdx.x * kScanItems;
    int sum = 0;
#pragma unroll
    for (int k = 0; k < kScanItems; ++k)
        if (base + k < n) sum += in[base + k];
    int total;
    (void)block_exclusive_scan(sum, &total);
    if (threadIdx.x == 0) block_sums[blockIdx.x] = total;
}

// out[i] = block_prefix[blockIdx] + exclusive scan inside the tile.
__global__ __launch_bounds__(kScanThreads) void scan_apply_kernel(const int32_t *in, int32_t *out,
                                                                    const int32_t *__restrict__ block_prefix, size_t n) {
    const size_t base = (size_t)blockIdx.x * kScanTile + (size_t)threadIdx.x * kScanItems;
    int v[kScanItems];
    int sum = 0;
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) {
        v[k] = (base + k < n) ? in[base + k] : 0;
        sum += v[k];
    }
    int total;
    int run = block_exclusive_scan(sum, &total) + (block_prefix ? block_prefix[blockIdx.x] : 0);
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) {
        if (base + k < n) out[base + k] = run;
        run += v[k];
    }
}

size_t scan_tmp_ints(size_t n) {
    size_t total = 0;
    while (n > (size_t)kScanTile) {
        n = (n + kScanTile - 1) / kScanTile;
        total += align_up(n * sizeof(int32_t)) / sizeof(int32_t);
    }
    return total + 64;
}

int exclusive_scan_i32(const int32_t *in, int32_t *out, size_t n, int32_t *tmp, hipStream_t s) {
    if (n == 0) return ASNN_OK;
    const size_t nb = (n + kScanTile - 1) / kScanTile;
    if (nb == 1) {
        hipLaunchKernelGGL(scan_apply_kernel, dim3(1), dim3(kScanThreads), 0, s, in, out, (const int32_t *)nullptr, n);
        ASNN_HIP_TRY(hipGetLastError());
        return ASNN_OK;
    }
    int32_t *sums = tmp;
    int32_t *rest = tmp + align_up(nb * sizeof(int32_t)) / sizeof(int32_t);
    hipLaunchKernelGGL(scan_reduce_kernel, dim3((unsigned)nb), dim3(kScanThreads), 0, s, in, sums, n);
    ASNN_HIP_TRY(hipGetLastError());
    ASNN_TRY(exclusive_scan_i32(sums, sums, nb, rest, s));
    hipLaunchKernelGGL(scan_apply_kernel, dim3((unsigned)nb), dim3(kScanThreads), 0, s, in, out, (const int32_t *)sums, n);
    ASNN_HIP_TRY(hipGetLastError());
    return ASNN_OK;
}

// ------------------------------------------------------------ radix sort
constexpr int kRadixBits = 8;
constexpr int kRadixBins = 1 << kRadixBits;
constexpr int kRadixRounds = 16;
constexpr int kRadixTile = kWave * kRadixRounds;   // 1024 pairs per one-wave block

// hist[d * nblocks + block] = number of keys of this block's tile with digit d.
__global__ __launch_bounds__(kWave) void radix_hist_kernel(const uint32_t *__restrict__ keys, size_t n, int shift,
                                                            int32_t *__restrict__ hist, unsigned nblocks) {
    __shared__ int bins[kRadixBins];
    for (int d = threadIdx.x; d < kRadixBins; d += kWave) bins[d] = 0;
    __syncthreads();
    const size_t base = (size_t)blockIdx.x * kRadixTile;
#pragma unroll 4
    for (int r = 0; r < kRadixRounds; ++r) {
        size_t i = base + (size_t)r * kWave + threadIdx.x;
        if (i < n) atomicAdd(&bins[(keys[i] >> shift) & (kRadixBins - 1)], 1);
    }
    __syncthreads();
    for (int d = threadIdx.x; d < kRadixBins; d += kWave) hist[(size_t)d * nblocks + blockIdx.x] = bins[d];
}

// Stable scatter: pairs of one tile keep their relative order inside a digit.
__global__ __launch_bounds__(kWave) void radix_scatter_kernel(const uint32_t *__restrict__ keys_in,
                                                               const uint32_t *__restrict__ vals_in,
                                                               uint32_t *__restrict__ keys_out,
                                                               uint32_t *__restrict__ vals_out, size_t n, int shift,
                                                               const int32_t *__restrict__ offsets, unsigned nblocks) {
    __shared__ int next[kRadixBins];
    for (int d = threadIdx.x; d < kRadixBins; d += kWave) next[d] = offsets[(size_t)d * nblocks + blockIdx.x];
    __syncthreads();
    const size_t base = (size_t)blockIdx.x * kRadixTile;
    const int lane = threadIdx.x;
    const unsigned long long below = (lane == 0) ? 0ull : (~0ull >> (kWave - lane));
    for (int r = 0; r < kRadixRounds; ++r) {
        const size_t i = base + (size_t)r * kWave + lane;
        const bool valid = i < n;
        uint32_t key = 0, val = 0;
        if (valid) { key = keys_in[i]; val = vals_in[i]; }
        const int d = (key >> shift) & (kRadixBins - 1);
        unsigned long long peers = __ballot(valid);
#pragma unroll
        for (int b = 0; b < kRadixBits; ++b) {
            const int bit = (d >> b) & 1;
            const unsigned long long m = __ballot(bit);
            peers &= bit ? m : ~m;
        }
        const int rank = __popcll(peers & below);
        const int count = __popcll(peers);
        int start = 0;
        if (valid) start = next[d];
        __syncthreads();
        if (valid && rank == 0) next[d] = start + count;
        __syncthreads();
        if (valid) {
            keys_out[start + rank] = key;
            vals_out[start + rank] = val;
        }
    }
}

size_t radix_tmp_ints(size_t n) {
    const size_t nblocks = (n + kRadixTile - 1) / kRadixTile + 1;
    const size_t hist = align_up(nblocks * kRadixBins * sizeof(int32_t)) / sizeof(int32_t);
    return hist + scan_tmp_ints(nblocks * kRadixBins);
}

int radix_sort_pairs_u32(uint32_t *keys_a, uint32_t *vals_a, uint32_t *keys_b, uint32_t *vals_b, size_t n, int bits,
                         int32_t *tmp, hipStream_t s, uint32_t **keys_sorted, uint32_t **vals_sorted) {
    *keys_sorted = keys_a;
    *vals_sorted = vals_a;
    if (n == 0) return ASNN_OK;
    const unsigned nblocks = (unsigned)((n + kRadixTile - 1) / kRadixTile);
    const size_t hist_len = (size_t)nblocks * kRadixBins;
    int32_t *hist = tmp;
    int32_t *scan_tmp = tmp + align_up(hist_len * sizeof(int32_t)) / sizeof(int32_t);
    uint32_t *kin = keys_a, *vin = vals_a, *kout = keys_b, *vout = vals_b;
    for (int shift = 0; shift < bits; shift += kRadixBits) {
        hipLaunchKernelGGL(radix_hist_kernel, dim3(nblocks), dim3(kWave), 0, s, (const uint32_t *)kin, n, shift, hist,
                           nblocks);
        ASNN_HIP_TRY(hipGetLastError());
        ASNN_TRY(exclusive_scan_i32(hist, hist, hist_len, scan_tmp, s));
        hipLaunchKernelGGL(radix_scatter_kernel, dim3(nblocks), dim3(kWave), 0, s, (const uint32_t *)kin,
                           (const uint32_t *)vin, kout, vout, n, shift, (const int32_t *)hist, nblocks);
        ASNN_HIP_TRY(hipGetLastError());
        uint32_t *t;
        t = kin; kin = kout; kout = t;
        t = vin; vin = vout; vout = t;
    }
    *keys_sorted = kin;
    *vals_sorted = vin;
    return ASNN_OK;
}

}  // namespace asnn
