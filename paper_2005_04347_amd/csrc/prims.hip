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
// One pass = a histogram per tile, an exclusive scan over (digit, tile), and a stable scatter.
// A tile is 4096 pairs handled by a 256-thread block.  The scatter first brings the tile into
// digit order in LDS and then writes it out, so that the pairs of one digit leave as one
// contiguous run (16 pairs on average) instead of one by one.
constexpr int kRadixBits = 8;
constexpr int kRadixBins = 1 << kRadixBits;
constexpr int kRadixThreads = 256;
constexpr int kRadixWaves = kRadixThreads / kWave;
constexpr int kRadixRounds = 16;                                // pairs per thread
constexpr int kRadixTile = kRadixThreads * kRadixRounds;       // 4096 pairs per block
static_assert(kRadixBins == kRadixThreads, "the scatter gives every digit a thread of its own");

// hist[d * nblocks + block] = number of keys of this block's tile with digit d.
__global__ __launch_bounds__(kRadixThreads) void radix_hist_kernel(const uint32_t *__restrict__ keys, size_t n, int shift,
                                                                    int32_t *__restrict__ hist, unsigned nblocks) {
    __shared__ int bins[kRadixBins];
    bins[threadIdx.x] = 0;
    __syncthreads();
    const size_t base = (size_t)blockIdx.x * kRadixTile;
#pragma unroll 4
    for (int r = 0; r < kRadixRounds; ++r) {
        const size_t i = base + (size_t)r * kRadixThreads + threadIdx.x;
        if (i < n) atomicAdd(&bins[(keys[i] >> shift) & (kRadixBins - 1)], 1);
    }
    __syncthreads();
    hist[(size_t)threadIdx.x * nblocks + blockIdx.x] = bins[threadIdx.x];
}

// Stable scatter: pairs with the same digit keep their order.  Wavefront w takes pairs
// [1024 w, 1024 (w+1)) of the tile, 64 at a time; a pair's place among the pairs of its digit is
// (pairs of the digit in earlier wavefronts) + (in earlier rounds of its own) + (in lower lanes of
// its round), the last from ballots.
__global__ __launch_bounds__(kRadixThreads) void radix_scatter_kernel(const uint32_t *__restrict__ keys_in,
                                                                       const uint32_t *__restrict__ vals_in,
                                                                       uint32_t *__restrict__ keys_out,
                                                                       uint32_t *__restrict__ vals_out, size_t n, int shift,
                                                                       const int32_t *__restrict__ offsets, unsigned nblocks) {
    __shared__ uint32_t s_key[kRadixTile], s_val[kRadixTile];
    __shared__ int wave_count[kRadixWaves][kRadixBins];     // running count, later: pairs in earlier wavefronts
    __shared__ int tile_start[kRadixBins];                  // first place of the digit inside the sorted tile
    __shared__ int out_shift[kRadixBins];                   // global position = place inside the tile + this
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
#pragma unroll
    for (int w = 0; w < kRadixWaves; ++w) wave_count[w][threadIdx.x] = 0;
    __syncthreads();
    const size_t base = (size_t)blockIdx.x * kRadixTile;
    const size_t wave_base = base + (size_t)wave * (kRadixRounds * kWave);
    const unsigned long long below = (lane == 0) ? 0ull : (~0ull >> (kWave - lane));
    uint32_t key[kRadixRounds], val[kRadixRounds];
    int place[kRadixRounds];
#pragma unroll
    for (int r = 0; r < kRadixRounds; ++r) {
        const size_t i = wave_base + (size_t)r * kWave + lane;
        const bool valid = i < n;
        key[r] = 0;
        val[r] = 0;
        if (valid) { key[r] = keys_in[i]; val[r] = vals_in[i]; }
        const int d = (key[r] >> shift) & (kRadixBins - 1);
        unsigned long long peers = __ballot(valid);
#pragma unroll
        for (int b = 0; b < kRadixBits; ++b) {
            const int bit = (d >> b) & 1;
            const unsigned long long m = __ballot(bit);
            peers &= bit ? m : ~m;
        }
        // LDS accesses of one wavefront complete in program order: every lane has read the
        // running count before the first lane of each digit adds this round's pairs to it
        const int before = valid ? wave_count[wave][d] : 0;
        if (valid && (peers & below) == 0) wave_count[wave][d] = before + __popcll(peers);
        place[r] = before + __popcll(peers & below);
    }
    __syncthreads();
    {   // thread d owns digit d: counts of the wavefronts -> exclusive prefix over them, digit totals -> tile_start
        const int d = threadIdx.x;
        int run = 0;
#pragma unroll
        for (int w = 0; w < kRadixWaves; ++w) {
            const int c = wave_count[w][d];
            wave_count[w][d] = run;
            run += c;
        }
        int total;
        const int start = block_exclusive_scan(run, &total);
        tile_start[d] = start;
        out_shift[d] = offsets[(size_t)d * nblocks + blockIdx.x] - start;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kRadixRounds; ++r) {
        const size_t i = wave_base + (size_t)r * kWave + lane;
        if (i < n) {
            const int d = (key[r] >> shift) & (kRadixBins - 1);
            const int p = tile_start[d] + wave_count[wave][d] + place[r];
            s_key[p] = key[r];
            s_val[p] = val[r];
        }
    }
    __syncthreads();
    const size_t left = n - base;
    const int n_tile = left < (size_t)kRadixTile ? (int)left : kRadixTile;
    for (int i = threadIdx.x; i < n_tile; i += kRadixThreads) {
        const uint32_t k = s_key[i];
        const size_t o = (size_t)(out_shift[(k >> shift) & (kRadixBins - 1)] + i);
        keys_out[o] = k;
        vals_out[o] = s_val[i];
    }
}

// ------------------------------------------------------------ runs of sorted keys
// first[k] = where the run of key k starts in the sorted keys ...
__global__ void run_heads_kernel(const uint32_t *__restrict__ keys, size_t n, int32_t *__restrict__ first) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
        if (i == 0 || keys[i - 1] != keys[i]) first[keys[i]] = (int32_t)i;
}

// ... and count[k] = its length.
__global__ void run_lengths_kernel(const uint32_t *__restrict__ keys, size_t n, const int32_t *__restrict__ first,
                                   int32_t *__restrict__ count) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
        if (i == n - 1 || keys[i + 1] != keys[i]) count[keys[i]] = (int32_t)(i + 1) - first[keys[i]];
}

int sorted_run_lengths(const uint32_t *keys, size_t n, int32_t *first, int32_t *count, hipStream_t s) {
    if (n == 0) return ASNN_OK;
    const dim3 grid(blocks_for(n, 256, 65535)), block(256);
    hipLaunchKernelGGL(run_heads_kernel, grid, block, 0, s, keys, n, first);
    ASNN_HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(run_lengths_kernel, grid, block, 0, s, keys, n, (const int32_t *)first, count);
    ASNN_HIP_TRY(hipGetLastError());
    return ASNN_OK;
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
        hipLaunchKernelGGL(radix_hist_kernel, dim3(nblocks), dim3(kRadixThreads), 0, s, (const uint32_t *)kin, n, shift,
                           hist, nblocks);
        ASNN_HIP_TRY(hipGetLastError());
        ASNN_TRY(exclusive_scan_i32(hist, hist, hist_len, scan_tmp, s));
        hipLaunchKernelGGL(radix_scatter_kernel, dim3(nblocks), dim3(kRadixThreads), 0, s, (const uint32_t *)kin,
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
