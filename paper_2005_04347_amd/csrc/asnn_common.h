// Internal helpers shared by the libasnn translation units (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "asnn.h"

namespace asnn {

constexpr int kWave = 64;   // CDNA wavefront width

// Records the hipError_t behind ASNN_ERR_HIP for asnn_last_hip_error().
void set_last_hip_error(hipError_t e);

#define ASNN_HIP_TRY(expr)                          \
    do {                                            \
        hipError_t _e = (expr);                     \
        if (_e != hipSuccess) {                     \
            ::asnn::set_last_hip_error(_e);         \
            return ASNN_ERR_HIP;                    \
        }                                           \
    } while (0)

#define ASNN_TRY(expr)                              \
    do {                                            \
        int _rc = (expr);                           \
        if (_rc != ASNN_OK) return _rc;             \
    } while (0)

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// ---- work units ---------------------------------------------------------
// Work units of the dataflow schedule, one 16-wavefront workgroup each.  A heavy row (in-degree
// d >= ASNN_HEAVY_INDEGREE) is cut into chunks of its connections, one unit each, so that a row
// with thousands of connections is gathered by several compute units at once instead of round
// after round by one: at most kMaxHeavyChunks chunks of at least kHeavyChunk connections (512
// is one gather round of a workgroup at 64 batch columns; 256 and 1024 both measured slower).
// A medium row is a unit of its own (all 16 wavefronts on it) in levels of fewer than
// kMediumGroupFrom medium rows; in wider levels they go kMediumUnitRows to a unit, 4 wavefronts each
// (a pruned multilayer perceptron is a thousand medium rows per level: as one-row units they take the
// chip's 512 workgroups several rounds with little in each, 35-47 us against 21-25 us at batch widths up to
// 64; a level of 40 such rows runs 15-30 % slower grouped, its rows being what the next level waits for).
// Light rows go kLightUnitRows to a unit, one wavefront each: sixteen fill the workgroup (eight
// measured faster only as long as the polling loop serialised its reloads; now sixteen win at every
// batch width, by 2 % at 64 columns and 12 % at 1024).
constexpr int kHeavyChunk = 512;
constexpr int kMaxHeavyChunks = 16;
constexpr int kMediumUnitRows = 4;
constexpr int kMediumGroupFrom = 256;
constexpr int kLightUnitRows = 16;
__host__ __device__ inline int heavy_chunk_len(int d) {
    const int spread = (d + kMaxHeavyChunks - 1) / kMaxHeavyChunks;
    return spread > kHeavyChunk ? spread : kHeavyChunk;
}
__host__ __device__ inline int heavy_chunks(int d) {
    const int len = heavy_chunk_len(d);
    const int n = (d + len - 1) / len;
    return n > 0 ? n : 1;
}

// Carves 256-byte aligned pieces out of a caller-provided workspace.
struct Carver {
    char *base;
    size_t off = 0;
    explicit Carver(void *p) : base(static_cast<char *>(p)) {}
    template <typename T>
    T *take(size_t count) {
        T *p = reinterpret_cast<T *>(base + off);
        off += align_up(count * sizeof(T));
        return p;
    }
};

// ---- device-wide primitives (prims.hip) --------------------------------
// Exclusive prefix sum of n int32 values; out may alias in.  out[n] is NOT
// written.  tmp must hold scan_tmp_ints(n) ints.
size_t scan_tmp_ints(size_t n);
int exclusive_scan_i32(const int32_t *in, int32_t *out, size_t n, int32_t *tmp, hipStream_t s);

// Stable LSD radix sort of (key, value) pairs on the low `bits` bits of the
// key.  Sorted pairs end in keys_out/vals_out (which may be either of the
// ping-pong buffers: the function reports where).  tmp >= radix_tmp_ints(n).
size_t radix_tmp_ints(size_t n);
int radix_sort_pairs_u32(uint32_t *keys_a, uint32_t *vals_a, uint32_t *keys_b, uint32_t *vals_b,
                         size_t n, int bits, int32_t *tmp, hipStream_t s,
                         uint32_t **keys_sorted, uint32_t **vals_sorted);

// Runs of equal keys in a sorted key array (every key < the length of first/count):
// first[k] = index of the first occurrence of k, count[k] = number of occurrences.  Entries of
// keys that do not occur are left as they are (the caller clears count beforehand).
int sorted_run_lengths(const uint32_t *keys, size_t n, int32_t *first, int32_t *count, hipStream_t s);

inline int bits_for(uint64_t max_value) {   // number of bits needed to hold max_value
    int b = 1;
    while (b < 32 && (max_value >> b) != 0) ++b;
    return b;
}

inline unsigned blocks_for(size_t n, unsigned per_block, unsigned cap = 0x7fffffffu) {
    size_t b = (n + per_block - 1) / per_block;
    if (b < 1) b = 1;
    if (b > cap) b = cap;
    return static_cast<unsigned>(b);
}

}  // namespace asnn
