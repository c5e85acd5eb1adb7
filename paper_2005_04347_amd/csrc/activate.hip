// asnn_activate: level-synchronous activation of a packed ASNN on gfx950.
//
// The paper runs one thread per node of the current layer with a serial loop
// over the node's incoming connections and a block barrier between layers.
// Here the value matrix carries a batch dimension, V[row][b], so the unit of
// work is (row, tile of batch columns): the lanes of a wavefront own batch
// columns, each incoming connection costs one coalesced vector load of the
// source row's tile, and the connection's (col, w) pair is wave-uniform (it is
// fetched once per wave through the scalar path and reused across the whole
// tile).  For narrow batches the 64 lanes split into G groups that walk G
// connections at a time and are folded with a fixed butterfly.  Rows with many
// connections are shared by 4 (medium) or 16 (heavy) wavefronts whose partial
// sums meet in LDS in wave order.  Nothing depends on timing: the same inputs
// give the same bits.  The layer barrier is the boundary between two launches
// on the stream.
//
// Arithmetic: products and sums in ACC (double by default, float with
// ASNN_FLAG_ACC_F32), sigmoid(x) = 1/(1+e^(-4.97x)) in ACC, one rounding to
// float on store.
#include "asnn_common.h"

namespace asnn {

namespace {

constexpr int kMixedBlock = 1024;                    // 16 wavefronts
constexpr int kMixedWaves = kMixedBlock / kWave;
constexpr int kMediumWaves = 4;                      // wavefronts per medium row
constexpr int kUnroll = 8;                           // row tiles in flight per wavefront

template <int VEC> struct Vec;
template <> struct Vec<1> { using type = float; };
template <> struct Vec<2> { using type = float2; };
template <> struct Vec<4> { using type = float4; };

template <int VEC>
__device__ inline void load_vec(const float *p, float (&out)[VEC]) {
    typename Vec<VEC>::type v = *reinterpret_cast<const typename Vec<VEC>::type *>(p);
    if constexpr (VEC == 1) { out[0] = v; }
    if constexpr (VEC == 2) { out[0] = v.x; out[1] = v.y; }
    if constexpr (VEC == 4) { out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w; }
}

template <int VEC>
__device__ inline void store_vec(float *p, const float (&in)[VEC]) {
    typename Vec<VEC>::type v;
    if constexpr (VEC == 1) { v = in[0]; }
    if constexpr (VEC == 2) { v.x = in[0]; v.y = in[1]; }
    if constexpr (VEC == 4) { v.x = in[0]; v.y = in[1]; v.z = in[2]; v.w = in[3]; }
    *reinterpret_cast<typename Vec<VEC>::type *>(p) = v;
}

// sigmoid with the paper's slope.  e^(+big) = inf gives 1/inf = 0, never NaN.
__device__ inline float squash(double s) { return (float)(1.0 / (1.0 + exp(-4.97 * s))); }
__device__ inline float squash(float s) { return 1.0f / (1.0f + __expf(-4.97f * s)); }

// Partial weighted sum of connections [e_begin, e_end) of one row for this
// lane's VEC batch columns starting at column c0 (a valid column, possibly
// clamped).  LPG lanes cover one tile; the 64/LPG lane groups take
// connections round-robin.  On return every lane holds the sum over all groups.
template <int VEC, int LPG, typename ACC, int U>
__device__ inline void row_sum(const int32_t *__restrict__ col, const float *__restrict__ w,
                               const float *__restrict__ V, int B, int e_begin, int e_end, int c0, ACC (&acc)[VEC]) {
    constexpr int G = kWave / LPG;
#pragma unroll
    for (int j = 0; j < VEC; ++j) acc[j] = ACC(0);
    const float *Vc = V + c0;
    if constexpr (G == 1) {
        // (col, w) are wave-uniform: scalar loads; the row base lives in SGPRs.
        int e = e_begin;
        for (; e + U <= e_end; e += U) {
            int cc[U];
            float ww[U];
            float vals[U][VEC];
#pragma unroll
            for (int k = 0; k < U; ++k) { cc[k] = col[e + k]; ww[k] = w[e + k]; }
#pragma unroll
            for (int k = 0; k < U; ++k) load_vec<VEC>(Vc + (size_t)cc[k] * (size_t)B, vals[k]);
#pragma unroll
            for (int k = 0; k < U; ++k)
#pragma unroll
                for (int j = 0; j < VEC; ++j) acc[j] += (ACC)ww[k] * (ACC)vals[k][j];
        }
        const int rem = e_end - e;          // 0 .. U-1, wave-uniform
        if (rem > 0) {
            int cc[U];
            float ww[U];
            float vals[U][VEC];
#pragma unroll
            for (int k = 0; k < U - 1; ++k) {
                const int ek = (k < rem) ? e + k : e;     // clamp: re-read a valid connection
                cc[k] = col[ek];
                ww[k] = w[ek];
            }
#pragma unroll
            for (int k = 0; k < U - 1; ++k) load_vec<VEC>(Vc + (size_t)cc[k] * (size_t)B, vals[k]);
#pragma unroll
            for (int k = 0; k < U - 1; ++k)
                if (k < rem) {
#pragma unroll
                    for (int j = 0; j < VEC; ++j) acc[j] += (ACC)ww[k] * (ACC)vals[k][j];
                }
        }
    } else {
        const int g = (threadIdx.x & (kWave - 1)) / LPG;
        for (int base = e_begin; base < e_end; base += G * U) {
            int cc[U];
            float ww[U];
            bool ok[U];
            float vals[U][VEC];
#pragma unroll
            for (int k = 0; k < U; ++k) {
                const int ek = base + k * G + g;
                ok[k] = ek < e_end;
                cc[k] = ok[k] ? col[ek] : 0;
                ww[k] = ok[k] ? w[ek] : 0.0f;
            }
#pragma unroll
            for (int k = 0; k < U; ++k) load_vec<VEC>(Vc + (size_t)cc[k] * (size_t)B, vals[k]);
#pragma unroll
            for (int k = 0; k < U; ++k)
#pragma unroll
                for (int j = 0; j < VEC; ++j) {
                    const ACC t = acc[j] + (ACC)ww[k] * (ACC)vals[k][j];
                    acc[j] = ok[k] ? t : acc[j];     // a padded slot must not turn 0*inf into NaN
                }
        }
#pragma unroll
        for (int off = LPG; off < kWave; off <<= 1)
#pragma unroll
            for (int j = 0; j < VEC; ++j) acc[j] += __shfl_xor(acc[j], off, kWave);
    }
}

// Light rows: one single-wavefront block per (row, tile).  Rows
// [row_begin, row_end) all belong to one level, so every source row was
// written by an earlier launch.  One wave per block keeps the scheduling
// granularity at a wavefront: a slot frees as soon as its row is done.
template <int VEC, int LPG, typename ACC, int U>
__global__ __launch_bounds__(kWave) void gather_light_kernel(const int32_t *__restrict__ row_ptr,
                                                               const int32_t *__restrict__ col,
                                                               const float *__restrict__ w, float *V, int B,
                                                               int row_begin, int row_end, int tiles_per_row) {
    constexpr int T = LPG * VEC;                 // batch columns per tile
    const int item = blockIdx.x;
    const int row = row_begin + item / tiles_per_row;
    const int tile = item % tiles_per_row;
    if (row >= row_end) return;
    const int lane = threadIdx.x;
    const int c = tile * T + (lane % LPG) * VEC;
    const bool active = c < B;
    const int e0 = row_ptr[row], e1 = row_ptr[row + 1];
    ACC acc[VEC];
    row_sum<VEC, LPG, ACC, U>(col, w, V, B, e0, e1, active ? c : 0, acc);
    if (active && lane < LPG) {
        float out[VEC];
#pragma unroll
        for (int j = 0; j < VEC; ++j) out[j] = squash(acc[j]);
        store_vec<VEC>(V + (size_t)row * (size_t)B + c, out);
    }
}

// A level that holds heavy or medium rows: one launch of 16-wave blocks.
// Blocks [0, heavy_items) take one heavy (row, tile) each, all 16 waves on it;
// the next medium_blocks blocks take four medium (row, tile) items, 4 waves on
// each; the remaining blocks take sixteen light items, one wave each.  The
// waves of one item split its connections into contiguous chunks; partial sums
// meet in LDS and are added in wave order.
template <int VEC, int LPG, typename ACC, int U>
__global__ __launch_bounds__(kMixedBlock) void gather_mixed_kernel(const int32_t *__restrict__ row_ptr,
                                                                    const int32_t *__restrict__ col,
                                                                    const float *__restrict__ w, float *V, int B,
                                                                    int heavy_begin, int medium_begin, int light_begin,
                                                                    int light_end, int tiles_per_row,
                                                                    unsigned heavy_items, unsigned medium_blocks) {
    constexpr int T = LPG * VEC;
    __shared__ ACC part[kMixedWaves][LPG * VEC];
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
    const int lane = threadIdx.x & (kWave - 1);
    int share, row_begin, row_end;      // waves per item, row range of this block's class
    long long item;
    if (blockIdx.x < heavy_items) {
        share = kMixedWaves; row_begin = heavy_begin; row_end = medium_begin;
        item = blockIdx.x;
    } else if (blockIdx.x < heavy_items + medium_blocks) {
        share = kMediumWaves; row_begin = medium_begin; row_end = light_begin;
        item = (long long)(blockIdx.x - heavy_items) * (kMixedWaves / kMediumWaves) + wave / kMediumWaves;
    } else {
        share = 1; row_begin = light_begin; row_end = light_end;
        item = (long long)(blockIdx.x - heavy_items - medium_blocks) * kMixedWaves + wave;
    }
    const long long row_ll = row_begin + item / tiles_per_row;
    const bool valid = row_ll < row_end;          // wave-uniform; invalid waves still reach the barrier
    const int row = valid ? (int)row_ll : row_begin;
    const int tile = (int)(item % tiles_per_row);
    const int c = tile * T + (lane % LPG) * VEC;
    const bool active = valid && c < B;
    const int slice = wave % share;               // which chunk of the row's connections
    ACC acc[VEC];
    if (valid) {
        const int e0 = row_ptr[row], e1 = row_ptr[row + 1];
        const int chunk = (e1 - e0 + share - 1) / share;
        const int b0 = min(e0 + slice * chunk, e1), b1 = min(b0 + chunk, e1);
        row_sum<VEC, LPG, ACC, U>(col, w, V, B, b0, b1, active ? c : 0, acc);
    } else {
#pragma unroll
        for (int j = 0; j < VEC; ++j) acc[j] = ACC(0);
    }
    if (share > 1) {                               // block-uniform
        if (lane < LPG) {
#pragma unroll
            for (int j = 0; j < VEC; ++j) part[wave][lane * VEC + j] = acc[j];
        }
        __syncthreads();
        if (slice == 0 && lane < LPG) {
#pragma unroll
            for (int j = 0; j < VEC; ++j) {
                ACC s = ACC(0);
                for (int k = 0; k < share; ++k) s += part[wave + k][lane * VEC + j];
                acc[j] = s;
            }
        }
    }
    if (active && slice == 0 && lane < LPG) {
        float out[VEC];
#pragma unroll
        for (int j = 0; j < VEC; ++j) out[j] = squash(acc[j]);
        store_vec<VEC>(V + (size_t)row * (size_t)B + c, out);
    }
}

// Sensors: V[row of input_ids[k]][b] = sigmoid(X[k][b]) (or X raw).
template <typename ACC>
__global__ void stage_inputs_kernel(const int32_t *__restrict__ input_ids, const int32_t *__restrict__ inv_perm,
                                    const float *__restrict__ X, float *__restrict__ V, int32_t n_inputs,
                                    int32_t n_nodes, int B, int raw) {
    const int64_t total = (int64_t)n_inputs * B;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        const int k = (int)(i / B), b = (int)(i % B);
        const int32_t id = input_ids[k];
        if (id < 0 || id >= n_nodes) continue;
        const float x = X[i];
        V[(size_t)inv_perm[id] * (size_t)B + b] = raw ? x : squash((ACC)x);
    }
}

__global__ void extract_outputs_kernel(const int32_t *__restrict__ output_ids, const int32_t *__restrict__ inv_perm,
                                       const float *__restrict__ V, float *__restrict__ Y, int32_t n_outputs,
                                       int32_t n_nodes, int B) {
    const int64_t total = (int64_t)n_outputs * B;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        const int o = (int)(i / B), b = (int)(i % B);
        const int32_t id = output_ids[o];
        Y[i] = (id < 0 || id >= n_nodes) ? __builtin_nanf("") : V[(size_t)inv_perm[id] * (size_t)B + b];
    }
}

struct LevelArgs {
    const int32_t *row_ptr;
    const int32_t *col;
    const float *w;
    float *V;
    int B;
    hipStream_t s;
};

// One level: rows [hb, mb) heavy, [mb, lb) medium, [lb, le) light.
template <int VEC, int LPG, typename ACC>
int launch_level(const LevelArgs &a, int hb, int mb, int lb, int le) {
    const int vecs = a.B / VEC;
    const int tiles = (vecs + LPG - 1) / LPG;
    if (le <= hb) return ASNN_OK;
    if (lb == hb) {      // light rows only
        const long long items = (long long)(le - lb) * tiles;
        if (items > 0x7fffffffLL) return ASNN_ERR_SIZE;
        hipLaunchKernelGGL((gather_light_kernel<VEC, LPG, ACC, kUnroll>), dim3((unsigned)items), dim3(kWave), 0, a.s,
                           a.row_ptr, a.col, a.w, a.V, a.B, lb, le, tiles);
        ASNN_HIP_TRY(hipGetLastError());
        return ASNN_OK;
    }
    const long long heavy_items = (long long)(mb - hb) * tiles;
    const long long medium_items = (long long)(lb - mb) * tiles;
    const long long light_items = (long long)(le - lb) * tiles;
    const int per_block = kMixedWaves / kMediumWaves;
    const long long medium_blocks = (medium_items + per_block - 1) / per_block;
    const long long light_blocks = (light_items + kMixedWaves - 1) / kMixedWaves;
    const long long blocks = heavy_items + medium_blocks + light_blocks;
    if (blocks > 0x7fffffffLL) return ASNN_ERR_SIZE;
    hipLaunchKernelGGL((gather_mixed_kernel<VEC, LPG, ACC, kUnroll>), dim3((unsigned)blocks), dim3(kMixedBlock), 0, a.s,
                       a.row_ptr, a.col, a.w, a.V, a.B, hb, mb, lb, le, tiles, (unsigned)heavy_items,
                       (unsigned)medium_blocks);
    ASNN_HIP_TRY(hipGetLastError());
    return ASNN_OK;
}

template <int VEC, typename ACC>
int launch_level_vec(const LevelArgs &a, int hb, int mb, int lb, int le) {
    const int vecs = a.B / VEC;
    if (vecs > 32) return launch_level<VEC, 64, ACC>(a, hb, mb, lb, le);
    if (vecs > 16) return launch_level<VEC, 32, ACC>(a, hb, mb, lb, le);
    if (vecs > 8) return launch_level<VEC, 16, ACC>(a, hb, mb, lb, le);
    if (vecs > 4) return launch_level<VEC, 8, ACC>(a, hb, mb, lb, le);
    if (vecs > 2) return launch_level<VEC, 4, ACC>(a, hb, mb, lb, le);
    if (vecs > 1) return launch_level<VEC, 2, ACC>(a, hb, mb, lb, le);
    return launch_level<VEC, 1, ACC>(a, hb, mb, lb, le);
}

template <typename ACC>
int launch_level_any(const LevelArgs &a, int hb, int mb, int lb, int le) {
    if (a.B % 4 == 0) return launch_level_vec<4, ACC>(a, hb, mb, lb, le);
    if (a.B % 2 == 0) return launch_level_vec<2, ACC>(a, hb, mb, lb, le);
    return launch_level_vec<1, ACC>(a, hb, mb, lb, le);
}

}  // namespace
}  // namespace asnn

using namespace asnn;

extern "C" int asnn_activate(int32_t n_nodes, int64_t n_edges, int32_t n_levels, const int32_t *level_ptr_host,
                             const int32_t *row_ptr, const int32_t *col, const float *w_packed,
                             const int32_t *inv_perm, const int32_t *input_ids, int32_t n_inputs,
                             const int32_t *output_ids, int32_t n_outputs, const float *X, int32_t B, float *V,
                             float *Y, uint32_t flags, void *stream) {
    if (n_nodes <= 0 || n_edges < 0 || n_edges >= (int64_t)INT32_MAX || n_levels <= 0 || n_inputs < 0 ||
        n_outputs < 0 || B <= 0)
        return ASNN_ERR_SIZE;
    if ((int64_t)n_nodes * (int64_t)B >= ((int64_t)1 << 40)) return ASNN_ERR_SIZE;
    if (!level_ptr_host || !row_ptr || !inv_perm || !V) return ASNN_ERR_NULL;
    if (n_edges > 0 && (!col || !w_packed)) return ASNN_ERR_NULL;
    if (n_inputs > 0 && (!input_ids || !X)) return ASNN_ERR_NULL;
    if (Y && n_outputs > 0 && !output_ids) return ASNN_ERR_NULL;
    if (((uintptr_t)V & 15u) != 0) return ASNN_ERR_SIZE;
    // the level table must be a monotone cover of the rows
    const int n_keys = ASNN_CLASSES * n_levels;
    if (level_ptr_host[0] != 0 || level_ptr_host[n_keys] != n_nodes) return ASNN_ERR_SIZE;
    for (int k = 0; k < n_keys; ++k)
        if (level_ptr_host[k] > level_ptr_host[k + 1]) return ASNN_ERR_SIZE;

    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool f32 = (flags & ASNN_FLAG_ACC_F32) != 0;
    const int raw = (flags & ASNN_FLAG_RAW_INPUTS) ? 1 : 0;
    LevelArgs a{row_ptr, col, w_packed, V, B, s};

    for (int l = 0; l < n_levels; ++l) {
        const int32_t *lp = level_ptr_host + ASNN_CLASSES * l;
        const int hb = lp[0], mb = lp[1], lb = lp[2], le = lp[3];
        if (l == 0) {
            // Level 0 has no incoming connections.  Rows that are no sensors get
            // sigmoid(0); when every row of the level is a sensor the fill is skipped.
            if (le - hb != n_inputs)
                ASNN_TRY(f32 ? launch_level_any<float>(a, hb, mb, lb, le) : launch_level_any<double>(a, hb, mb, lb, le));
            if (n_inputs > 0) {
                const unsigned blocks = blocks_for((size_t)n_inputs * (size_t)B, 256, 8192);
                if (f32)
                    hipLaunchKernelGGL(stage_inputs_kernel<float>, dim3(blocks), dim3(256), 0, s, input_ids, inv_perm, X,
                                       V, n_inputs, n_nodes, B, raw);
                else
                    hipLaunchKernelGGL(stage_inputs_kernel<double>, dim3(blocks), dim3(256), 0, s, input_ids, inv_perm,
                                       X, V, n_inputs, n_nodes, B, raw);
                ASNN_HIP_TRY(hipGetLastError());
            }
            continue;
        }
        ASNN_TRY(f32 ? launch_level_any<float>(a, hb, mb, lb, le) : launch_level_any<double>(a, hb, mb, lb, le));
    }
    if (Y && n_outputs > 0) {
        const unsigned blocks = blocks_for((size_t)n_outputs * (size_t)B, 256, 8192);
        hipLaunchKernelGGL(extract_outputs_kernel, dim3(blocks), dim3(256), 0, s, output_ids, inv_perm,
                           (const float *)V, Y, n_outputs, n_nodes, B);
        ASNN_HIP_TRY(hipGetLastError());
    }
    return ASNN_OK;
}
