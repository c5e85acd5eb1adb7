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
// connections are shared by 8 (medium) or 16 (heavy) wavefronts whose partial
// sums meet in LDS in wave order.  Nothing depends on timing: the same inputs
// give the same bits.
//
// Three schedules provide the layer barrier (all produce identical values):
//   level launches  the boundary between two launches on the stream;
//   dataflow        one persistent launch in which a row waits only for its own
//                   source rows (for deep networks with small layers);
//   workgroup       the paper's arrangement, one workgroup per tile of batch
//                   columns walking all layers behind a workgroup barrier, in
//                   one launch (for small networks and narrow batches).
//
// Arithmetic: products and sums in ACC (double by default, float with
// ASNN_FLAG_ACC_F32), sigmoid(x) = 1/(1+e^(-4.97x)) in ACC, one rounding to
// float on store.
#include <atomic>

#include "asnn_common.h"

namespace asnn {

namespace {

constexpr int kMixedBlock = 1024;                    // 16 wavefronts
constexpr int kMaxDevices = 64;                       // per-device caches of launch parameters
constexpr int kMixedWaves = kMixedBlock / kWave;
constexpr int kMediumWaves = 8;                      // wavefronts per medium row in a level launch
constexpr int kUnroll = 8;                           // row tiles in flight per wavefront
constexpr int kXcds = 8;                             // accelerator dies: workgroup i of a launch runs on die i % 8

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

// sigmoid with the paper's slope, 1 / (1 + e^(-4.97 s)), the fp64 value rounded to float.
// Where one wavefront's sigmoid sits between two levels its chain of dependent instructions is what
// the level waits for, and a library exponential followed by a full fp64 division is about 45
// deep.  Written out: e^y = 2^k e^r with k = round(y / ln 2), e^r by its Taylor series to r^13
// (|r| <= 0.347: the next term is below 5e-18), the reciprocal by the hardware's estimate and two
// Newton steps (none of the division's scaling and fix-up: the denominator is in [1, 1e308]); a few
// ulp of fp64, far inside the float the result is rounded to.  (Estrin's scheme for the series is
// another 1.5 % shorter per level at one input vector and costs the bandwidth-bound kernels 0.8 %.)
// y is kept in [-745, 709]: beyond, e^y is 0 or would overflow, and the float result is exactly 1 or
// 0 already at the bounds.  NaN stays NaN.
__device__ inline float squash(double s) {
    double y = -4.97 * s;
    y = y > 709.0 ? 709.0 : y;
    y = y < -745.0 ? -745.0 : y;
    const double k = __builtin_rint(y * 1.4426950408889634074);
    double r = __builtin_fma(k, -6.93147180369123816490e-01, y);     // ln 2, high part (k * it is exact)
    r = __builtin_fma(k, -1.90821492927058770002e-10, r);            // low part
    double p = 1.0 / 6227020800.0;
    p = __builtin_fma(p, r, 1.0 / 479001600.0);
    p = __builtin_fma(p, r, 1.0 / 39916800.0);
    p = __builtin_fma(p, r, 1.0 / 3628800.0);
    p = __builtin_fma(p, r, 1.0 / 362880.0);
    p = __builtin_fma(p, r, 1.0 / 40320.0);
    p = __builtin_fma(p, r, 1.0 / 5040.0);
    p = __builtin_fma(p, r, 1.0 / 720.0);
    p = __builtin_fma(p, r, 1.0 / 120.0);
    p = __builtin_fma(p, r, 1.0 / 24.0);
    p = __builtin_fma(p, r, 1.0 / 6.0);
    p = __builtin_fma(p, r, 0.5);
    p = __builtin_fma(p, r, 1.0);
    p = __builtin_fma(p, r, 1.0);
    const double e = __builtin_ldexp(p, (int)k);
    const double d = 1.0 + e;
    double x = __builtin_amdgcn_rcp(d);
    x = __builtin_fma(x, __builtin_fma(-d, x, 1.0), x);
    x = __builtin_fma(x, __builtin_fma(-d, x, 1.0), x);
    return (float)x;
}
// (fast mode: hardware exponential and reciprocal, about an ulp each; e^(+big) = inf gives 0, never NaN)
__device__ inline float squash(float s) { return __builtin_amdgcn_rcpf(1.0f + __expf(-4.97f * s)); }

// ---- sums across the lane groups of a wavefront ---------------------------
// Value of the lane SHIFT places further on in the same row of 16 lanes, wrapping round: one DPP
// move per dword.
template <int SHIFT>
__device__ inline float from_lane_rotated(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x120 + SHIFT, 0xf, 0xf, false));
}
template <int SHIFT>
__device__ inline double from_lane_rotated(double x) {
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(x), 0x120 + SHIFT, 0xf, 0xf, false);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(x), 0x120 + SHIFT, 0xf, 0xf, false);
    return __hiloint2double(hi, lo);
}

// x plus the value of the same lane in the partner row (rows of 16 lanes: 0 with 1, 2 with 3), and
// in the partner half of the wavefront: the lane-swap instructions of gfx950 hand each lane both.
__device__ inline float plus_partner_row(float x) {
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ inline double plus_partner_row(double x) {
    const unsigned lo = (unsigned)__double2loint(x), hi = (unsigned)__double2hiint(x);
    const auto rl = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
    const auto rh = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
    return __hiloint2double((int)rh[0], (int)rl[0]) + __hiloint2double((int)rh[1], (int)rl[1]);
}
__device__ inline float plus_partner_half(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ inline double plus_partner_half(double x) {
    const unsigned lo = (unsigned)__double2loint(x), hi = (unsigned)__double2hiint(x);
    const auto rl = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
    const auto rh = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
    return __hiloint2double((int)rh[0], (int)rl[0]) + __hiloint2double((int)rh[1], (int)rl[1]);
}

// Sum over the lane groups of a team (16 consecutive lanes, 16/LPG groups of LPG lanes each),
// pairwise at distances 8, 4, ... LPG.  Every group ends up with the same total.
template <int VEC, int LPG, typename ACC>
__device__ inline void team_sum(ACC (&acc)[VEC]) {
#pragma unroll
    for (int j = 0; j < VEC; ++j) {
        if constexpr (LPG <= 8) acc[j] += from_lane_rotated<8>(acc[j]);
        if constexpr (LPG <= 4) acc[j] += from_lane_rotated<4>(acc[j]);
        if constexpr (LPG <= 2) acc[j] += from_lane_rotated<2>(acc[j]);
        if constexpr (LPG <= 1) acc[j] += from_lane_rotated<1>(acc[j]);
    }
}

// Sum over all 64/LPG lane groups of the wavefront: inside the rows of 16 lanes first, then the
// rows pairwise, then the halves.  Every group ends up with the same total; all vector-ALU moves
// (shuffles through the LDS crossbar cost a round trip per step).
template <int VEC, int LPG, typename ACC>
__device__ inline void wave_sum(ACC (&acc)[VEC]) {
    team_sum<VEC, LPG, ACC>(acc);
#pragma unroll
    for (int j = 0; j < VEC; ++j) {
        if constexpr (LPG <= 16) acc[j] = plus_partner_row(acc[j]);
        if constexpr (LPG <= 32) acc[j] = plus_partner_half(acc[j]);
    }
}

// Partial weighted sum of connections [e_begin, e_end) of one row for this
// lane's VEC batch columns starting at column c0 (a valid column, possibly
// clamped).  LPG lanes cover one tile; the 64/LPG lane groups take
// connections round-robin.  On return every lane holds the sum over all groups.
template <int VEC, int LPG, typename ACC, int U, bool EXACT_TAIL = false>
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
        if constexpr (EXACT_TAIL) {
            // The remaining connections go in blocks of U/2, U/4, ... 1: first the gathers of every
            // block that is there, then their sums in the same order, each block behind a scalar
            // branch.  Against the padded round below that is 3.5 gathers, conversions and sums on
            // average instead of U-1, and no selects: 0.7 % on the 100k-node workload and 1.5 % on the
            // population, where a wavefront has one row and the vector ALU is busy more than half the
            // time.  Each block waits for its own (col, w), though, which costs a short-lived
            // workgroup of medium rows more than it saves (the pruned MLP: +8 %).
            float ww[U];
            float vals[U][VEC];
            int at = 0;
#pragma unroll
            for (int size = U / 2; size >= 1; size /= 2) {
                if (rem & size) {
                    int cc[U / 2];
#pragma unroll
                    for (int k = 0; k < size; ++k) {
                        cc[k] = col[e + at + k];
                        ww[size - 1 + k] = w[e + at + k];
                    }
#pragma unroll
                    for (int k = 0; k < size; ++k) load_vec<VEC>(Vc + (size_t)cc[k] * (size_t)B, vals[size - 1 + k]);
                    at += size;
                }
            }
#pragma unroll
            for (int size = U / 2; size >= 1; size /= 2) {
                if (rem & size) {
#pragma unroll
                    for (int k = 0; k < size; ++k)
#pragma unroll
                        for (int j = 0; j < VEC; ++j) acc[j] += (ACC)ww[size - 1 + k] * (ACC)vals[size - 1 + k][j];
                }
            }
        } else if (rem > 0) {
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
        // UG slots per group and round: 32 connections or more per round for every G >= 4 (a
        // medium row of a narrow batch would leave most of 8 slots per group padded).
        constexpr int UG = G >= 16 ? 2 : (G >= 8 ? 4 : U);
        const int g = (threadIdx.x & (kWave - 1)) / LPG;
        for (int base = e_begin; base < e_end; base += G * UG) {
            int cc[UG];
            float ww[UG];
            float vals[UG][VEC];
#pragma unroll
            for (int k = 0; k < UG; ++k) {
                const int ek = min(base + k * G + g, e_end - 1);      // padded slots re-read the last connection
                cc[k] = col[ek];
                ww[k] = w[ek];
            }
#pragma unroll
            for (int k = 0; k < UG; ++k) load_vec<VEC>(Vc + (size_t)cc[k] * (size_t)B, vals[k]);
#pragma unroll
            for (int k = 0; k < UG; ++k)
#pragma unroll
                for (int j = 0; j < VEC; ++j) {
                    const ACC t = acc[j] + (ACC)ww[k] * (ACC)vals[k][j];
                    acc[j] = (base + k * G + g < e_end) ? t : acc[j];     // a padded slot adds nothing
                }
        }
        wave_sum<VEC, LPG, ACC>(acc);
    }
}

// Light rows: one single-wavefront block per (row, tile).  Rows
// [row_begin, row_end) all belong to one level, so every source row was
// written by an earlier launch.  One wave per block keeps the scheduling
// granularity at a wavefront: a slot frees as soon as its row is done.
//
// Block -> (row, tile) is row-major on purpose.  Workgroups are dealt to the
// 8 XCDs round-robin, so with t tiles per row XCD x only ever gathers the
// column tiles congruent to x modulo gcd(t, 8): with 8 tiles (1024 columns of
// float2) each XCD's L2 sees one eighth of V.  Rotating the tile index by the
// row, which shows every tile to every XCD, costs 14 % on the 100k-node
// workload.  Padding an odd tile count to an even one is not worth it: a
// block that exits at once still takes a dispatch slot, and the launch rate
// of single-wavefront blocks is within 3x of the dispatcher's.  Tile counts
// that are no multiple of 8 get the alignment from the order of the items
// instead (items_per_xcd, below): 4-8 % on batch widths of 3, 5, 6, 7, 9, 10
// tiles.
template <int VEC, int LPG, typename ACC, int U>
__global__ __launch_bounds__(kWave) void gather_light_kernel(const int32_t *__restrict__ row_ptr,
                                                               const int32_t *__restrict__ col,
                                                               const float *__restrict__ w, float *V, int B,
                                                               int row_begin, int row_end, int tiles_per_row,
                                                               int items_per_xcd) {
    constexpr int T = LPG * VEC;                 // batch columns per tile
    int row, tile;
    if (items_per_xcd == 0) {                    // tile counts that the round-robin aligns by itself
        const int item = blockIdx.x;
        row = row_begin + item / tiles_per_row;
        tile = item % tiles_per_row;
        if (row >= row_end) return;
    } else {
        // Any other tile count (3, 5, 6 ... tiles): the (tile, row) items in tile-major order are cut into
        // eight equal runs and XCD x (the workgroups congruent to x modulo 8) walks run x, so that it
        // gathers from at most two column tiles (one more per eight tiles) instead of from all of them.
        const int rows = row_end - row_begin;
        const long long q = (long long)(blockIdx.x % kXcds) * items_per_xcd + blockIdx.x / kXcds;
        if (q >= (long long)rows * tiles_per_row) return;
        tile = (int)(q / rows);
        row = row_begin + (int)(q % rows);
    }
    const int lane = threadIdx.x;
    const int c = tile * T + (lane % LPG) * VEC;
    const bool active = c < B;
    const int e0 = row_ptr[row], e1 = row_ptr[row + 1];
    ACC acc[VEC];
    row_sum<VEC, LPG, ACC, U, true>(col, w, V, B, e0, e1, active ? c : 0, acc);
    if (active && lane < LPG) {
        float out[VEC];
#pragma unroll
        for (int j = 0; j < VEC; ++j) out[j] = squash(acc[j]);
        store_vec<VEC>(V + (size_t)row * (size_t)B + c, out);
    }
}

// A level that holds heavy or medium rows: one launch of 16-wave blocks.
// Blocks [0, heavy_items) take one heavy (row, tile) each, all 16 waves on it;
// the next medium_blocks blocks take two medium (row, tile) items, 8 waves on
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


// ---------------------------------------------------------------- dataflow
// One persistent launch instead of one launch per level.  Workgroups claim
// work items (unit, tile) in packed order from a global counter.  Before the
// launch every row above level 0 is filled with a signalling-NaN pattern that
// no arithmetic result can have; a wavefront gathers its source tiles and
// simply re-reads those that still show the pattern, so the data is its own
// ready flag and a row costs one device-scope round trip after its last
// source, not a flag round trip plus a data round trip.  An item only waits
// for items with a smaller index, and an item is claimed by a running
// workgroup after every smaller item was claimed, so the smallest unfinished
// item never waits for anything: no deadlock for any grid size.
//
// Cross-workgroup visibility without cache flushes: V tiles are read and
// written with device-scope (sc1) accesses, which bypass the per-XCD L2 for
// lines that another XCD may have written.
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));
constexpr int kAuxDeviceScope = 16;                 // cache-policy bit sc1
constexpr int kBufferFlags = 0x27000;               // raw 32-bit buffer, gfx9 descriptor word 3
constexpr long long kWaitTicks = 200000000LL;       // 2 s of the 100 MHz wall clock
// "Not written yet": exponent all ones, quiet bit clear, payload set.  Arithmetic only ever
// produces quiet NaNs, so no stored activation has these bits.
constexpr unsigned int kNotReady = 0x7fa5c0deu;

struct DataflowCtl {
    int head;       // next work item
    int error;      // raised when a wait gave up
    int magic;      // kCtlMagic once a dataflow launch has reset this block (the workspace may arrive uninitialised)
    int pad[61];
};
constexpr int kCtlMagic = 0x41534e4e;

// Tiles of V travel with device scope (sc1) and 64-bit addresses: a value matrix may exceed the
// 4 GiB that the 32-bit offsets of a buffer descriptor cover.  16 bytes per lane through the scoped
// 128-bit global load / store, 8 and 4 bytes as relaxed atomics of that scope (the same instructions
// with the sc1 bit).
typedef __attribute__((address_space(1))) uintx4 *global_uintx4_ptr;
template <int VEC>
__device__ inline void load_vec_device_scope(const float *p, float (&out)[VEC]) {
    if constexpr (VEC == 4) {
        const floatx4 v = __builtin_bit_cast(floatx4, __builtin_amdgcn_global_load_b128((global_uintx4_ptr)const_cast<float *>(p), "agent"));
        out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
    }
    if constexpr (VEC == 2) {
        const floatx2 v = __builtin_bit_cast(floatx2, __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        out[0] = v.x; out[1] = v.y;
    }
    if constexpr (VEC == 1) {
        out[0] = __builtin_bit_cast(float, __hip_atomic_load(reinterpret_cast<const unsigned int *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    }
}

template <int VEC>
__device__ inline void store_vec_device_scope(float *p, const float (&in)[VEC]) {
    if constexpr (VEC == 4) {
        const floatx4 v = {in[0], in[1], in[2], in[3]};
        __builtin_amdgcn_global_store_b128((global_uintx4_ptr)p, __builtin_bit_cast(uintx4, v), "agent");
    }
    if constexpr (VEC == 2) {
        const floatx2 v = {in[0], in[1]};
        __hip_atomic_store(reinterpret_cast<unsigned long long *>(p), __builtin_bit_cast(unsigned long long, v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if constexpr (VEC == 1) {
        __hip_atomic_store(reinterpret_cast<unsigned int *>(p), __builtin_bit_cast(unsigned int, in[0]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// True when one of the values still holds the not-ready pattern.  Written as a minimum over
// (bits xor pattern) on purpose: an `or` over VEC comparisons was compiled into two dozen
// instructions per tile, and a polling pass looks at 8 tiles.
template <int VEC>
__device__ inline bool shows_not_ready(const float (&v)[VEC]) {
    unsigned int m = __builtin_bit_cast(unsigned int, v[0]) ^ kNotReady;
#pragma unroll
    for (int j = 1; j < VEC; ++j) m = min(m, __builtin_bit_cast(unsigned int, v[j]) ^ kNotReady);
    return m == 0u;
}

// Partial sums of the chunks of a split heavy row travel through the workspace in ACC precision,
// marked "not written yet" the same way.  For double the pattern sits in the high word, where it
// reads as a number near 7e306: no sum of products of floats comes anywhere near (at most
// 2^128 * 2^128 per product), so it cannot be taken for a value either.
template <typename ACC> struct PartialBits;
template <> struct PartialBits<float> {
    __device__ static inline float load(__amdgpu_buffer_rsrc_t r, uint32_t off, bool &ready) {
        const unsigned int b = __builtin_amdgcn_raw_buffer_load_b32(r, off, 0, kAuxDeviceScope);
        ready = b != kNotReady;
        return __builtin_bit_cast(float, b);
    }
    __device__ static inline void store(__amdgpu_buffer_rsrc_t r, uint32_t off, float v) {
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned int, v), r, off, 0, kAuxDeviceScope);
    }
};
template <> struct PartialBits<double> {
    __device__ static inline double load(__amdgpu_buffer_rsrc_t r, uint32_t off, bool &ready) {
        const uintx2 b = __builtin_amdgcn_raw_buffer_load_b64(r, off, 0, kAuxDeviceScope);
        ready = b.y != kNotReady;
        return __builtin_bit_cast(double, b);
    }
    __device__ static inline void store(__amdgpu_buffer_rsrc_t r, uint32_t off, double v) {
        __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(uintx2, v), r, off, 0, kAuxDeviceScope);
    }
};

// Bounded back-off between two attempts to read a tile that is not written yet.
// Returns false when the wait must be abandoned (time limit, or another wave gave up).
struct Patience {
    long long t0 = 0;
    int spins = 0;
    __device__ inline bool again(DataflowCtl *ctl) {
        if (spins == 0) t0 = wall_clock64();
        __builtin_amdgcn_s_sleep(1);
        if ((++spins & 63) == 0) {
            const int err = __hip_atomic_load(&ctl->error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (err != 0 || wall_clock64() - t0 > kWaitTicks) {
                __hip_atomic_store(&ctl->error, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                return false;
            }
        }
        return true;
    }
};

// row_sum for the dataflow schedule: connections are taken 64 at a time (one
// per lane) and gathered with device-scope loads; tiles of rows at or above
// first_row that still hold the not-ready pattern are read again.
template <int VEC, int LPG, typename ACC, int U>
__device__ inline void row_sum_dataflow(const int32_t *__restrict__ col, const float *__restrict__ w,
                                        const float *V, int B, int e_begin, int e_end, int c0, int first_row,
                                        DataflowCtl *ctl, ACC (&acc)[VEC]) {
    constexpr int G = kWave / LPG;
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int j = 0; j < VEC; ++j) acc[j] = ACC(0);
    Patience patience;
    for (int eb = e_begin; eb < e_end; eb += kWave) {
        const int n = min(kWave, e_end - eb);
        const int my = eb + min(lane, n - 1);
        const int mc = col[my];
        const float mw = (lane < n) ? w[my] : 0.0f;
        if constexpr (G == 1) {
            for (int i = 0; i < n; i += U) {
                float vals[U][VEC];
                float ww[U];
                const float *at[U];     // this lane's part of the source tile
                bool watch[U];          // wave-uniform: a real connection whose source is above level 0
#pragma unroll
                for (int k = 0; k < U; ++k) {
                    const int idx = min(i + k, n - 1);
                    const int ck = __builtin_amdgcn_readlane(mc, idx);
                    ww[k] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, mw), idx));
                    at[k] = V + (size_t)ck * (size_t)B + (size_t)c0;
                    watch[k] = (i + k < n) && ck >= first_row;
                    load_vec_device_scope<VEC>(at[k], vals[k]);
                }
                for (;;) {      // look at every slot first, then request the missing tiles again (see below)
                    bool again[U];      // wave-uniform
                    bool retry = false;
#pragma unroll
                    for (int k = 0; k < U; ++k) {
                        again[k] = watch[k] && __any(shows_not_ready<VEC>(vals[k]));
                        retry = retry || again[k];
                    }
                    if (!retry) break;
#pragma unroll
                    for (int k = 0; k < U; ++k)
                        if (again[k]) load_vec_device_scope<VEC>(at[k], vals[k]);
                    if (!patience.again(ctl)) break;
                }
#pragma unroll
                for (int k = 0; k < U; ++k)
                    if (i + k < n) {        // wave-uniform
#pragma unroll
                        for (int j = 0; j < VEC; ++j) acc[j] += (ACC)ww[k] * (ACC)vals[k][j];
                    }
            }
        } else {
            // UD slots per lane group and round: with many groups (a narrow batch) one, two or four
            // cover the 64 connections of a pass; more would be padding that is loaded and looked at all the same.
            constexpr int UD = kWave / G < U ? kWave / G : U;
            const int g = lane / LPG;
            for (int i = 0; i < n; i += G * UD) {
                float vals[UD][VEC];
                float ww[UD];
                const float *at[UD];
                bool ok[UD], watch[UD];   // per lane group
#pragma unroll
                for (int k = 0; k < UD; ++k) {
                    const int idx = i + k * G + g;
                    ok[k] = idx < n;
                    const int sel = min(idx, n - 1);
                    const int ck = __shfl(mc, sel, kWave);
                    ww[k] = __shfl(mw, sel, kWave);
                    at[k] = V + (size_t)ck * (size_t)B + (size_t)c0;
                    watch[k] = ok[k] && ck >= first_row;
                    load_vec_device_scope<VEC>(at[k], vals[k]);     // padded slots re-read a valid tile
                }
                // All slots are looked at first (which takes every load of the last pass), then the
                // tiles that are still missing are requested again back to back: measured 6 % faster on the
                // deep workload than looking at a slot and requesting it again one slot at a time.
                for (;;) {
                    bool again[UD];
                    bool mine = false;
#pragma unroll
                    for (int k = 0; k < UD; ++k) {
                        again[k] = watch[k] && shows_not_ready<VEC>(vals[k]);
                        mine = mine || again[k];
                    }
                    if (!__any(mine)) break;
#pragma unroll
                    for (int k = 0; k < UD; ++k)
                        if (again[k]) load_vec_device_scope<VEC>(at[k], vals[k]);
                    if (!patience.again(ctl)) break;
                }
#pragma unroll
                for (int k = 0; k < UD; ++k)
#pragma unroll
                    for (int j = 0; j < VEC; ++j) {
                        const ACC t = acc[j] + (ACC)ww[k] * (ACC)vals[k][j];
                        acc[j] = ok[k] ? t : acc[j];
                    }
            }
        }
    }
    if constexpr (G >= 16) {
        wave_sum<VEC, LPG, ACC>(acc);
    } else if constexpr (G > 1) {
        // (up to three steps: shuffles; the lane-swap sum measured 1.7 % slower on the deep workload, two steps)
#pragma unroll
        for (int off = LPG; off < kWave; off <<= 1)
#pragma unroll
            for (int j = 0; j < VEC; ++j) acc[j] += __shfl_xor(acc[j], off, kWave);
    }
}

// Marks every value of rows [first_row, n_nodes) and every partial-sum word as not written and
// resets the control block.  (For double partial sums every 32-bit word gets the pattern: the
// high word is the one that is tested.)
__global__ void dataflow_reset_kernel(unsigned int *v_begin, size_t n_values, unsigned int *partial_words,
                                      size_t n_partial_words, DataflowCtl *ctl) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_values; i += stride) v_begin[i] = kNotReady;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_partial_words; i += stride)
        partial_words[i] = kNotReady;
    if (blockIdx.x == 0 && threadIdx.x < 64)
        reinterpret_cast<int *>(ctl)[threadIdx.x] = (threadIdx.x == 2) ? kCtlMagic : 0;
}

// Partial-sum slot of chunk 0 of a split heavy row whose connections start at e_begin: split rows
// have more than kHeavyChunk connections and at most one chunk per kHeavyChunk of them, so
// slots of kHeavyChunk/2 connections never collide between two rows.
__host__ __device__ inline uint32_t partial_slot(int e_begin) { return (uint32_t)e_begin / (kHeavyChunk / 2); }

template <int VEC, int LPG, typename ACC, int U>
__global__ __launch_bounds__(kMixedBlock) void dataflow_kernel(const int32_t *__restrict__ row_ptr,
                                                                const int32_t *__restrict__ col,
                                                                const float *__restrict__ w, float *V,
                                                                int B, const int32_t *__restrict__ unit_ptr,
                                                                int first_unit, int n_work, int tiles, int first_row,
                                                                DataflowCtl *ctl, void *partials, uint32_t partial_bytes,
                                                                const int32_t *__restrict__ output_ids,
                                                                const int32_t *__restrict__ inv_perm,
                                                                float *__restrict__ Y, int n_outputs, int n_nodes) {
    constexpr int T = LPG * VEC;
    constexpr int E = T >= kWave ? T / kWave : 1;       // tile elements per lane when one wavefront holds the tile
    constexpr int EL = T >= kWave ? kWave : T;          // lanes that hold them
    __shared__ ACC part[kMixedWaves][T];
    __shared__ ACC others[kMaxHeavyChunks - 1][T];      // partial sums of the other chunks of a split row
    __shared__ int s_claim;
    const __amdgpu_buffer_rsrc_t pres = __builtin_amdgcn_make_buffer_rsrc(partials, 0, (int)partial_bytes, kBufferFlags);
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
    const int lane = threadIdx.x & (kWave - 1);
    for (;;) {
        if (threadIdx.x == 0)
            s_claim = __hip_atomic_fetch_add(&ctl->head, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        const int q = s_claim;
        __syncthreads();
        if (q >= n_work) {                            // block-uniform
            // The items behind the last row copy the output rows to Y, 16 outputs (one per wavefront)
            // by one tile each.  They wait for their rows like any other item (and are claimed last).
            const int x = q - n_work;
            if (x >= ((n_outputs + kMixedWaves - 1) / kMixedWaves) * tiles) return;
            const int o = (x / tiles) * kMixedWaves + wave;
            const int c = (x % tiles) * T + (lane % LPG) * VEC;
            if (o < n_outputs && lane < LPG && c < B) {
                const int32_t id = output_ids[o];
                float out[VEC];
                if (id >= 0 && id < n_nodes) {
                    const int32_t row = inv_perm[id];
                    const float *at = V + (size_t)row * (size_t)B + (size_t)c;
                    Patience patience;
                    for (;;) {
                        load_vec_device_scope<VEC>(at, out);
                        if (row < first_row || !shows_not_ready<VEC>(out) || !patience.again(ctl)) break;
                    }
                    // A wait that was given up anywhere leaves rows computed from unwritten sources:
                    // the outputs copied from then on say so themselves instead of looking like results.
                    if (__hip_atomic_load(&ctl->error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
#pragma unroll
                        for (int j = 0; j < VEC; ++j) out[j] = __builtin_nanf("");
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < VEC; ++j) out[j] = __builtin_nanf("");
                }
                store_vec<VEC>(Y + (size_t)o * (size_t)B + c, out);
            }
            continue;
        }
        const int u = first_unit + q / tiles;
        const int tile = q % tiles;
        const int r0 = unit_ptr[u], r1 = unit_ptr[u + 1];
        const int row0_begin = row_ptr[r0], row0_end = row_ptr[r0 + 1];
        const int d0 = row0_end - row0_begin;
        const bool heavy = d0 >= ASNN_HEAVY_INDEGREE;
        // wavefronts on one row: 16 on a heavy row, 16, 8 or 4 on the 1, 2 or 3-4 medium rows of a unit, 1 on a light row
        const int share = d0 < ASNN_MEDIUM_INDEGREE ? 1 : (heavy || r1 - r0 == 1) ? kMixedWaves : (r1 - r0 == 2 ? 8 : 4);
        // A heavy row may be cut into chunks, one unit each (consecutive units that name the same row).
        const int n_chunks = heavy ? heavy_chunks(d0) : 1;
        int chunk = 0;
        if (n_chunks > 1) {
#pragma unroll
            for (int k = 1; k < kMaxHeavyChunks; ++k) chunk += (u - k >= 0 && unit_ptr[max(u - k, 0)] == r0) ? 1 : 0;
        }
        const int row_try = r0 + wave / share;
        const bool valid = heavy || row_try < r1;
        const int row = valid ? row_try : r0;
        const int slice = wave % share;
        const int c = tile * T + (lane % LPG) * VEC;
        const bool active = valid && c < B;
        ACC acc[VEC];
        if (valid) {
            int e0 = row_ptr[row], e1 = row_ptr[row + 1];
            if (n_chunks > 1) {
                const int len = heavy_chunk_len(d0);
                e0 = row0_begin + chunk * len;
                e1 = min(e0 + len, row0_end);
            }
            const int per = (e1 - e0 + share - 1) / share;
            const int b0 = min(e0 + slice * per, e1), b1 = min(b0 + per, e1);
            row_sum_dataflow<VEC, LPG, ACC, U>(col, w, V, B, b0, b1, active ? c : 0, first_row, ctl, acc);
        } else {
#pragma unroll
            for (int j = 0; j < VEC; ++j) acc[j] = ACC(0);
        }
        if (share > 1) {                               // block-uniform: a heavy row (`row` is r0) or medium rows
            // The wavefronts' partial sums meet in LDS.  From here on the tile is spread over all
            // lanes of wavefront 0 (E elements per lane), so that the additions, the sigmoid and the
            // store that follow the last gathered source take as few instructions as possible.
            if (lane < LPG) {
#pragma unroll
                for (int j = 0; j < VEC; ++j) part[wave][lane * VEC + j] = acc[j];
            }
            const bool split = n_chunks > 1, last_chunk = chunk == n_chunks - 1;     // block-uniform
            const uint32_t slot0 = partial_slot(row0_begin);
            const uint32_t slot_elems = (uint32_t)tiles * T;
            const uint32_t el = (uint32_t)lane * E;            // this lane's first element of the tile
            if (split && last_chunk && wave < n_chunks - 1 && lane < EL) {
                // The unit that holds the last chunk of a split row collects the partial sums of the
                // other chunks: wavefront k waits for chunk k, so the waits overlap.
                ACC p[E];
                Patience patience;
                for (;;) {
                    bool ok = true;
#pragma unroll
                    for (int j = 0; j < E; ++j) {
                        bool ready;
                        p[j] = PartialBits<ACC>::load(pres, (uint32_t)(((slot0 + wave) * slot_elems + (uint32_t)tile * T + el + j) * sizeof(ACC)), ready);
                        ok = ok && ready;
                    }
                    if (ok || !patience.again(ctl)) break;
                }
#pragma unroll
                for (int j = 0; j < E; ++j) others[wave][el + j] = p[j];
            }
            __syncthreads();
            if (slice == 0 && valid && lane < EL) {         // the first wavefront of every row
                ACC sum[E];
#pragma unroll
                for (int j = 0; j < E; ++j) {
                    ACC t = ACC(0);
                    if (share == kMixedWaves) {
#pragma unroll
                        for (int k = 0; k < kMixedWaves; ++k) t += part[k][el + j];
                    } else {                            // grouped medium rows: not what a level waits for
#pragma unroll 1
                        for (int k = 0; k < share; ++k) t += part[wave + k][el + j];
                    }
                    sum[j] = t;
                }
                if (split && !last_chunk) {
                    // not the last chunk: hand the partial sum to the unit that holds the last one
#pragma unroll
                    for (int j = 0; j < E; ++j)
                        PartialBits<ACC>::store(pres, (uint32_t)(((slot0 + chunk) * slot_elems + (uint32_t)tile * T + el + j) * sizeof(ACC)), sum[j]);
                } else {
                    if (split) {
                        // the last chunk adds the others in chunk order, then its own
#pragma unroll
                        for (int j = 0; j < E; ++j) {
                            ACC total = ACC(0);
#pragma unroll 1
                            for (int k = 0; k < n_chunks - 1; ++k) total += others[k][el + j];
                            sum[j] = total + sum[j];
                        }
                    }
                    const uint32_t ce = (uint32_t)tile * T + el;
                    if (ce < (uint32_t)B) {
                        float out[E];
#pragma unroll
                        for (int j = 0; j < E; ++j) out[j] = squash(sum[j]);
                        store_vec_device_scope<E>(V + (size_t)row * (size_t)B + ce, out);
                    }
                }
            }
        } else if constexpr (kWave / LPG >= VEC && VEC > 1) {
            // light rows, one wavefront each, of a batch narrow enough for VEC lane groups or more: every
            // group holds the sums, so group j finishes column j of its lanes' VEC columns (one sigmoid per
            // lane instead of VEC in a row; a reader takes a tile as written once all its columns are).
            const int gsel = lane / LPG;
            if (active && gsel < VEC) {
                ACC mine = acc[0];
#pragma unroll
                for (int j = 1; j < VEC; ++j) mine = (gsel == j) ? acc[j] : mine;
                const float out[1] = {squash(mine)};
                store_vec_device_scope<1>(V + (size_t)row * (size_t)B + (size_t)(c + gsel), out);
            }
        } else if (active && lane < LPG) {               // light rows: one wavefront each
            float out[VEC];
#pragma unroll
            for (int j = 0; j < VEC; ++j) out[j] = squash(acc[j]);
            store_vec_device_scope<VEC>(V + (size_t)row * (size_t)B + (size_t)c, out);
        }
    }
}

// ------------------------------------------------------- one workgroup per tile
// The paper's kernel shape: one workgroup walks all levels with a workgroup
// barrier between two levels, and nothing is exchanged between workgroups.
// Batch columns are independent, so there is one such workgroup per tile of
// batch columns; it also stages the sensor values of its tile first and
// copies the output rows last, which makes the whole activation one launch.
// A small network spends its time on launches and level hand-overs, not on
// connections: this schedule pays about a microsecond per level.
//
// Lanes: LPG lanes cover the tile's columns, so a wavefront holds G = 64/LPG
// lane groups.  Light rows are taken one per lane group, each group walking
// its row's connections serially in edge-list order (for B = 1 that is the
// paper's thread per node with a serial loop); medium rows one per wavefront,
// the groups striding over the connections; heavy rows by all 16 wavefronts.

// Serial weighted sum of one row's connections for a lane group (per-lane col/w loads,
// U gathers in flight).  e_begin/e_end may differ between the groups of a wavefront.
template <int VEC, typename ACC, int U>
__device__ inline void row_sum_serial(const int32_t *__restrict__ col, const float *__restrict__ w, const float *V, int B,
                                      int e_begin, int e_end, int c0, ACC (&acc)[VEC]) {
#pragma unroll
    for (int j = 0; j < VEC; ++j) acc[j] = ACC(0);
    const float *Vc = V + c0;
    for (int e = e_begin; e < e_end; e += U) {
        int cc[U];
        float ww[U];
        float vals[U][VEC];
#pragma unroll
        for (int k = 0; k < U; ++k) {
            const int ek = min(e + k, e_end - 1);        // padded slots re-read the last connection
            cc[k] = col[ek];
            ww[k] = w[ek];
        }
#pragma unroll
        for (int k = 0; k < U; ++k) load_vec<VEC>(Vc + (size_t)cc[k] * (size_t)B, vals[k]);
#pragma unroll
        for (int k = 0; k < U; ++k)
#pragma unroll
            for (int j = 0; j < VEC; ++j) {
                const ACC t = acc[j] + (ACC)ww[k] * (ACC)vals[k][j];
                acc[j] = (e + k < e_end) ? t : acc[j];
            }
    }
}

// STAGED = 2: the packed connections and the workgroup's tile of V live in LDS for the whole
// activation (dynamic LDS: V tile [n_nodes][T] floats, then row_ptr, col, w, level_ptr), so a level costs
// LDS round trips instead of L2 ones; the tile is copied to V in global memory at the end.
// STAGED = 1: only the tile of V does (a network too large for LDS whose values still fit): the
// loads that depend on the level below are the LDS ones.  STAGED = 0: everything in global memory.
template <int VEC, int LPG, typename ACC, int U, int STAGED>
__global__ __launch_bounds__(kMixedBlock) void workgroup_kernel(
    const int32_t *__restrict__ level_ptr, int n_levels, const int32_t *__restrict__ row_ptr,
    const int32_t *__restrict__ col, const float *__restrict__ w, float *V, int B,
    const int32_t *__restrict__ input_ids, const int32_t *__restrict__ inv_perm, const float *__restrict__ X,
    int n_inputs, int raw, const int32_t *__restrict__ output_ids, float *__restrict__ Y, int n_outputs, int n_nodes,
    int n_edges) {
    constexpr int T = LPG * VEC;
    constexpr int G = kWave / LPG;
    __shared__ ACC part[kMixedWaves][T];
    extern __shared__ __align__(16) unsigned char staged[];
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
    const int lane = threadIdx.x & (kWave - 1);
    const int g = lane / LPG;                          // lane group inside the wavefront
    const int slot = wave * G + g;                     // lane group inside the workgroup
    constexpr int kSlots = kMixedWaves * G;
    const int ct = (lane % LPG) * VEC;                 // first column of this lane inside the tile
    const int c = blockIdx.x * T + ct;
    const bool col_ok = c < B;

    // where the sums read: the LDS copies, or global memory
    float *s_V = reinterpret_cast<float *>(staged);
    int32_t *s_row_ptr = reinterpret_cast<int32_t *>(staged + (((size_t)n_nodes * T * 4 + 15) & ~(size_t)15));
    int32_t *s_col = s_row_ptr + (n_nodes + 1);
    float *s_w = reinterpret_cast<float *>(s_col + n_edges);
    int32_t *s_level_ptr = reinterpret_cast<int32_t *>(s_w + n_edges);
    const int32_t *lp = STAGED == 2 ? s_level_ptr : level_ptr;
    const int32_t *rp = STAGED == 2 ? s_row_ptr : row_ptr;
    const int32_t *cl = STAGED == 2 ? s_col : col;
    const float *wt = STAGED == 2 ? s_w : w;
    const float *Vr = STAGED ? s_V : V;
    const int ld = STAGED ? T : B;                     // row stride of Vr
    const int cr = STAGED ? ct : (col_ok ? c : 0);     // this lane's first column in Vr
    // The first sensor and the first output row of this lane group are looked up now, beside the
    // staging loads, and kept in registers: two chains of dependent loads (id -> packed row -> value)
    // that would otherwise stand alone after a barrier each, a few microseconds of an activation
    // that takes five.  (Further sensors and outputs of the group, beyond kSlots of either, are
    // looked up where they are needed.)
    int32_t first_in_row = -1, first_out_row = -1;
    float first_x[VEC];
#pragma unroll
    for (int j = 0; j < VEC; ++j) first_x[j] = 0.0f;
    if (slot < n_inputs) {
        const int32_t id = input_ids[slot];
        if (col_ok) {
#pragma unroll
            for (int j = 0; j < VEC; ++j) first_x[j] = X[(size_t)slot * (size_t)B + c + j];
        }
        if (id >= 0 && id < n_nodes) first_in_row = inv_perm[id];
    }
    if (Y != nullptr && slot < n_outputs) {
        const int32_t id = output_ids[slot];
        if (id >= 0 && id < n_nodes) first_out_row = inv_perm[id];
    }
    if constexpr (STAGED == 2) {
        for (int i = threadIdx.x; i <= n_nodes; i += kMixedBlock) s_row_ptr[i] = row_ptr[i];
        // eight connections per thread and round, all their loads in flight before the first LDS store
        for (int i0 = threadIdx.x; i0 < n_edges; i0 += 8 * kMixedBlock) {
            int32_t cc[8];
            float ww[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int i = min(i0 + k * kMixedBlock, n_edges - 1);
                cc[k] = col[i];
                ww[k] = w[i];
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int i = i0 + k * kMixedBlock;
                if (i < n_edges) { s_col[i] = cc[k]; s_w[i] = ww[k]; }
            }
        }
        for (int i = threadIdx.x; i <= ASNN_CLASSES * n_levels; i += kMixedBlock) s_level_ptr[i] = level_ptr[i];
        __syncthreads();
    }
    // A staged workgroup keeps its values in LDS and copies the tile to V once at the end: a
    // global store before a barrier would make every level wait for its acknowledgement.
    auto put = [&](int row, const float (&out)[VEC]) {
        if constexpr (STAGED) {
            store_vec<VEC>(s_V + row * T + ct, out);
        } else {
            if (col_ok) store_vec<VEC>(V + (size_t)row * (size_t)B + c, out);
        }
    };

    // One column of a lane's VEC: lane group `gsel` of a wavefront all of whose groups hold the row's sums
    // finishes column gsel (one sigmoid per lane instead of VEC in a row in the first group alone).
    constexpr bool kSpread = G >= VEC && VEC > 1;
    const int gsel = lane / LPG;
    auto put_column = [&](int row, ACC sum) {             // column gsel of this lane's VEC
        const float out = squash(sum);
        if constexpr (STAGED) {
            s_V[row * T + ct + gsel] = out;
        } else {
            if (col_ok) V[(size_t)row * (size_t)B + c + gsel] = out;
        }
    };

    // Level 0 has no connections: sigmoid(0), then the sensors take their inputs.
    const int level0_end = lp[ASNN_CLASSES];
    {
        float half[VEC];
#pragma unroll
        for (int j = 0; j < VEC; ++j) half[j] = squash(ACC(0));
        for (int r = slot; r < level0_end; r += kSlots) put(r, half);
    }
    __syncthreads();
    if (first_in_row >= 0) {
        float out[VEC];
#pragma unroll
        for (int j = 0; j < VEC; ++j) out[j] = raw ? first_x[j] : squash((ACC)first_x[j]);
        put(first_in_row, out);
    }
    for (int k = slot + kSlots; k < n_inputs; k += kSlots) {
        const int32_t id = input_ids[k];
        if (id < 0 || id >= n_nodes) continue;
        float out[VEC];
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
            const float x = col_ok ? X[(size_t)k * (size_t)B + c + j] : 0.0f;
            out[j] = raw ? x : squash((ACC)x);
        }
        put(inv_perm[id], out);
    }
    __syncthreads();

    // teams of 16 lanes for the light rows of narrow levels (see there)
    constexpr bool kTeams = LPG <= 8;
    constexpr int S = kTeams ? 16 / LPG : 1;                 // lane groups per team
    constexpr int UT = 2 * LPG < 8 ? 2 * LPG : 8;            // connections per group and round
    // A pass of the teams over 64 rows takes about 0.45 us at one column per lane, a pass of the
    // serial walk (up to 1024 rows) 0.8 us from LDS and twice that from global memory: two passes
    // of the teams still pay.  With more columns per lane the sigmoids dominate both and the serial
    // walk wins from the second pass on.
    constexpr int kTeamRowsMost = (VEC == 1 ? 2 : 1) * (kMixedBlock / 16);

    for (int l = 1; l < n_levels; ++l) {
        const int hb = lp[ASNN_CLASSES * l], mb = lp[ASNN_CLASSES * l + 1], lb = lp[ASNN_CLASSES * l + 2],
                  le = lp[ASNN_CLASSES * l + 3];
        // heavy rows: all wavefronts on one row, partial sums meet in LDS in wave order
        for (int row = hb; row < mb; ++row) {
            const int e0 = rp[row], e1 = rp[row + 1];
            const int chunk = (e1 - e0 + kMixedWaves - 1) / kMixedWaves;
            const int b0 = min(e0 + wave * chunk, e1), b1 = min(b0 + chunk, e1);
            ACC acc[VEC];
            row_sum<VEC, LPG, ACC, U>(cl, wt, Vr, ld, b0, b1, cr, acc);
            if (lane < LPG) {
#pragma unroll
                for (int j = 0; j < VEC; ++j) part[wave][lane * VEC + j] = acc[j];
            }
            __syncthreads();
            if constexpr (kSpread) {
                if (wave == 0 && gsel < VEC) {            // lane group j adds up and finishes column j
                    ACC s = ACC(0);
                    for (int k = 0; k < kMixedWaves; ++k) s += part[k][(lane % LPG) * VEC + gsel];
                    put_column(row, s);
                }
            } else if (wave == 0 && lane < LPG) {
                float out[VEC];
#pragma unroll
                for (int j = 0; j < VEC; ++j) {
                    ACC s = ACC(0);
                    for (int k = 0; k < kMixedWaves; ++k) s += part[k][lane * VEC + j];
                    out[j] = squash(s);
                }
                put(row, out);
            }
            __syncthreads();
        }
        // medium rows: one wavefront per row
        for (int row = mb + wave; row < lb; row += kMixedWaves) {
            ACC acc[VEC];
            row_sum<VEC, LPG, ACC, U>(cl, wt, Vr, ld, rp[row], rp[row + 1], cr, acc);
            if constexpr (kSpread) {
                ACC mine = acc[0];
#pragma unroll
                for (int j = 1; j < VEC; ++j) mine = (gsel == j) ? acc[j] : mine;
                if (gsel < VEC) put_column(row, mine);
            } else if (lane < LPG) {
                float out[VEC];
#pragma unroll
                for (int j = 0; j < VEC; ++j) out[j] = squash(acc[j]);
                put(row, out);
            }
        }
        // light rows: one lane group per row (a full wavefront per row when the tile needs all lanes)
        if constexpr (G == 1) {
            for (int row = lb + wave; row < le; row += kMixedWaves) {
                ACC acc[VEC];
                row_sum<VEC, LPG, ACC, U>(cl, wt, Vr, ld, rp[row], rp[row + 1], cr, acc);
                float out[VEC];
#pragma unroll
                for (int j = 0; j < VEC; ++j) out[j] = squash(acc[j]);
                put(row, out);
            }
        } else if (kTeams && le - lb <= kTeamRowsMost) {     // workgroup-uniform
            // A level of few light rows: a lane group walking its row alone issues some 150
            // instructions per 8 connections, one after the other.  Here a team of 16 lanes shares
            // a row, its S groups taking every S-th connection (a light row has fewer than 32, so
            // one round of S x UT), and the groups' sums meet through DPP moves.
            const int sg = (lane % 16) / LPG;                 // lane group inside the team
            for (int row = lb + (int)(threadIdx.x / 16); row < le; row += kMixedBlock / 16) {
                const int e0 = rp[row], e1 = rp[row + 1];
                ACC acc[VEC];
#pragma unroll
                for (int j = 0; j < VEC; ++j) acc[j] = ACC(0);
                for (int base = e0; base < e1; base += S * UT) {
                    int cc[UT];
                    float ww[UT];
                    float vals[UT][VEC];
#pragma unroll
                    for (int k = 0; k < UT; ++k) {
                        const int ek = min(base + k * S + sg, e1 - 1);    // padded slots re-read the last connection
                        cc[k] = cl[ek];
                        ww[k] = wt[ek];
                    }
#pragma unroll
                    for (int k = 0; k < UT; ++k) load_vec<VEC>(Vr + (size_t)cc[k] * (size_t)ld + cr, vals[k]);
#pragma unroll
                    for (int k = 0; k < UT; ++k)
#pragma unroll
                        for (int j = 0; j < VEC; ++j) {
                            const ACC t = acc[j] + (ACC)ww[k] * (ACC)vals[k][j];
                            acc[j] = (base + k * S + sg < e1) ? t : acc[j];
                        }
                }
                team_sum<VEC, LPG, ACC>(acc);
                // the sigmoids of a lane's VEC columns go to different groups of the team
#pragma unroll
                for (int r = 0; r < (VEC + S - 1) / S; ++r) {
                    const int jsel = sg + r * S;
                    ACC mine = acc[0];
#pragma unroll
                    for (int j = 1; j < VEC; ++j) mine = (jsel == j) ? acc[j] : mine;
                    if (jsel < VEC) {
                        const float out = squash(mine);
                        if constexpr (STAGED) {
                            s_V[row * T + ct + jsel] = out;
                        } else {
                            if (col_ok) V[(size_t)row * (size_t)B + c + jsel] = out;
                        }
                    }
                }
            }
        } else {
            for (int row = lb + slot; row < le; row += kSlots) {
                ACC acc[VEC];
                row_sum_serial<VEC, ACC, U>(cl, wt, Vr, ld, rp[row], rp[row + 1], cr, acc);
                float out[VEC];
#pragma unroll
                for (int j = 0; j < VEC; ++j) out[j] = squash(acc[j]);
                put(row, out);
            }
        }
        __syncthreads();        // the layer barrier of the paper's kernel
    }

    if (Y != nullptr && col_ok) {
        if (slot < n_outputs) {
            const bool ok = first_out_row >= 0;
            const size_t row = ok ? (size_t)first_out_row : 0;
#pragma unroll
            for (int j = 0; j < VEC; ++j)
                Y[(size_t)slot * (size_t)B + c + j] = ok ? Vr[row * (size_t)ld + cr + j] : __builtin_nanf("");
        }
        for (int o = slot + kSlots; o < n_outputs; o += kSlots) {
            const int32_t id = output_ids[o];
            const bool ok = id >= 0 && id < n_nodes;
            const size_t row = ok ? (size_t)inv_perm[id] : 0;
#pragma unroll
            for (int j = 0; j < VEC; ++j)
                Y[(size_t)o * (size_t)B + c + j] = ok ? Vr[row * (size_t)ld + cr + j] : __builtin_nanf("");
        }
    }
    if constexpr (STAGED) {
        const int total = n_nodes * T;
        for (int i = threadIdx.x; i < total; i += kMixedBlock) {
            const int row = i / T, cc = blockIdx.x * T + i % T;
            if (cc < B) V[(size_t)row * (size_t)B + cc] = s_V[i];
        }
    }
}

// Level 0: every value is sigmoid(0) until a sensor overwrites its row.
template <typename ACC>
__global__ void fill_half_kernel(float *__restrict__ V, size_t n) {
    const float half = squash(ACC(0));
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) V[i] = half;
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

// Dataflow schedule: sensors and the reset of everything above level 0 (see dataflow_reset_kernel) in
// one launch: the two write disjoint rows, and a launch costs a few microseconds.
template <typename ACC>
__global__ void dataflow_prologue_kernel(const int32_t *__restrict__ input_ids, const int32_t *__restrict__ inv_perm,
                                         const float *__restrict__ X, float *__restrict__ V, int32_t n_inputs,
                                         int32_t n_nodes, int B, int raw, unsigned int *v_begin, size_t n_values,
                                         unsigned int *partial_words, size_t n_partial_words, DataflowCtl *ctl) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    const size_t first = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t total = (size_t)n_inputs * (size_t)B;
    for (size_t i = first; i < total; i += stride) {
        const int k = (int)(i / B), b = (int)(i % B);
        const int32_t id = input_ids[k];
        if (id < 0 || id >= n_nodes) continue;
        const float x = X[i];
        V[(size_t)inv_perm[id] * (size_t)B + b] = raw ? x : squash((ACC)x);
    }
    for (size_t i = first; i < n_values; i += stride) v_begin[i] = kNotReady;
    for (size_t i = first; i < n_partial_words; i += stride) partial_words[i] = kNotReady;
    if (blockIdx.x == 0 && threadIdx.x < 64)
        reinterpret_cast<int *>(ctl)[threadIdx.x] = (threadIdx.x == 2) ? kCtlMagic : 0;
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
        long long items = (long long)(le - lb) * tiles;
        int items_per_xcd = 0;
        if (tiles % kXcds != 0 && tiles > 1) {     // (8 | tiles: the row-major order aligns tiles and dies by itself)
            const long long per = (items + kXcds - 1) / kXcds;
            if (per <= 0x7fffffffLL / kXcds) {
                items_per_xcd = (int)per;
                items = per * kXcds;
            }
        }
        if (items > 0x7fffffffLL) return ASNN_ERR_SIZE;
        hipLaunchKernelGGL((gather_light_kernel<VEC, LPG, ACC, kUnroll>), dim3((unsigned)items), dim3(kWave), 0, a.s,
                           a.row_ptr, a.col, a.w, a.V, a.B, lb, le, tiles, items_per_xcd);
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

// Lane layout for a batch width.  A full wavefront per tile (64 lanes, wave-uniform connection:
// scalar (col, w), one source row per load instruction) is much cheaper per byte than the grouped
// layout, and among full-wavefront layouts two floats per lane (512 B per load, twice the number
// of independent wavefronts) measured 9 % faster than four on the 100k-node workload, so level
// launches take float2 tiles whenever the batch fills more than half a wavefront that way; only
// batches of 32 columns or fewer fall back to lane groups.  A level with few rows is a set of
// latency chains rather than a stream of bytes: below kSmallLevelItems (row, tile) items it takes
// float4 tiles when they still fill a wavefront (half the wavefronts and load instructions for
// the same bytes; 10 % faster on the pruned MLP, whose levels hold about 900 rows).
//
// The dataflow schedule is latency-bound as well (a row is a chain of gather rounds), so there the
// widest vector always wins: it puts the most connections into one round.
constexpr long long kSmallLevelItems = 4096;
inline int vec_for(int B, bool dataflow, long long rows = 1LL << 40) {
    if (!dataflow) {
        if (B % 4 == 0 && B / 4 >= kWave && rows * ((B / 2 + kWave - 1) / kWave) < kSmallLevelItems) return 4;
        if (B % 2 == 0 && B / 2 > 32) return 2;
        if (B > 32) return 1;
    }
    return (B % 4 == 0) ? 4 : (B % 2 == 0 ? 2 : 1);
}

template <typename ACC>
int launch_level_any(const LevelArgs &a, int hb, int mb, int lb, int le) {
    switch (vec_for(a.B, false, le - hb)) {
        case 4: return launch_level_vec<4, ACC>(a, hb, mb, lb, le);
        case 2: return launch_level_vec<2, ACC>(a, hb, mb, lb, le);
        default: return launch_level_vec<1, ACC>(a, hb, mb, lb, le);
    }
}

struct DataflowArgs {
    const int32_t *unit_ptr;
    int first_unit, n_work, first_row;
    DataflowCtl *ctl;
    int cus;
    int units_per_level;     // average, for sizing the persistent grid
    void *partials;          // partial sums of split heavy rows
    uint32_t partial_bytes;
    const int32_t *output_ids, *inv_perm;      // output rows are copied to Y by the same launch
    float *Y;
    int n_outputs, n_nodes;
};

template <int VEC, int LPG, typename ACC>
int launch_dataflow(const LevelArgs &a, const DataflowArgs &d) {
    const int vecs = a.B / VEC;
    const int tiles = (vecs + LPG - 1) / LPG;
    // resident 16-wave blocks per CU for this instantiation, per device (threads that race to fill
    // an entry store the same value)
    static std::atomic<int> per_cu_of[kMaxDevices];
    int dev = 0;
    ASNN_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return ASNN_ERR_NO_DEVICE;
    int per_cu = per_cu_of[dev].load(std::memory_order_relaxed);
    if (per_cu == 0) {
        int n = 0;
        ASNN_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, dataflow_kernel<VEC, LPG, ACC, kUnroll>,
                                                                  kMixedBlock, 0));
        per_cu = n > 0 ? n : 1;
        per_cu_of[dev].store(per_cu, std::memory_order_relaxed);
    }
    // Workgroups far ahead of the wavefront of finished rows only spin and re-read: a few levels'
    // worth of units in flight is enough.
    long long blocks = (long long)d.cus * per_cu;
    const long long useful = 2LL * d.units_per_level * tiles + 32;
    const long long items = (long long)d.n_work + (long long)((d.n_outputs + kMixedWaves - 1) / kMixedWaves) * tiles;
    if (blocks > useful) blocks = useful;
    if (blocks > items) blocks = items;
    if (blocks < 1) return ASNN_OK;
    hipLaunchKernelGGL((dataflow_kernel<VEC, LPG, ACC, kUnroll>), dim3((unsigned)blocks), dim3(kMixedBlock), 0, a.s,
                       a.row_ptr, a.col, a.w, a.V, a.B, d.unit_ptr, d.first_unit, d.n_work, tiles, d.first_row,
                       d.ctl, d.partials, d.partial_bytes, d.output_ids, d.inv_perm, d.Y, d.n_outputs, d.n_nodes);
    ASNN_HIP_TRY(hipGetLastError());
    return ASNN_OK;
}

template <int VEC, typename ACC>
int launch_dataflow_vec(const LevelArgs &a, const DataflowArgs &d) {
    const int vecs = a.B / VEC;
    if (vecs > 32) return launch_dataflow<VEC, 64, ACC>(a, d);
    if (vecs > 16) return launch_dataflow<VEC, 32, ACC>(a, d);
    if (vecs > 8) return launch_dataflow<VEC, 16, ACC>(a, d);
    if (vecs > 4) return launch_dataflow<VEC, 8, ACC>(a, d);
    if (vecs > 2) return launch_dataflow<VEC, 4, ACC>(a, d);
    if (vecs > 1) return launch_dataflow<VEC, 2, ACC>(a, d);
    return launch_dataflow<VEC, 1, ACC>(a, d);
}

template <typename ACC>
int launch_dataflow_any(const LevelArgs &a, const DataflowArgs &d) {
    switch (vec_for(a.B, true)) {
        case 4: return launch_dataflow_vec<4, ACC>(a, d);
        case 2: return launch_dataflow_vec<2, ACC>(a, d);
        default: return launch_dataflow_vec<1, ACC>(a, d);
    }
}

struct WorkgroupArgs {
    const int32_t *level_ptr;
    int n_levels;
    const int32_t *input_ids, *inv_perm;
    const float *X;
    int n_inputs, raw;
    const int32_t *output_ids;
    float *Y;
    int n_outputs, n_nodes;
    int64_t n_edges;
};

// Lane layout of the workgroup schedule.  Up to 64 columns: the widest vector, which leaves the
// most lane groups (rows in flight) per wavefront.  Wider batches: one float per lane, 64 columns
// per workgroup, because the workgroups are independent and more of them finish sooner.
inline int vec_for_workgroup(int B) {
    if (B > 64) return 1;
    return (B % 4 == 0) ? 4 : (B % 2 == 0 ? 2 : 1);
}

inline long long tiles_for_workgroup(int B) {
    const int vec = vec_for_workgroup(B);
    const int vecs = B / vec;
    int lpg = 1;
    while (lpg < 64 && lpg < vecs) lpg <<= 1;
    return (vecs + lpg - 1) / lpg;
}

// Dynamic LDS a staged workgroup needs; the packed network is staged when this fits what a
// workgroup may take beside the static arrays of the kernel (partial sums: 16 x T accumulators).
constexpr size_t kLdsDefaultPerWorkgroup = 64 * 1024;   // without raising the kernel attribute
inline size_t staged_lds_bytes(int n_nodes, int64_t n_edges, int n_levels, int T) {
    return (((size_t)n_nodes * (size_t)T * 4 + 15) & ~(size_t)15) + 4 * ((size_t)n_nodes + 1) + 8 * (size_t)n_edges +
           4 * ((size_t)ASNN_CLASSES * (size_t)n_levels + 1);
}

template <int VEC, int LPG, typename ACC>
int launch_workgroup(const LevelArgs &a, const WorkgroupArgs &g) {
    const int vecs = a.B / VEC;
    const int tiles = (vecs + LPG - 1) / LPG;
    const size_t lds = staged_lds_bytes(g.n_nodes, g.n_edges, g.n_levels, LPG * VEC);
    // dynamic LDS this instantiation may take on the current device (the attribute is per device)
    // (threads that race to fill an entry set the same attribute and store the same value)
    static std::atomic<size_t> budgets[kMaxDevices];
    int dev = 0;
    ASNN_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return ASNN_ERR_NO_DEVICE;
    size_t budget = budgets[dev].load(std::memory_order_acquire);
    if (budget == 0) {
        const size_t fixed = sizeof(ACC) * kMixedWaves * LPG * VEC + 256;       // static LDS of the kernel, rounded up
        int optin = 0;
        size_t most = kLdsDefaultPerWorkgroup;
        if (hipDeviceGetAttribute(&optin, hipDeviceAttributeSharedMemPerBlockOptin, dev) == hipSuccess &&
            (size_t)optin > most)
            most = (size_t)optin;
        budget = kLdsDefaultPerWorkgroup - fixed;
        if (most > kLdsDefaultPerWorkgroup &&
            hipFuncSetAttribute(reinterpret_cast<const void *>(&workgroup_kernel<VEC, LPG, ACC, kUnroll, 2>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)(most - fixed)) == hipSuccess &&
            hipFuncSetAttribute(reinterpret_cast<const void *>(&workgroup_kernel<VEC, LPG, ACC, kUnroll, 1>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)(most - fixed)) == hipSuccess)
            budget = most - fixed;
        (void)hipGetLastError();
        budgets[dev].store(budget, std::memory_order_release);
    }
    const size_t lds_values = ((size_t)g.n_nodes * (size_t)(LPG * VEC) * 4 + 15) & ~(size_t)15;      // the value tile alone
    if (lds <= budget) {
        hipLaunchKernelGGL((workgroup_kernel<VEC, LPG, ACC, kUnroll, 2>), dim3((unsigned)tiles), dim3(kMixedBlock), lds,
                           a.s, g.level_ptr, g.n_levels, a.row_ptr, a.col, a.w, a.V, a.B, g.input_ids, g.inv_perm, g.X,
                           g.n_inputs, g.raw, g.output_ids, g.Y, g.n_outputs, g.n_nodes, (int)g.n_edges);
    } else if (lds_values <= budget) {
        hipLaunchKernelGGL((workgroup_kernel<VEC, LPG, ACC, kUnroll, 1>), dim3((unsigned)tiles), dim3(kMixedBlock), lds_values,
                           a.s, g.level_ptr, g.n_levels, a.row_ptr, a.col, a.w, a.V, a.B, g.input_ids, g.inv_perm, g.X,
                           g.n_inputs, g.raw, g.output_ids, g.Y, g.n_outputs, g.n_nodes, (int)g.n_edges);
    } else {
        hipLaunchKernelGGL((workgroup_kernel<VEC, LPG, ACC, kUnroll, 0>), dim3((unsigned)tiles), dim3(kMixedBlock), 0,
                           a.s, g.level_ptr, g.n_levels, a.row_ptr, a.col, a.w, a.V, a.B, g.input_ids, g.inv_perm, g.X,
                           g.n_inputs, g.raw, g.output_ids, g.Y, g.n_outputs, g.n_nodes, (int)g.n_edges);
    }
    ASNN_HIP_TRY(hipGetLastError());
    return ASNN_OK;
}

template <int VEC, typename ACC>
int launch_workgroup_vec(const LevelArgs &a, const WorkgroupArgs &g) {
    const int vecs = a.B / VEC;
    if (vecs > 32) return launch_workgroup<VEC, 64, ACC>(a, g);
    if (vecs > 16) return launch_workgroup<VEC, 32, ACC>(a, g);
    if (vecs > 8) return launch_workgroup<VEC, 16, ACC>(a, g);
    if (vecs > 4) return launch_workgroup<VEC, 8, ACC>(a, g);
    if (vecs > 2) return launch_workgroup<VEC, 4, ACC>(a, g);
    if (vecs > 1) return launch_workgroup<VEC, 2, ACC>(a, g);
    return launch_workgroup<VEC, 1, ACC>(a, g);
}

template <typename ACC>
int launch_workgroup_any(const LevelArgs &a, const WorkgroupArgs &g) {
    switch (vec_for_workgroup(a.B)) {
        case 4: return launch_workgroup_vec<4, ACC>(a, g);
        case 2: return launch_workgroup_vec<2, ACC>(a, g);
        default: return launch_workgroup_vec<1, ACC>(a, g);
    }
}

// Tiles per row of the dataflow schedule for a given B (the same choice its launcher makes).
inline int tiles_for(int B) {
    const int vec = vec_for(B, true);
    const int vecs = B / vec;
    int lpg = 1;
    while (lpg < 64 && lpg < vecs) lpg <<= 1;
    return (vecs + lpg - 1) / lpg;
}

// Batch width rounded up to whole tiles of the dataflow lane layout.
inline int64_t padded_batch(int B) {
    const int vec = vec_for(B, true);
    const int vecs = B / vec;
    int lpg = 1;
    while (lpg < 64 && lpg < vecs) lpg <<= 1;
    return (int64_t)((vecs + lpg - 1) / lpg) * lpg * vec;
}

// Workspace of the dataflow schedule: the control block, then (only when some row is cut into
// chunks) one slot of padded_batch(B) partial sums per kHeavyChunk/2 connections.
struct ActivateWorkspace {
    DataflowCtl *ctl;
    unsigned int *partials;
    size_t partial_bytes;
    size_t bytes;
};

inline ActivateWorkspace carve_activate(void *ws, const asnn_packed *packed, int32_t B) {
    Carver c(ws);
    ActivateWorkspace w;
    w.ctl = c.take<DataflowCtl>(1);
    w.partial_bytes = 0;
    if (packed->max_heavy_indegree > kHeavyChunk) {
        const size_t slots = (size_t)(packed->n_edges / (kHeavyChunk / 2)) + kMaxHeavyChunks + 1;
        w.partial_bytes = slots * (size_t)padded_batch(B) * sizeof(double);
    }
    w.partials = c.take<unsigned int>(w.partial_bytes / sizeof(unsigned int) + 1);
    w.bytes = c.off;
    return w;
}

// Which schedule an activation takes: 0 = one launch per level, 1 = dataflow, 2 = one workgroup
// per tile, < 0 = error.
int choose_schedule(const asnn_packed *packed, int32_t B, bool has_workspace, uint32_t flags);

// Level launches against the persistent dataflow launch: a cost model per level, in
// microseconds, fitted to measurements on MI355X (w = connections*samples of an average level).
//   level launches: 3.5 + w / 2.0e6 (w / 3.0e6 when the value matrix fits the L2 caches, 32 MiB:
//     the dataflow schedule reads around them), plus the tail of the level's heaviest row, which
//     one 16-wave workgroup per tile walks 128 connections at a time (about 0.6 us per round);
//   dataflow: w / 1.5e6 with the batch rounded up to whole tiles, but at least the latency of a
//     level hand-over (2 us; 3.8 us when rows are split over workgroups) and at least the time the
//     level's work items take at 5 us each on the 512 workgroups the chip holds (a pruned
//     multilayer perceptron at a narrow batch is one item per row and tile with little in it),
//     plus its share of the 5 us the extra launch and the start of the persistent grid cost once.
// Without heavy rows the two meet near 20 M connections*samples per level.
constexpr double kLevelLaunchUs = 3.5, kLevelWorkPerUs = 2.0e6, kLevelWorkPerUsCached = 3.0e6, kHeavyRoundUs = 0.6;
constexpr double kCachedValueBytes = 32.0 * 1024.0 * 1024.0;
constexpr double kDataflowWorkPerUs = 1.5e6, kDataflowHopUs = 2.0, kDataflowSplitHopUs = 3.8, kDataflowStartUs = 5.0;
constexpr double kDataflowItemUs = 5.0, kDataflowResidentWorkgroups = 512.0;
// Connections up to which one workgroup per tile beats the schedules that spread a level over the
// chip: base + per_level * n_levels.  Measured on MI355X at B = 1: the workgroup schedule takes
// about 11 us + 0.45 us per level + 0.6 ns per connection (next to nothing per connection while
// the network fits in LDS), the dataflow schedule about 9 us + 1.9 us per level and next to
// nothing per connection, so the break-even grows with the depth (20k connections at 5 levels,
// 70k at 40, 130k at 80).  Wider tiles leave the workgroup fewer rows in flight (16 * 64/LPG
// lane groups) and more sigmoids per lane: break-evens read off sweeps over 4k-150k connections
// x 5-80 levels at B = 4, 16, 64 and 256 were about 6.5k + 400 L, 2.8k + 130 L, 0.7k + 45 L and
// 220 L connections, which the factors below follow.
constexpr double kWorkgroupBaseConnections = 13000.0;
constexpr double kWorkgroupConnectionsPerLevel = 1500.0;          // one column per lane
constexpr double kWorkgroupConnectionsPerLevelVec2 = 800.0;       // two
constexpr double kWorkgroupConnectionsPerLevelVec4 = 400.0;       // four
inline double workgroup_break_even(int B, int n_levels) {
    const int vec = vec_for_workgroup(B);
    const int vecs = B / vec;
    int lpg = 1;
    while (lpg < 64 && lpg < vecs) lpg <<= 1;
    const double base = kWorkgroupBaseConnections * (vec == 4 ? 0.5 : vec == 2 ? 0.75 : 1.0) /
                        (lpg > 1 ? (double)lpg / 1.7 : 1.0);
    const double per_level = (vec == 1 ? kWorkgroupConnectionsPerLevel
                                       : vec == 2 ? kWorkgroupConnectionsPerLevelVec2 : kWorkgroupConnectionsPerLevelVec4) /
                             pow((double)lpg, vec == 1 ? 0.42 : 0.8);
    return base + per_level * (double)n_levels;
}

}  // namespace
}  // namespace asnn

using namespace asnn;

namespace asnn {
namespace {
int choose_schedule(const asnn_packed *packed, int32_t B, bool has_workspace, uint32_t flags) {
    const int32_t n_nodes = packed->n_nodes, n_levels = packed->n_levels;
    const uint32_t forced = flags & (ASNN_FLAG_LEVEL_LAUNCHES | ASNN_FLAG_DATAFLOW | ASNN_FLAG_WORKGROUP);
    if (forced & (forced - 1)) return ASNN_ERR_SIZE;            // more than one schedule forced
    const long long n_work = (long long)(packed->n_units - packed->first_unit) * tiles_for(B);
    const bool possible = has_workspace && packed->unit_ptr && n_levels > 1 && packed->n_units > 0 &&
                          packed->first_unit >= 0 && packed->first_unit <= packed->n_units &&
                          n_work > 0 && n_work < 0x3fffffffLL &&
                          carve_activate(nullptr, packed, B).partial_bytes <= 0xffffffffull;
    const bool workgroup_possible = packed->level_ptr != nullptr && tiles_for_workgroup(B) <= 0x7fffffffLL;
    if (flags & ASNN_FLAG_WORKGROUP) return workgroup_possible ? 2 : ASNN_ERR_NULL;
    if (flags & ASNN_FLAG_DATAFLOW) {
        if (!has_workspace) return ASNN_ERR_NULL;
        if (!possible && n_levels > 1) return ASNN_ERR_SIZE;
        return possible ? 1 : 0;
    }
    if (flags & ASNN_FLAG_LEVEL_LAUNCHES) return 0;
    // (one workgroup per tile: beyond the 512 workgroups the chip holds they run in rounds)
    const double workgroup_rounds = ceil((double)tiles_for_workgroup(B) / kDataflowResidentWorkgroups);
    if (workgroup_possible && (double)packed->n_edges * workgroup_rounds <= workgroup_break_even(B, n_levels)) return 2;
    if (!possible) return 0;
    const double per_level = (double)packed->n_edges / (double)(n_levels - 1);
    const bool cached = (double)n_nodes * (double)B * 4.0 <= kCachedValueBytes;
    const double levels_us = kLevelLaunchUs + per_level * (double)B / (cached ? kLevelWorkPerUsCached : kLevelWorkPerUs) +
                             kHeavyRoundUs * (double)(packed->max_heavy_indegree / (kMixedWaves * kUnroll));
    const double hop_us = packed->max_heavy_indegree > kHeavyChunk ? kDataflowSplitHopUs : kDataflowHopUs;
    const double stream_us = per_level * (double)padded_batch(B) / kDataflowWorkPerUs;
    const double items_us = (double)n_work / (double)(n_levels - 1) / kDataflowResidentWorkgroups * kDataflowItemUs;
    double flow_us = stream_us > hop_us ? stream_us : hop_us;
    if (items_us > flow_us) flow_us = items_us;
    flow_us += kDataflowStartUs / (double)(n_levels - 1);
    return flow_us < levels_us ? 1 : 0;
}
}  // namespace
}  // namespace asnn

extern "C" int asnn_activate_schedule(const asnn_packed *packed, int32_t B, int has_workspace, uint32_t flags) {
    if (!packed) return ASNN_ERR_NULL;
    if (packed->n_nodes <= 0 || packed->n_levels <= 0 || packed->n_edges < 0 || B <= 0) return ASNN_ERR_SIZE;
    return choose_schedule(packed, B, has_workspace != 0, flags);
}

extern "C" size_t asnn_activate_workspace_bytes(const asnn_packed *packed, int32_t B) {
    if (!packed || packed->n_nodes <= 0 || packed->n_edges < 0 || B <= 0) return 0;
    return carve_activate(nullptr, packed, B).bytes;
}

// ---- scratch of the entry point that allocates nothing ---------------------
// asnn_activate_static runs asnn_activate with this array in the place of the caller's workspace
// (the control block of the dataflow schedule and the partial sums of split heavy rows).  The
// array's name is only a host-side handle: its device address is looked up once per device, with
// that device current, and from then on only that address is used (every device holds its own
// copy of the array at its own address).
static __device__ __align__(256) unsigned char scratch[ASNN_STATIC_SCRATCH_BYTES];

namespace asnn {
namespace {
int static_scratch(void **out) {
    static std::atomic<void *> address_of[kMaxDevices];
    int dev = 0;
    ASNN_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return ASNN_ERR_NO_DEVICE;
    void *p = address_of[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        ASNN_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (p == nullptr || ((uintptr_t)p & 255u) != 0) return ASNN_ERR_WORKSPACE;
        address_of[dev].store(p, std::memory_order_release);      // (racing threads store the same address)
    }
    *out = p;
    return ASNN_OK;
}
}  // namespace
}  // namespace asnn

extern "C" int asnn_activate_status(const void *workspace, void *stream) {
    ASNN_HIP_TRY(hipStreamSynchronize(static_cast<hipStream_t>(stream)));
    if (!workspace) return ASNN_OK;
    if (workspace == ASNN_STATIC_SCRATCH) {
        void *p = nullptr;
        ASNN_TRY(static_scratch(&p));
        workspace = p;
    }
    DataflowCtl host;
    ASNN_HIP_TRY(hipMemcpy(&host, workspace, sizeof(host), hipMemcpyDeviceToHost));
    return (host.magic == kCtlMagic && host.error) ? ASNN_ERR_TIMEOUT : ASNN_OK;
}

extern "C" int asnn_activate_static(const asnn_packed *packed, const int32_t *input_ids, int32_t n_inputs,
                                    const int32_t *output_ids, int32_t n_outputs, const float *X, int32_t B,
                                    float *V, float *Y, uint32_t flags, void *stream) {
    if (!packed) return ASNN_ERR_NULL;
    if (packed->n_nodes <= 0 || packed->n_edges < 0 || B <= 0) return ASNN_ERR_SIZE;
    if (asnn_activate_workspace_bytes(packed, B) > (size_t)ASNN_STATIC_SCRATCH_BYTES) return ASNN_ERR_SCRATCH;
    void *p = nullptr;
    ASNN_TRY(static_scratch(&p));
    return asnn_activate(packed, input_ids, n_inputs, output_ids, n_outputs, X, B, V, Y, p,
                         (size_t)ASNN_STATIC_SCRATCH_BYTES, flags, stream);
}

extern "C" int asnn_activate(const asnn_packed *packed, const int32_t *input_ids, int32_t n_inputs,
                             const int32_t *output_ids, int32_t n_outputs, const float *X, int32_t B, float *V,
                             float *Y, void *workspace, size_t workspace_bytes, uint32_t flags, void *stream) {
    if (!packed) return ASNN_ERR_NULL;
    const int32_t n_nodes = packed->n_nodes, n_levels = packed->n_levels;
    const int64_t n_edges = packed->n_edges;
    const int32_t *level_ptr_host = packed->level_ptr_host;
    if (n_nodes <= 0 || n_edges < 0 || n_edges >= (int64_t)INT32_MAX || n_levels <= 0 || n_inputs < 0 ||
        n_outputs < 0 || B <= 0)
        return ASNN_ERR_SIZE;
    if ((int64_t)n_nodes * (int64_t)B >= ((int64_t)1 << 40)) return ASNN_ERR_SIZE;
    if (!level_ptr_host || !packed->row_ptr || !packed->inv_perm || !V) return ASNN_ERR_NULL;
    if (n_edges > 0 && (!packed->col || !packed->w)) return ASNN_ERR_NULL;
    if (n_inputs > 0 && (!input_ids || !X)) return ASNN_ERR_NULL;
    if (Y && n_outputs > 0 && !output_ids) return ASNN_ERR_NULL;
    if (((uintptr_t)V & 15u) != 0) return ASNN_ERR_SIZE;
    // the level table must be a monotone cover of the rows
    const int n_keys = ASNN_CLASSES * n_levels;
    if (level_ptr_host[0] != 0 || level_ptr_host[n_keys] != n_nodes) return ASNN_ERR_SIZE;
    for (int k = 0; k < n_keys; ++k)
        if (level_ptr_host[k] > level_ptr_host[k + 1]) return ASNN_ERR_SIZE;
    const int plan = choose_schedule(packed, B, workspace != nullptr, flags);
    if (plan < 0) return plan;
    const bool dataflow = plan == 1;
    const int tiles = tiles_for(B);
    const int first_row = n_levels > 1 ? level_ptr_host[ASNN_CLASSES] : n_nodes;
    const long long n_work = (long long)(packed->n_units - packed->first_unit) * tiles;
    if (dataflow && (((uintptr_t)workspace & 255u) != 0 || workspace_bytes < asnn_activate_workspace_bytes(packed, B)))
        return ASNN_ERR_WORKSPACE;

    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool f32 = (flags & ASNN_FLAG_ACC_F32) != 0;
    const int raw = (flags & ASNN_FLAG_RAW_INPUTS) ? 1 : 0;
    LevelArgs a{packed->row_ptr, packed->col, packed->w, V, B, s};

    if (plan == 2) {        // staging, every level and the output copy in one launch
        WorkgroupArgs g{packed->level_ptr, n_levels, input_ids, packed->inv_perm, X, n_inputs, raw,
                        output_ids, n_outputs > 0 ? Y : nullptr, n_outputs, n_nodes, n_edges};
        return f32 ? launch_workgroup_any<float>(a, g) : launch_workgroup_any<double>(a, g);
    }

    // Level 0 has no incoming connections: every row of it gets sigmoid(0), then the sensors take
    // their inputs.  (The fill is not skipped when the level holds as many rows as there are input
    // ids: the ids are the caller's, unchecked here, and one that is out of range or listed twice
    // would leave a root that is no sensor unwritten.)
    {
        const size_t n0 = (size_t)level_ptr_host[ASNN_CLASSES] * (size_t)B;
        if (n0 > 0) {
            const dim3 grid(blocks_for(n0, 256 * 4, 4096));
            if (f32)
                hipLaunchKernelGGL(fill_half_kernel<float>, grid, dim3(256), 0, s, V, n0);
            else
                hipLaunchKernelGGL(fill_half_kernel<double>, grid, dim3(256), 0, s, V, n0);
            ASNN_HIP_TRY(hipGetLastError());
        }
        if (n_inputs > 0 && !dataflow) {
            const unsigned blocks = blocks_for((size_t)n_inputs * (size_t)B, 256, 8192);
            if (f32)
                hipLaunchKernelGGL(stage_inputs_kernel<float>, dim3(blocks), dim3(256), 0, s, input_ids,
                                   (const int32_t *)packed->inv_perm, X, V, n_inputs, n_nodes, B, raw);
            else
                hipLaunchKernelGGL(stage_inputs_kernel<double>, dim3(blocks), dim3(256), 0, s, input_ids,
                                   (const int32_t *)packed->inv_perm, X, V, n_inputs, n_nodes, B, raw);
            ASNN_HIP_TRY(hipGetLastError());
        }
    }
    if (dataflow) {
        static std::atomic<int> cus_of[kMaxDevices];
        int dev = 0;
        ASNN_HIP_TRY(hipGetDevice(&dev));
        if (dev < 0 || dev >= kMaxDevices) return ASNN_ERR_NO_DEVICE;
        int cus = cus_of[dev].load(std::memory_order_relaxed);
        if (cus == 0) {
            int n = 0;
            ASNN_HIP_TRY(hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev));
            cus = n > 0 ? n : 1;
            cus_of[dev].store(cus, std::memory_order_relaxed);
        }
        // work items and output items are numbered by one 32-bit counter
        if ((long long)((n_outputs + kMixedWaves - 1) / kMixedWaves) * tiles >= 0x3fffffffLL) return ASNN_ERR_SIZE;
        ActivateWorkspace ws = carve_activate(workspace, packed, B);
        const size_t n_values = (size_t)(n_nodes - first_row) * (size_t)B;
        unsigned int *v_begin = reinterpret_cast<unsigned int *>(V + (size_t)first_row * (size_t)B);
        const size_t n_partial_words = ws.partial_bytes / sizeof(unsigned int);
        if (n_inputs > 0) {
            const size_t most = n_values > (size_t)n_inputs * (size_t)B ? n_values : (size_t)n_inputs * (size_t)B;
            const unsigned blocks = blocks_for(most, 256 * 8, 4096);
            if (f32)
                hipLaunchKernelGGL(dataflow_prologue_kernel<float>, dim3(blocks), dim3(256), 0, s, input_ids,
                                   (const int32_t *)packed->inv_perm, X, V, n_inputs, n_nodes, B, raw, v_begin, n_values,
                                   ws.partials, n_partial_words, ws.ctl);
            else
                hipLaunchKernelGGL(dataflow_prologue_kernel<double>, dim3(blocks), dim3(256), 0, s, input_ids,
                                   (const int32_t *)packed->inv_perm, X, V, n_inputs, n_nodes, B, raw, v_begin, n_values,
                                   ws.partials, n_partial_words, ws.ctl);
        } else {
            hipLaunchKernelGGL(dataflow_reset_kernel, dim3(blocks_for(n_values, 256 * 8, 4096)), dim3(256), 0, s, v_begin,
                               n_values, ws.partials, n_partial_words, ws.ctl);
        }
        ASNN_HIP_TRY(hipGetLastError());
        const int units_per_level = (packed->n_units - packed->first_unit + n_levels - 2) / (n_levels - 1);
        DataflowArgs d{packed->unit_ptr, packed->first_unit, (int)n_work, first_row, ws.ctl, cus, units_per_level,
                       ws.partials, (uint32_t)ws.partial_bytes, output_ids, packed->inv_perm, Y,
                       (Y && n_outputs > 0) ? n_outputs : 0, n_nodes};
        ASNN_TRY(f32 ? launch_dataflow_any<float>(a, d) : launch_dataflow_any<double>(a, d));
        return ASNN_OK;      // the outputs were copied by the same launch
    } else {
        for (int l = 1; l < n_levels; ++l) {
            const int32_t *lp = level_ptr_host + ASNN_CLASSES * l;
            ASNN_TRY(f32 ? launch_level_any<float>(a, lp[0], lp[1], lp[2], lp[3])
                         : launch_level_any<double>(a, lp[0], lp[1], lp[2], lp[3]));
        }
    }
    if (Y && n_outputs > 0) {
        const unsigned blocks = blocks_for((size_t)n_outputs * (size_t)B, 256, 8192);
        hipLaunchKernelGGL(extract_outputs_kernel, dim3(blocks), dim3(256), 0, s, output_ids,
                           (const int32_t *)packed->inv_perm, (const float *)V, Y, n_outputs, n_nodes, B);
        ASNN_HIP_TRY(hipGetLastError());
    }
    return ASNN_OK;
}
