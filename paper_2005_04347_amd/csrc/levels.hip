// asnn_build_levels: dependency layers of an ASNN on the GPU.
//
// The paper segments the network on the CPU with a set-based loop that rescans
// every connection per layer and names GPU segmentation as future work.  The
// same layers come out of a frontier (Kahn) sweep: a node joins layer k+1 in
// the sweep that removes its last unassigned predecessor, which is exactly
// "its entire input set is already assigned" and makes its layer one more
// than its deepest predecessor.  All arithmetic is integer; the result is
// unique, so the order in which atomics land does not matter.
#include "asnn_common.h"

namespace asnn {

namespace {

constexpr int kThreads = 256;
constexpr int kSweepsPerSync = 64;     // frontier sweeps enqueued between two host reads
constexpr int kGroup = 16;             // lanes that share one frontier node's out-edges
// Grid-wide sweeps: 256 workgroups of 512 threads.  Larger workgroups add up more releases of a hot destination
// before they touch its counter (a deep network with such destinations in every layer: 9.9 -> 9.0 ms against 512
// workgroups of 256 threads; 1024 threads gain a little more there and lose 10 % where there are none).
constexpr int kSweepThreads = 512;
constexpr unsigned kSweepBlocks = 256;
constexpr unsigned kReachBlocks = 512;    // the backward sweeps of the required set: workgroups of kThreads
constexpr int kBatch = 4;              // out-edges a lane releases per round trip: a node with up to 64 takes one
constexpr int kFoundCap = 2048;        // frontier nodes a workgroup collects in LDS before appending them
// A destination with this many incoming connections can receive thousands of returning atomics
// on its counter in one sweep, which serialise.  Its entries in the out-adjacency carry kHotBit, and
// a workgroup first adds up its releases of such destinations in a small LDS hash table.
constexpr int kHotIndegree = ASNN_HEAVY_INDEGREE;
constexpr int32_t kHotBit = INT32_MIN;
constexpr int kHotSlots = 1024;        // hash slots per workgroup
constexpr int kHotProbes = 16;         // after that many occupied slots the release goes straight to memory
// Narrow frontiers: one workgroup runs sweep after sweep without leaving the device.
constexpr int kNarrowThreads = 1024;
constexpr int kNarrowCap = 2048;       // frontier nodes it keeps in LDS
constexpr int kNarrowMaxEdges = 4096;  // out-edges of one frontier it still takes alone (a single compute unit issues about one request per clock)
constexpr int kNarrowBatch = 16;       // out-edges a thread releases per round trip
constexpr int kNarrowBigOut = 64;      // out-degree from which the whole workgroup shares a node
constexpr int64_t kSortedAdjacencyEdges = 1 << 21;     // connections from which the out-adjacency is sorted, not counted

// Slots of the small control block in device memory.
enum Ctl : int {
    kErr = 0,          // first error code seen (0 = none)
    kAssigned = 1,     // nodes that received a level so far
    kLevels = 2,       // number of non-empty frontiers so far
    kSweep = 3,        // index of the next sweep (written by narrow_sweeps_kernel)
    kCount0 = 4,       // three rotating frontier sizes: sweep k reads kCount0 + k % 3
    kCtlInts = 16
};

__device__ inline void flag_error(int *ctl, int code) { atomicCAS(&ctl[kErr], 0, code); }

// Appends `node` to list[] for every active lane with `has` set, with one atomic
// on *count per wavefront instead of one per lane (thousands of lanes adding
// to one address serialise).  May be called from divergent code.
__device__ inline void wave_append(bool has, int32_t node, int32_t *__restrict__ list, int *count) {
    const unsigned long long mask = __ballot(has);
    if (mask == 0) return;
    const int lane = threadIdx.x & (kWave - 1);
    const int leader = __ffsll((long long)mask) - 1;
    int base = 0;
    if (lane == leader) base = atomicAdd(count, __popcll(mask));
    base = __shfl(base, leader, kWave);
    const unsigned long long below = (lane == 0) ? 0ull : (~0ull >> (kWave - lane));
    if (has) list[base + __popcll(mask & below)] = node;
}

// Checks every connection's ids and, with indeg given, counts the incoming connections of every
// node (the counters the sweeps count down).
__global__ void check_and_count_kernel(const int32_t *__restrict__ src, const int32_t *__restrict__ dst, int64_t n_edges,
                                       int32_t n_nodes, int32_t *indeg, int *ctl) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n_edges; e += stride) {
        const int32_t a = src[e], b = dst[e];
        if (a < 0 || a >= n_nodes || b < 0 || b >= n_nodes) {
            flag_error(ctl, ASNN_ERR_INDEX);
            continue;
        }
        if (indeg != nullptr) atomicAdd(&indeg[b], 1);
    }
}

__global__ void mark_inputs_kernel(const int32_t *__restrict__ input_ids, int32_t n_inputs, int32_t n_nodes,
                                   const int32_t *__restrict__ indeg, int32_t *is_input, int *ctl) {
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= n_inputs) return;
    const int32_t v = input_ids[k];
    if (v < 0 || v >= n_nodes) { flag_error(ctl, ASNN_ERR_INDEX); return; }
    if (atomicAdd(&is_input[v], 1) != 0) flag_error(ctl, ASNN_ERR_DUP_INPUT);
    if (indeg[v] != 0) flag_error(ctl, ASNN_ERR_INPUT_HAS_INEDGE);
}

// Small networks: out-degree histogram with atomics (together with the in-degree counters), ...
__global__ void degree_kernel(const int32_t *__restrict__ from, const int32_t *__restrict__ to, int64_t n_edges,
                              int32_t n_nodes, int32_t *indeg, int32_t *outdeg, int *ctl) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n_edges; e += stride) {
        const int32_t a = from[e], b = to[e];
        if (a < 0 || a >= n_nodes || b < 0 || b >= n_nodes) {
            flag_error(ctl, ASNN_ERR_INDEX);
            continue;
        }
        if (indeg != nullptr) atomicAdd(&indeg[b], 1);
        atomicAdd(&outdeg[a], 1);
    }
}

// ... and a scatter into the lists with one returning atomic per connection (the order inside a
// list is irrelevant for levels).  Hot destinations are marked as in out_pair_kernel.
__global__ void fill_out_kernel(const int32_t *__restrict__ from, const int32_t *__restrict__ to, int64_t n_edges,
                                int32_t n_nodes, const int32_t *__restrict__ out_ptr, int32_t *cursor,
                                const int32_t *__restrict__ indeg, int32_t *__restrict__ out_dst) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n_edges; e += stride) {
        const int32_t a = from[e], b = to[e];
        if (a < 0 || a >= n_nodes || b < 0 || b >= n_nodes) continue;   // already flagged
        const int32_t pos = out_ptr[a] + atomicAdd(&cursor[a], 1);
        out_dst[pos] = (indeg != nullptr && indeg[b] >= kHotIndegree) ? (b | kHotBit) : b;
    }
}

// Large networks: the out-adjacency comes from a stable sort of (source, destination) pairs by
// source instead (from a few million connections on, two atomics per connection cost more than
// the sort passes; below, the sort's extra launches do).  Key = source, value = destination; with indeg given (the final in-degrees: the sweeps
// have not started), destinations with many incoming connections are marked with kHotBit.  A
// connection with an id out of range (already flagged) is filed under node 0 -> node 0, so that
// nothing reads out of bounds before the host sees the error.
__global__ void out_pair_kernel(const int32_t *__restrict__ from, const int32_t *__restrict__ to, int64_t n_edges,
                                int32_t n_nodes, const int32_t *__restrict__ indeg, uint32_t *__restrict__ keys,
                                uint32_t *__restrict__ vals) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n_edges; e += stride) {
        int32_t a = from[e], b = to[e];
        if (a < 0 || a >= n_nodes || b < 0 || b >= n_nodes) a = b = 0;
        keys[e] = (uint32_t)a;
        vals[e] = (uint32_t)((indeg != nullptr && indeg[b] >= kHotIndegree) ? (b | kHotBit) : b);
    }
}

// Level 0 = every node without an incoming connection.
// Grid-stride over the nodes; a workgroup collects its roots in LDS and appends them with one
// atomic on the frontier size (see sweep_kernel).
__global__ __launch_bounds__(kThreads) void first_frontier_kernel(int32_t n_nodes, const int32_t *__restrict__ indeg,
                                                                   int32_t *__restrict__ level,
                                                                   int32_t *__restrict__ frontier, int *ctl) {
    __shared__ int32_t found[kFoundCap];
    __shared__ int n_found, found_base;
    if (threadIdx.x == 0) n_found = 0;
    __syncthreads();
    const int stride = gridDim.x * kThreads;
    for (int v = blockIdx.x * kThreads + threadIdx.x; v < n_nodes; v += stride) {
        const int32_t d = indeg[v];
        level[v] = d == 0 ? 0 : -1;
        if (d == 0) {
            const int pos = atomicAdd(&n_found, 1);                      // LDS
            if (pos < kFoundCap) found[pos] = v;
            else frontier[atomicAdd(&ctl[kCount0], 1)] = v;              // LDS list full: append directly
        }
    }
    __syncthreads();
    const int n = min(n_found, kFoundCap);
    if (threadIdx.x == 0 && n > 0) found_base = atomicAdd(&ctl[kCount0], n);
    __syncthreads();
    for (int i = threadIdx.x; i < n; i += kThreads) frontier[found_base + i] = found[i];
}

// Adds one release of hot destination u to the workgroup's hash table (slot_node preset to -1,
// slot_count to 0).  Returns false when kHotProbes slots in a row belong to other nodes: the
// caller then releases u in memory like any other destination.
__device__ inline bool hot_add(int32_t u, int32_t *slot_node, int32_t *slot_count) {
    unsigned h = ((unsigned)u * 2654435761u) >> 12;
    for (int probe = 0; probe < kHotProbes; ++probe, ++h) {
        h &= (unsigned)(kHotSlots - 1);
        const int32_t seen = atomicCAS(&slot_node[h], -1, u);
        if (seen == -1 || seen == u) {
            atomicAdd(&slot_count[h], 1);
            return true;
        }
    }
    return false;
}

// One sweep: every node of frontier k releases its out-edges; a destination
// whose remaining in-degree drops to zero gets level k+1 and joins frontier k+1.
// A sweep over an empty frontier does nothing, so the host may enqueue more
// sweeps than the network has layers.
//
// 16 lanes share one frontier node's out-edges, kBatch of them per lane and round trip (with one
// per round trip, every node with more than 16 out-edges held its layer up by a second round).  The
// nodes a workgroup adds to
// the next frontier are collected in LDS and appended with ONE atomic on the
// frontier size (with tens of thousands of nodes per frontier, one atomic per
// wavefront on that single address was most of the sweep time).  Releases of
// hot destinations are first added up per workgroup in LDS, so such a
// destination is decremented once per workgroup, by the number of connections
// the workgroup's nodes send it.
__global__ __launch_bounds__(kSweepThreads) void sweep_kernel(int k, const int32_t *__restrict__ out_ptr,
                                                          const int32_t *__restrict__ out_dst, int32_t *indeg,
                                                          int32_t *__restrict__ level,
                                                          const int32_t *__restrict__ frontier_in,
                                                          int32_t *__restrict__ frontier_out, int *ctl) {
    __shared__ int32_t slot_node[kHotSlots];
    __shared__ int32_t slot_count[kHotSlots];
    __shared__ int32_t found[kFoundCap];
    __shared__ int n_found, found_base, n_hot;
    const int count = ctl[kCount0 + k % 3];
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        ctl[kCount0 + (k + 2) % 3] = 0;          // read by sweep k-1 (finished), filled by sweep k+1
        if (count > 0) {
            ctl[kLevels] = k + 1;
            atomicAdd(&ctl[kAssigned], count);
        }
    }
    if (count == 0) return;
    int *count_out = &ctl[kCount0 + (k + 1) % 3];
    constexpr int kNodesPerBlock = kSweepThreads / kGroup;
    const int sub = threadIdx.x % kGroup;
    const int stride = gridDim.x * kNodesPerBlock;
    if (threadIdx.x == 0) { n_found = 0; n_hot = 0; }
    for (int i = threadIdx.x; i < kHotSlots; i += kSweepThreads) { slot_node[i] = -1; slot_count[i] = 0; }
    __syncthreads();
    auto assign = [&](int32_t u) {
        level[u] = k + 1;
        const int pos = atomicAdd(&n_found, 1);                  // LDS
        if (pos < kFoundCap) found[pos] = u;
        else frontier_out[atomicAdd(count_out, 1)] = u;          // LDS list full: append directly
    };
    for (int f = blockIdx.x * kNodesPerBlock + threadIdx.x / kGroup; f < count; f += stride) {
        const int32_t v = frontier_in[f];
        const int32_t end = out_ptr[v + 1];
        for (int32_t x = out_ptr[v] + sub; x < end; x += kGroup * kBatch) {
            // all loads, then all decrements, then what they returned: one round trip each per kBatch
            // out-edges (positions past the end re-read the last one and are not released)
            int32_t raw[kBatch], old[kBatch];
#pragma unroll
            for (int j = 0; j < kBatch; ++j) raw[j] = out_dst[min(x + j * kGroup, end - 1)];
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                old[j] = 0;
                if (x + j * kGroup < end && raw[j] >= 0) old[j] = atomicSub(&indeg[raw[j]], 1);
            }
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                if (x + j * kGroup >= end) continue;
                if (raw[j] >= 0) {
                    if (old[j] == 1) assign(raw[j]);
                    continue;
                }
                const int32_t u = raw[j] & ~kHotBit;
                if (hot_add(u, slot_node, slot_count)) n_hot = 1;            // LDS, same value from every writer
                else if (atomicSub(&indeg[u], 1) == 1) assign(u);
            }
        }
    }
    __syncthreads();
    if (n_hot != 0) {                                            // block-uniform
        for (int i = threadIdx.x; i < kHotSlots; i += kSweepThreads) {
            const int32_t u = slot_node[i];
            if (u >= 0) {
                const int32_t c = slot_count[i];
                if (atomicSub(&indeg[u], c) == c) assign(u);
            }
        }
        __syncthreads();
    }
    const int n = min(n_found, kFoundCap);
    if (threadIdx.x == 0 && n > 0) found_base = atomicAdd(count_out, n);
    __syncthreads();
    for (int i = threadIdx.x; i < n; i += kSweepThreads) frontier_out[found_base + i] = found[i];
}

// Narrow frontiers.  A network with many small layers spends its sweeps on launches and on the
// chain of device round trips inside each (frontier size, node, out-range, destination,
// counter).  ONE workgroup therefore runs sweep after sweep, starting with sweep k0, for as long as
// the frontier fits its LDS (kNarrowCap nodes, kNarrowMaxEdges out-edges): the frontier never leaves
// LDS, the layer barrier is a workgroup barrier, and a thread releases up to kNarrowBatch out-edges
// of its node per round trip.  It stops at the first frontier that is empty (the network is done) or
// too wide; that frontier is then in frontier_a/frontier_b (by the parity of its sweep index) with
// its size in the control block, and ctl[kSweep] names the sweep that comes next, exactly as
// sweep_kernel expects it.
__global__ __launch_bounds__(kNarrowThreads) void narrow_sweeps_kernel(int k0, const int32_t *__restrict__ out_ptr,
                                                                       const int32_t *__restrict__ out_dst,
                                                                       int32_t *indeg, int32_t *__restrict__ level,
                                                                       int32_t *frontier_a, int32_t *frontier_b,
                                                                       int *ctl) {
    __shared__ int32_t fr[2][kNarrowCap];            // current and next frontier
    __shared__ int32_t e_begin[kNarrowCap], e_end[kNarrowCap];
    __shared__ int32_t big[kNarrowCap];              // positions of frontier nodes with many out-edges
    __shared__ int32_t slot_node[kHotSlots];
    __shared__ int32_t slot_count[kHotSlots];
    __shared__ int n_next, n_big, n_edges_out, n_hot;
    const int tid = threadIdx.x;
    int k = k0;
    int n_cur = ctl[kCount0 + k % 3];
    if (n_cur <= 0 || n_cur > kNarrowCap) {          // block-uniform: nothing for this kernel to do
        if (tid == 0) ctl[kSweep] = k;
        return;
    }
    {
        const int32_t *f0 = (k & 1) ? frontier_b : frontier_a;
        for (int i = tid; i < n_cur; i += kNarrowThreads) fr[0][i] = f0[i];
    }
    int cur = 0;
    int assigned = 0, levels = 0;                    // what thread 0 reports at the end
    bool in_lds_only = false;                        // the current frontier is not in global memory
    int n_exit;                                      // size of the frontier the next kernel starts with
    for (;;) {
        if (tid == 0) { n_next = 0; n_big = 0; n_edges_out = 0; n_hot = 0; }
        for (int i = tid; i < kHotSlots; i += kNarrowThreads) { slot_node[i] = -1; slot_count[i] = 0; }
        __syncthreads();
        int mine = 0;
        for (int i = tid; i < n_cur; i += kNarrowThreads) {
            const int32_t v = fr[cur][i];
            const int32_t b = out_ptr[v], e = out_ptr[v + 1];
            e_begin[i] = b;
            e_end[i] = e;
            mine += e - b;
            if (e - b > kNarrowBigOut) big[atomicAdd(&n_big, 1)] = i;
        }
        if (mine > 0) atomicAdd(&n_edges_out, min(mine, kNarrowMaxEdges + 1));      // the sum cannot overflow
        __syncthreads();
        if (n_edges_out > kNarrowMaxEdges) {         // block-uniform: too much work for one workgroup
            n_exit = n_cur;
            if (in_lds_only) {
                int32_t *f = (k & 1) ? frontier_b : frontier_a;
                for (int i = tid; i < n_cur; i += kNarrowThreads) f[i] = fr[cur][i];
            }
            break;
        }
        assigned += n_cur;
        levels = k + 1;
        int32_t *spill = ((k + 1) & 1) ? frontier_b : frontier_a;      // where frontier k+1 goes beyond the LDS list
        int32_t *next = fr[cur ^ 1];
        auto assign = [&](int32_t u) {
            level[u] = k + 1;
            const int pos = atomicAdd(&n_next, 1);               // LDS
            if (pos < kNarrowCap) next[pos] = u;
            else spill[pos] = u;                                 // positions are final: this kernel owns the whole frontier
        };
        auto release = [&](int32_t raw) {
            const int32_t u = raw & ~kHotBit;
            if (raw < 0 && hot_add(u, slot_node, slot_count)) {
                n_hot = 1;
                return;
            }
            if (atomicSub(&indeg[u], 1) == 1) assign(u);
        };
        // one thread per frontier node, kNarrowBatch out-edges per round trip
        for (int i = tid; i < n_cur; i += kNarrowThreads) {
            const int32_t b = e_begin[i], e = e_end[i];
            if (e - b > kNarrowBigOut) continue;
            for (int32_t x = b; x < e; x += kNarrowBatch) {
                int32_t raw[kNarrowBatch], old[kNarrowBatch];
#pragma unroll
                for (int j = 0; j < kNarrowBatch; ++j) raw[j] = out_dst[min(x + j, e - 1)];
#pragma unroll
                for (int j = 0; j < kNarrowBatch; ++j) {
                    old[j] = 0;
                    if (x + j < e && raw[j] >= 0) old[j] = atomicSub(&indeg[raw[j]], 1);
                }
#pragma unroll
                for (int j = 0; j < kNarrowBatch; ++j) {
                    if (x + j >= e) continue;
                    if (raw[j] >= 0) {
                        if (old[j] == 1) assign(raw[j]);
                    } else {
                        release(raw[j]);
                    }
                }
            }
        }
        // nodes with many out-edges: the whole workgroup strides over each one's list
        const int nb = n_big;                        // block-uniform (written before the last barrier)
        for (int q = 0; q < nb; ++q) {
            const int i = big[q];
            const int32_t e = e_end[i];
            for (int32_t x = e_begin[i] + tid; x < e; x += kNarrowThreads) release(out_dst[x]);
        }
        __syncthreads();
        if (n_hot != 0) {                            // block-uniform
            for (int i = tid; i < kHotSlots; i += kNarrowThreads) {
                const int32_t u = slot_node[i];
                if (u >= 0) {
                    const int32_t c = slot_count[i];
                    if (atomicSub(&indeg[u], c) == c) assign(u);
                }
            }
            __syncthreads();
        }
        const int n = n_next;                        // block-uniform
        ++k;
        if (n == 0 || n > kNarrowCap) {
            n_exit = n;
            if (n > kNarrowCap)                      // the first kNarrowCap nodes join the rest in global memory
                for (int i = tid; i < kNarrowCap; i += kNarrowThreads) spill[i] = next[i];
            break;
        }
        cur ^= 1;
        n_cur = n;
        in_lds_only = true;
        __syncthreads();                             // n_next is reset at the top of the loop
    }
    if (tid == 0) {
        if (assigned > 0) {
            atomicAdd(&ctl[kAssigned], assigned);
            ctl[kLevels] = levels;
        }
        ctl[kSweep] = k;
        ctl[kCount0 + k % 3] = n_exit;
        ctl[kCount0 + (k + 1) % 3] = 0;
        ctl[kCount0 + (k + 2) % 3] = 0;
    }
}

}  // namespace

struct LevelsWorkspace {
    int *ctl;
    int32_t *indeg, *out_ptr, *first, *is_input, *frontier_a, *frontier_b, *scan_tmp, *radix_tmp;
    uint32_t *keys_a, *keys_b, *vals_a, *vals_b;     // sort buffers; the out-adjacency ends up in one of the vals
    size_t bytes;
};

static LevelsWorkspace carve_levels(void *ws, int32_t n_nodes, int64_t n_edges) {
    Carver c(ws);
    LevelsWorkspace w;
    const size_t n = (size_t)n_nodes, e = (size_t)n_edges;
    w.ctl = c.take<int>(kCtlInts);
    w.indeg = c.take<int32_t>(n + 1);
    w.out_ptr = c.take<int32_t>(n + 1);
    w.first = c.take<int32_t>(n + 1);
    w.is_input = c.take<int32_t>(n + 1);
    w.keys_a = c.take<uint32_t>(e + 1);
    w.keys_b = c.take<uint32_t>(e + 1);
    w.vals_a = c.take<uint32_t>(e + 1);
    w.vals_b = c.take<uint32_t>(e + 1);
    w.frontier_a = c.take<int32_t>(n + 1);
    w.frontier_b = c.take<int32_t>(n + 1);
    w.scan_tmp = c.take<int32_t>(scan_tmp_ints(n + 1));
    w.radix_tmp = c.take<int32_t>(radix_tmp_ints(e + 1));
    w.bytes = c.off;
    return w;
}

// Groups the connections from[e] -> to[e] by `from`: w.out_ptr[n_nodes + 1] and, through *adjacent,
// the `to` ids of each node, contiguous (in edge-list order when they were sorted).  count_incoming also fills w.indeg
// (and marks hot destinations in the lists).  Clears the control block and the per-node arrays first.
static int group_connections(const LevelsWorkspace &w, int32_t n_nodes, int64_t n_edges, const int32_t *from,
                             const int32_t *to, bool count_incoming, hipStream_t s, const int32_t **adjacent) {
    // ctl, indeg, out_ptr, first and is_input are adjacent: clear them in one go.
    const size_t clear_bytes = (size_t)((char *)w.keys_a - (char *)w.ctl);
    ASNN_HIP_TRY(hipMemsetAsync(w.ctl, 0, clear_bytes, s));
    *adjacent = reinterpret_cast<const int32_t *>(w.vals_a);
    int32_t *indeg = count_incoming ? w.indeg : (int32_t *)nullptr;
    const dim3 grid(blocks_for((size_t)(n_edges > 0 ? n_edges : 1), kThreads, 65535)), block(kThreads);
    if (n_edges > 0 && n_edges < kSortedAdjacencyEdges) {
        hipLaunchKernelGGL(degree_kernel, grid, block, 0, s, from, to, n_edges, n_nodes, indeg, w.out_ptr, w.ctl);
        ASNN_HIP_TRY(hipGetLastError());
        ASNN_TRY(exclusive_scan_i32(w.out_ptr, w.out_ptr, (size_t)n_nodes + 1, w.scan_tmp, s));
        hipLaunchKernelGGL(fill_out_kernel, grid, block, 0, s, from, to, n_edges, n_nodes, (const int32_t *)w.out_ptr,
                           w.first, (const int32_t *)indeg, reinterpret_cast<int32_t *>(w.vals_a));
        ASNN_HIP_TRY(hipGetLastError());
        return ASNN_OK;
    }
    if (n_edges > 0) {
        hipLaunchKernelGGL(check_and_count_kernel, grid, block, 0, s, from, to, n_edges, n_nodes, indeg, w.ctl);
        ASNN_HIP_TRY(hipGetLastError());
        hipLaunchKernelGGL(out_pair_kernel, grid, block, 0, s, from, to, n_edges, n_nodes, (const int32_t *)indeg, w.keys_a,
                           w.vals_a);
        ASNN_HIP_TRY(hipGetLastError());
        uint32_t *ks = nullptr, *vs = nullptr;
        ASNN_TRY(radix_sort_pairs_u32(w.keys_a, w.vals_a, w.keys_b, w.vals_b, (size_t)n_edges,
                                      bits_for((uint64_t)n_nodes - 1), w.radix_tmp, s, &ks, &vs));
        *adjacent = reinterpret_cast<const int32_t *>(vs);
        ASNN_TRY(sorted_run_lengths(ks, (size_t)n_edges, w.first, w.out_ptr, s));
    }
    // out-degree histogram -> out_ptr (n_nodes + 1 entries; the extra zero yields the total)
    return exclusive_scan_i32(w.out_ptr, w.out_ptr, (size_t)n_nodes + 1, w.scan_tmp, s);
}

}  // namespace asnn

using namespace asnn;

extern "C" size_t asnn_levels_workspace_bytes(int32_t n_nodes, int64_t n_edges) {
    if (n_nodes < 0 || n_edges < 0) return 0;
    return carve_levels(nullptr, n_nodes, n_edges).bytes;
}

extern "C" int asnn_build_levels(int32_t n_nodes, int64_t n_edges, const int32_t *src, const int32_t *dst,
                                 const int32_t *input_ids, int32_t n_inputs, int32_t *level_out, int32_t *n_levels_out,
                                 void *workspace, size_t workspace_bytes, void *stream) {
    if (n_nodes < 0 || n_edges < 0 || n_edges > (int64_t)ASNN_MAX_EDGES || n_inputs < 0) return ASNN_ERR_SIZE;
    if (!n_levels_out) return ASNN_ERR_NULL;
    if (n_nodes == 0) {
        if (n_edges > 0 || n_inputs > 0) return ASNN_ERR_INDEX;
        *n_levels_out = 0;
        return ASNN_OK;
    }
    if (!level_out || (n_edges > 0 && (!src || !dst)) || (n_inputs > 0 && !input_ids)) return ASNN_ERR_NULL;
    if (!workspace) return ASNN_ERR_NULL;
    if (((uintptr_t)workspace & 255u) != 0 || workspace_bytes < asnn_levels_workspace_bytes(n_nodes, n_edges))
        return ASNN_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    LevelsWorkspace w = carve_levels(workspace, n_nodes, n_edges);

    const int32_t *out_dst = nullptr;
    ASNN_TRY(group_connections(w, n_nodes, n_edges, src, dst, true, s, &out_dst));
    if (n_inputs > 0) {
        hipLaunchKernelGGL(mark_inputs_kernel, dim3(blocks_for((size_t)n_inputs, kThreads)), dim3(kThreads), 0, s,
                           input_ids, n_inputs, n_nodes, (const int32_t *)w.indeg, w.is_input, w.ctl);
        ASNN_HIP_TRY(hipGetLastError());
    }
    hipLaunchKernelGGL(first_frontier_kernel, dim3(blocks_for((size_t)n_nodes, 4 * kThreads, 2048)), dim3(kThreads), 0, s,
                       n_nodes, (const int32_t *)w.indeg, level_out, w.frontier_a, w.ctl);
    ASNN_HIP_TRY(hipGetLastError());

    // Grid-wide sweeps are enqueued kSweepsPerSync at a time between two looks at the control block.
    // Where the frontier looks small enough for one workgroup (its size times the mean out-degree),
    // narrow_sweeps_kernel takes over and runs sweep after sweep on the device until the frontier is
    // empty or outgrows it.  The first frontier is not known to the host: small networks start narrow.
    const int64_t mean_out = n_edges / n_nodes > 1 ? n_edges / n_nodes : 1;
    bool narrow = n_edges <= 16LL * kNarrowMaxEdges;
    int host_ctl[kCtlInts];
    int k = 0;
    for (;;) {
        if (narrow) {
            hipLaunchKernelGGL(narrow_sweeps_kernel, dim3(1), dim3(kNarrowThreads), 0, s, k, (const int32_t *)w.out_ptr,
                               out_dst, w.indeg, level_out, w.frontier_a, w.frontier_b, w.ctl);
            ASNN_HIP_TRY(hipGetLastError());
        } else {
            for (int i = 0; i < kSweepsPerSync; ++i, ++k) {
                const int32_t *fin = (k & 1) ? w.frontier_b : w.frontier_a;
                int32_t *fout = (k & 1) ? w.frontier_a : w.frontier_b;
                hipLaunchKernelGGL(sweep_kernel, dim3(kSweepBlocks), dim3(kSweepThreads), 0, s, k, (const int32_t *)w.out_ptr,
                                   out_dst, w.indeg, level_out, fin, fout, w.ctl);
                ASNN_HIP_TRY(hipGetLastError());
            }
        }
        ASNN_HIP_TRY(hipMemcpyAsync(host_ctl, w.ctl, sizeof(host_ctl), hipMemcpyDeviceToHost, s));
        ASNN_HIP_TRY(hipStreamSynchronize(s));
        if (host_ctl[kErr] != 0) return host_ctl[kErr];
        if (narrow) k = host_ctl[kSweep];
        if (k < 0 || k > n_nodes + kSweepsPerSync) break;     // cannot happen: at most n_nodes layers
        const int count = host_ctl[kCount0 + k % 3];         // the frontier the next sweep would read
        if (count == 0) break;
        // a narrow run that stopped on a non-empty frontier found it too wide: grid-wide sweeps next
        narrow = !narrow && count <= kNarrowCap && (int64_t)count * mean_out <= kNarrowMaxEdges;
    }
    if (host_ctl[kAssigned] != n_nodes) return ASNN_ERR_CYCLE;
    *n_levels_out = host_ctl[kLevels];
    return ASNN_OK;
}

// ------------------------------------------------------------ required set
// The segmentation algorithm only layers nodes of the "required" set R: the
// nodes needed to compute the outputs.  R is what reaches an output, found by
// the same frontier sweep on the transposed graph (out-adjacency of (dst, src)
// = incoming connections grouped by node), started from the outputs.
namespace asnn {
namespace {

__global__ void seed_outputs_kernel(const int32_t *__restrict__ output_ids, int32_t n_outputs, int32_t n_nodes,
                                    int32_t *required, int32_t *__restrict__ frontier, int *ctl) {
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    bool first = false;
    int32_t v = 0;
    if (k < n_outputs) {
        v = output_ids[k];
        if (v < 0 || v >= n_nodes) flag_error(ctl, ASNN_ERR_INDEX);
        else first = atomicExch(&required[v], 1) == 0;          // an id listed twice is seeded once
    }
    wave_append(first, v, frontier, &ctl[kCount0]);
}

__global__ __launch_bounds__(kThreads) void reach_sweep_kernel(int k, const int32_t *__restrict__ in_ptr,
                                                                const int32_t *__restrict__ in_src, int32_t *required,
                                                                const int32_t *__restrict__ frontier_in,
                                                                int32_t *__restrict__ frontier_out, int *ctl) {
    const int count = ctl[kCount0 + k % 3];
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        ctl[kCount0 + (k + 2) % 3] = 0;
        if (count > 0) atomicAdd(&ctl[kAssigned], count);
    }
    if (count == 0) return;
    int *count_out = &ctl[kCount0 + (k + 1) % 3];
    const int sub = threadIdx.x % kGroup;
    const int groups = gridDim.x * (kThreads / kGroup);
    // newly reached nodes are collected per workgroup and appended with one atomic (see sweep_kernel)
    __shared__ int32_t found[kFoundCap];
    __shared__ int n_found, found_base;
    if (threadIdx.x == 0) n_found = 0;
    __syncthreads();
    for (int f = blockIdx.x * (kThreads / kGroup) + threadIdx.x / kGroup; f < count; f += groups) {
        const int32_t v = frontier_in[f];
        const int32_t e1 = in_ptr[v + 1];
        for (int32_t e = in_ptr[v] + sub; e < e1; e += kGroup) {
            const int32_t a = in_src[e];
            if (atomicExch(&required[a], 1) == 0) {
                const int pos = atomicAdd(&n_found, 1);                  // LDS
                if (pos < kFoundCap) found[pos] = a;
                else frontier_out[atomicAdd(count_out, 1)] = a;
            }
        }
    }
    __syncthreads();
    const int n = min(n_found, kFoundCap);
    if (threadIdx.x == 0 && n > 0) found_base = atomicAdd(count_out, n);
    __syncthreads();
    for (int i = threadIdx.x; i < n; i += kThreads) frontier_out[found_base + i] = found[i];
}

__global__ void keep_flag_kernel(const int32_t *__restrict__ src, const int32_t *__restrict__ dst,
                                 const int32_t *__restrict__ required, int64_t n_edges, int32_t n_nodes,
                                 int32_t *__restrict__ keep, int *err) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e <= n_edges; e += stride) {
        if (e == n_edges) { keep[e] = 0; continue; }
        const int32_t a = src[e], b = dst[e];
        if (a < 0 || a >= n_nodes || b < 0 || b >= n_nodes) { atomicCAS(err, 0, ASNN_ERR_INDEX); keep[e] = 0; continue; }
        keep[e] = required[b] != 0 ? 1 : 0;
    }
}

__global__ void compact_edges_kernel(const int32_t *__restrict__ src, const int32_t *__restrict__ dst,
                                     const float *__restrict__ w, const int32_t *__restrict__ pos, int64_t n_edges,
                                     int32_t *__restrict__ src_out, int32_t *__restrict__ dst_out,
                                     float *__restrict__ w_out) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n_edges; e += stride) {
        const int32_t p = pos[e];
        if (pos[e + 1] != p) {          // kept: exclusive scan of the keep flags gives its slot
            src_out[p] = src[e];
            dst_out[p] = dst[e];
            w_out[p] = w[e];
        }
    }
}

// Compaction to the required set: nodes of R get the dense ids 0 .. |R|-1 in the order of their
// old ids (pos = exclusive prefix sum of the required flags), everything else gets -1.
__global__ void new_id_kernel(const int32_t *__restrict__ required, const int32_t *__restrict__ pos, int32_t n_nodes,
                              int32_t *__restrict__ new_id) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < n_nodes; v += stride)
        new_id[v] = required[v] != 0 ? pos[v] : -1;
}

__global__ void required_flag_kernel(const int32_t *__restrict__ required, int32_t n_nodes, int32_t *__restrict__ flag) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v <= n_nodes; v += stride)
        flag[v] = (v < n_nodes && required[v] != 0) ? 1 : 0;
}

// ids[k] -> new_id[ids[k]] (-1 for an id out of range or outside R)
__global__ void relabel_kernel(const int32_t *__restrict__ ids, int64_t n, const int32_t *__restrict__ new_id,
                               int32_t n_nodes, int32_t *__restrict__ out) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; k < n; k += stride) {
        const int32_t v = ids[k];
        out[k] = (v >= 0 && v < n_nodes) ? new_id[v] : -1;
    }
}

struct FilterWorkspace {
    int *err;
    int32_t *pos, *scan_tmp;
    size_t bytes;
};

FilterWorkspace carve_filter(void *ws, int64_t n_edges) {
    Carver c(ws);
    FilterWorkspace w;
    const size_t e = (size_t)n_edges;
    w.err = c.take<int>(64);
    w.pos = c.take<int32_t>(e + 2);
    w.scan_tmp = c.take<int32_t>(scan_tmp_ints(e + 1));
    w.bytes = c.off;
    return w;
}

}  // namespace
}  // namespace asnn

extern "C" size_t asnn_required_workspace_bytes(int32_t n_nodes, int64_t n_edges) {
    return asnn_levels_workspace_bytes(n_nodes, n_edges);
}

extern "C" int asnn_required_set(int32_t n_nodes, int64_t n_edges, const int32_t *src, const int32_t *dst,
                                 const int32_t *output_ids, int32_t n_outputs, int32_t *required_out,
                                 int32_t *n_required_out, void *workspace, size_t workspace_bytes, void *stream) {
    if (n_nodes <= 0 || n_edges < 0 || n_edges > (int64_t)ASNN_MAX_EDGES || n_outputs < 0) return ASNN_ERR_SIZE;
    if (!required_out || !n_required_out || !workspace) return ASNN_ERR_NULL;
    if ((n_edges > 0 && (!src || !dst)) || (n_outputs > 0 && !output_ids)) return ASNN_ERR_NULL;
    if (((uintptr_t)workspace & 255u) != 0 || workspace_bytes < asnn_required_workspace_bytes(n_nodes, n_edges))
        return ASNN_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    LevelsWorkspace w = carve_levels(workspace, n_nodes, n_edges);
    ASNN_HIP_TRY(hipMemsetAsync(required_out, 0, sizeof(int32_t) * (size_t)n_nodes, s));
    // transposed: the connections grouped by destination
    const int32_t *in_src = nullptr;
    ASNN_TRY(group_connections(w, n_nodes, n_edges, dst, src, false, s, &in_src));
    if (n_outputs > 0) {
        hipLaunchKernelGGL(seed_outputs_kernel, dim3(blocks_for((size_t)n_outputs, kThreads)), dim3(kThreads), 0, s,
                           output_ids, n_outputs, n_nodes, required_out, w.frontier_a, w.ctl);
        ASNN_HIP_TRY(hipGetLastError());
    }
    int host_ctl[kCtlInts];
    int k = 0;
    for (;;) {
        for (int i = 0; i < kSweepsPerSync; ++i, ++k) {
            const int32_t *fin = (k & 1) ? w.frontier_b : w.frontier_a;
            int32_t *fout = (k & 1) ? w.frontier_a : w.frontier_b;
            hipLaunchKernelGGL(reach_sweep_kernel, dim3(kReachBlocks), dim3(kThreads), 0, s, k,
                               (const int32_t *)w.out_ptr, in_src, required_out, fin, fout, w.ctl);
            ASNN_HIP_TRY(hipGetLastError());
        }
        ASNN_HIP_TRY(hipMemcpyAsync(host_ctl, w.ctl, sizeof(host_ctl), hipMemcpyDeviceToHost, s));
        ASNN_HIP_TRY(hipStreamSynchronize(s));
        if (host_ctl[kErr] != 0) return host_ctl[kErr];
        if (host_ctl[kCount0 + k % 3] == 0) break;
        if (k > n_nodes) break;          // every sweep with a non-empty frontier marks new nodes: at most n_nodes sweeps
    }
    *n_required_out = host_ctl[kAssigned];
    return ASNN_OK;
}

extern "C" size_t asnn_filter_workspace_bytes(int64_t n_edges) {
    if (n_edges < 0) return 0;
    return carve_filter(nullptr, n_edges).bytes;
}

extern "C" int asnn_filter_required(int32_t n_nodes, int64_t n_edges, const int32_t *src, const int32_t *dst,
                                    const float *w, const int32_t *required, int32_t *src_out, int32_t *dst_out,
                                    float *w_out, int64_t *n_kept_out, void *workspace, size_t workspace_bytes,
                                    void *stream) {
    if (n_nodes <= 0 || n_edges < 0 || n_edges > (int64_t)ASNN_MAX_EDGES) return ASNN_ERR_SIZE;
    if (!required || !n_kept_out || !workspace) return ASNN_ERR_NULL;
    if (n_edges > 0 && (!src || !dst || !w || !src_out || !dst_out || !w_out)) return ASNN_ERR_NULL;
    if (((uintptr_t)workspace & 255u) != 0 || workspace_bytes < asnn_filter_workspace_bytes(n_edges))
        return ASNN_ERR_WORKSPACE;
    if (n_edges == 0) { *n_kept_out = 0; return ASNN_OK; }
    hipStream_t s = static_cast<hipStream_t>(stream);
    FilterWorkspace ws = carve_filter(workspace, n_edges);
    ASNN_HIP_TRY(hipMemsetAsync(ws.err, 0, 256, s));
    const unsigned eb = blocks_for((size_t)n_edges + 1, kThreads, 65535);
    hipLaunchKernelGGL(keep_flag_kernel, dim3(eb), dim3(kThreads), 0, s, src, dst, required, n_edges, n_nodes, ws.pos,
                       ws.err);
    ASNN_HIP_TRY(hipGetLastError());
    ASNN_TRY(exclusive_scan_i32(ws.pos, ws.pos, (size_t)n_edges + 1, ws.scan_tmp, s));
    hipLaunchKernelGGL(compact_edges_kernel, dim3(eb), dim3(kThreads), 0, s, src, dst, w, (const int32_t *)ws.pos,
                       n_edges, src_out, dst_out, w_out);
    ASNN_HIP_TRY(hipGetLastError());
    int host_err = 0;
    int32_t kept = 0;
    ASNN_HIP_TRY(hipMemcpyAsync(&host_err, ws.err, sizeof(int), hipMemcpyDeviceToHost, s));
    ASNN_HIP_TRY(hipMemcpyAsync(&kept, ws.pos + n_edges, sizeof(int32_t), hipMemcpyDeviceToHost, s));
    ASNN_HIP_TRY(hipStreamSynchronize(s));
    *n_kept_out = kept;
    return host_err;
}

extern "C" size_t asnn_compact_workspace_bytes(int32_t n_nodes) {
    if (n_nodes < 0) return 0;
    return carve_filter(nullptr, (int64_t)n_nodes).bytes;
}

extern "C" int asnn_compact_required(int32_t n_nodes, const int32_t *required, int32_t *new_id_out,
                                     int32_t *n_required_out, void *workspace, size_t workspace_bytes, void *stream) {
    if (n_nodes <= 0) return ASNN_ERR_SIZE;
    if (!required || !new_id_out || !n_required_out || !workspace) return ASNN_ERR_NULL;
    if (((uintptr_t)workspace & 255u) != 0 || workspace_bytes < asnn_compact_workspace_bytes(n_nodes))
        return ASNN_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    FilterWorkspace ws = carve_filter(workspace, (int64_t)n_nodes);
    const unsigned nb = blocks_for((size_t)n_nodes + 1, kThreads, 65535);
    hipLaunchKernelGGL(required_flag_kernel, dim3(nb), dim3(kThreads), 0, s, required, n_nodes, ws.pos);
    ASNN_HIP_TRY(hipGetLastError());
    ASNN_TRY(exclusive_scan_i32(ws.pos, ws.pos, (size_t)n_nodes + 1, ws.scan_tmp, s));
    hipLaunchKernelGGL(new_id_kernel, dim3(nb), dim3(kThreads), 0, s, required, (const int32_t *)ws.pos, n_nodes, new_id_out);
    ASNN_HIP_TRY(hipGetLastError());
    int32_t count = 0;
    ASNN_HIP_TRY(hipMemcpyAsync(&count, ws.pos + n_nodes, sizeof(int32_t), hipMemcpyDeviceToHost, s));
    ASNN_HIP_TRY(hipStreamSynchronize(s));
    *n_required_out = count;
    return ASNN_OK;
}

extern "C" int asnn_relabel_ids(const int32_t *ids, int64_t n_ids, const int32_t *new_id, int32_t n_nodes,
                                int32_t *ids_out, void *stream) {
    if (n_ids < 0 || n_nodes <= 0) return ASNN_ERR_SIZE;
    if (n_ids == 0) return ASNN_OK;
    if (!ids || !new_id || !ids_out) return ASNN_ERR_NULL;
    hipLaunchKernelGGL(relabel_kernel, dim3(blocks_for((size_t)n_ids, kThreads, 65535)), dim3(kThreads), 0,
                       static_cast<hipStream_t>(stream), ids, n_ids, new_id, n_nodes, ids_out);
    ASNN_HIP_TRY(hipGetLastError());
    return ASNN_OK;
}
