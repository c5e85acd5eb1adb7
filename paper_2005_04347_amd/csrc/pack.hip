// asnn_pack_csr: level-contiguous, destination-sorted CSR.
//
// The paper keeps one record per node (id, layer, numInNodes, inNodes[],
// inWeights[]), sorts the record array by layer and keeps the node count of
// every layer.  The same information is laid out here as flat arrays: nodes
// renumbered so that a level is a contiguous range of rows ("packed rows"),
// one CSR over packed rows whose column indices are packed rows too, so the
// value matrix V[row][batch] is level-contiguous and a level launch touches
// only rows below its own range.
//
// Everything is built from two stable radix sorts (nodes by level key, edges
// by destination) and prefix sums, so the packed arrays are a
// deterministic function of the input: a node's connections keep their
// edge-list order; nodes are ordered by level, in-degree class, short-row
// flag, then original id.
#include "asnn_common.h"

namespace asnn {

namespace {

constexpr int kThreads = 256;

__device__ inline void flag_error(int *err, int code) { atomicCAS(err, 0, code); }

__global__ void indegree_kernel(const int32_t *__restrict__ src, const int32_t *__restrict__ dst,
                                const int32_t *__restrict__ level, int64_t n_edges, int32_t n_nodes, int32_t n_levels,
                                int32_t *indeg, int *err) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n_edges; e += stride) {
        const int32_t a = src[e], b = dst[e];
        if (a < 0 || a >= n_nodes || b < 0 || b >= n_nodes) { flag_error(err, ASNN_ERR_INDEX); continue; }
        const int32_t la = level[a], lb = level[b];
        if (la < 0 || la >= n_levels || lb < 0 || lb >= n_levels) { flag_error(err, ASNN_ERR_INDEX); continue; }
        if (la >= lb) flag_error(err, ASNN_ERR_LEVEL_ORDER);
        atomicAdd(&indeg[b], 1);
    }
}

// Rows of a level start in packed order, so a level should end with short rows: when its
// last rows are long ones the launch drains with most of the chip idle.  Inside the light
// class the rows with at most 3/4 of the mean in-degree (about a fifth of the rows for
// Poisson-like degrees, one fill of the chip) go last; everything else keeps the order of
// the original ids, which keeps the rows of one network of a population together.
// key = ((3*level + class) << 1) | short, class 0 heavy, 1 medium, 2 light.
constexpr int kRankBits = 1;

__global__ void node_key_kernel(const int32_t *__restrict__ level, const int32_t *__restrict__ indeg, int32_t n_nodes,
                                int32_t n_levels, int32_t mean_indegree, uint32_t *__restrict__ keys,
                                uint32_t *__restrict__ vals, int *err) {
    const int v = blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= n_nodes) return;
    int32_t l = level[v];
    if (l < 0 || l >= n_levels) { flag_error(err, ASNN_ERR_INDEX); l = 0; }
    const int32_t d = indeg[v];
    const uint32_t cls = d >= ASNN_HEAVY_INDEGREE ? 0u : (d >= ASNN_MEDIUM_INDEGREE ? 1u : 2u);
    const uint32_t is_short = (cls == 2u && 4 * (int64_t)d <= 3 * (int64_t)mean_indegree) ? 1u : 0u;
    keys[v] = (((uint32_t)ASNN_CLASSES * (uint32_t)l + cls) << kRankBits) | is_short;
    vals[v] = (uint32_t)v;
}

// perm = sorted node ids; inv_perm its inverse; packed_deg[i] = indeg[perm[i]].
__global__ void permutation_kernel(const uint32_t *__restrict__ sorted_ids, const int32_t *__restrict__ indeg,
                                   int32_t n_nodes, int32_t *__restrict__ perm, int32_t *__restrict__ inv_perm,
                                   int32_t *__restrict__ packed_deg) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i > n_nodes) return;
    if (i == n_nodes) { packed_deg[i] = 0; return; }
    const int32_t v = (int32_t)sorted_ids[i];
    perm[i] = v;
    inv_perm[v] = i;
    packed_deg[i] = indeg[v];
}

// level_ptr[k] = number of nodes whose (level, class) key is < k  (k = 0 .. 3*n_levels).
__global__ void level_ptr_kernel(const uint32_t *__restrict__ sorted_keys, int32_t n_nodes, int32_t n_keys,
                                 int32_t *__restrict__ level_ptr) {
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k > n_keys) return;
    int lo = 0, hi = n_nodes;
    while (lo < hi) {
        const int mid = lo + (hi - lo) / 2;
        if ((sorted_keys[mid] >> kRankBits) < (uint32_t)k) lo = mid + 1; else hi = mid;
    }
    level_ptr[k] = lo;
}

__global__ void edge_key_kernel(const int32_t *__restrict__ dst, const int32_t *__restrict__ inv_perm, int64_t n_edges,
                                int32_t n_nodes, uint32_t *__restrict__ keys, uint32_t *__restrict__ vals) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n_edges; e += stride) {
        const int32_t b = dst[e];
        keys[e] = (b >= 0 && b < n_nodes) ? (uint32_t)inv_perm[b] : 0u;
        vals[e] = (uint32_t)e;
    }
}

// Large networks: the connections are sorted by ORIGINAL destination before the packed order is
// known, which also yields the in-degrees (run lengths) without an atomic per connection; a
// node's run is then moved as a whole to its packed row.  Same checks as indegree_kernel; a
// connection with a bad id is filed under node 0 (the error is already flagged).
__global__ void edge_key_by_id_kernel(const int32_t *__restrict__ src, const int32_t *__restrict__ dst,
                                      const int32_t *__restrict__ level, int64_t n_edges, int32_t n_nodes,
                                      int32_t n_levels, uint32_t *__restrict__ keys, uint32_t *__restrict__ vals, int *err) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n_edges; e += stride) {
        const int32_t a = src[e];
        int32_t b = dst[e];
        if (a < 0 || a >= n_nodes || b < 0 || b >= n_nodes) {
            flag_error(err, ASNN_ERR_INDEX);
            b = 0;
        } else {
            const int32_t la = level[a], lb = level[b];
            if (la < 0 || la >= n_levels || lb < 0 || lb >= n_levels) flag_error(err, ASNN_ERR_INDEX);
            else if (la >= lb) flag_error(err, ASNN_ERR_LEVEL_ORDER);
        }
        keys[e] = (uint32_t)b;
        vals[e] = (uint32_t)e;
    }
}

// sorted position i (destination sorted_dst[i], i - first[destination] connections of the same
// node before it) -> packed position row_ptr[packed row of the destination] + that offset.
__global__ void place_edges_kernel(const uint32_t *__restrict__ sorted_dst, const uint32_t *__restrict__ sorted_edge,
                                   const int32_t *__restrict__ first, const int32_t *__restrict__ row_ptr,
                                   const int32_t *__restrict__ src, const float *__restrict__ w,
                                   const int32_t *__restrict__ inv_perm, int64_t n_edges, int32_t n_nodes,
                                   int32_t *__restrict__ col, float *__restrict__ w_packed) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_edges; i += stride) {
        const uint32_t b = sorted_dst[i], e = sorted_edge[i];
        const int64_t p = (int64_t)row_ptr[inv_perm[b]] + (i - first[b]);
        const int32_t a = src[e];
        col[p] = (a >= 0 && a < n_nodes) ? inv_perm[a] : 0;
        w_packed[p] = w[e];
    }
}

__global__ void gather_edges_kernel(const uint32_t *__restrict__ sorted_edge, const int32_t *__restrict__ src,
                                    const float *__restrict__ w, const int32_t *__restrict__ inv_perm, int64_t n_edges,
                                    int32_t n_nodes, int32_t *__restrict__ col, float *__restrict__ w_packed) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < n_edges; j += stride) {
        const uint32_t e = sorted_edge[j];
        const int32_t a = src[e];
        col[j] = (a >= 0 && a < n_nodes) ? inv_perm[a] : 0;
        w_packed[j] = w[e];
    }
}


// Work units, in packed order: a heavy row gives one unit per chunk of its connections (see
// heavy_chunks), medium rows go one or four to a unit (by how many the level has), light rows
// sixteen; a unit never spans two (level, class) segments.  row_units[i] = units that START at packed row i.
__global__ void row_units_kernel(const uint32_t *__restrict__ sorted_keys, const int32_t *__restrict__ level_ptr,
                                 const int32_t *__restrict__ packed_deg, int32_t n_nodes,
                                 int32_t *__restrict__ row_units, int32_t *__restrict__ max_indegree) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i > n_nodes) return;
    if (i == n_nodes) { row_units[i] = 0; return; }
    const int k = (int)(sorted_keys[i] >> kRankBits);
    const int cls = k % ASNN_CLASSES;
    const int off = i - level_ptr[k];
    int units;
    if (cls == 0) atomicMax(max_indegree, packed_deg[i]);      // lighter rows cannot hold the maximum if a heavy one exists
    if (cls == 0) units = heavy_chunks(packed_deg[i]);
    else if (cls == 1) {
        const int group = level_ptr[k + 1] - level_ptr[k] >= kMediumGroupFrom ? kMediumUnitRows : 1;
        units = (off % group == 0) ? 1 : 0;
    }
    else units = (off % kLightUnitRows == 0) ? 1 : 0;
    row_units[i] = units;
}

// unit_ptr[u] = first packed row of unit u (the chunks of one heavy row repeat it);
// unit_ptr[n_units] = n_nodes.  first_unit[i] = exclusive scan of row_units.
__global__ void unit_ptr_kernel(const int32_t *__restrict__ first_unit, int32_t n_nodes,
                                int32_t *__restrict__ unit_ptr) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i > n_nodes) return;
    if (i == n_nodes) { unit_ptr[first_unit[n_nodes]] = n_nodes; return; }
    for (int u = first_unit[i]; u < first_unit[i + 1]; ++u) unit_ptr[u] = i;
}

// out[0] = first unit above level 0, out[1] = number of units (out[2] holds the largest heavy in-degree).
__global__ void unit_counts_kernel(const int32_t *__restrict__ first_unit, const int32_t *__restrict__ level_ptr,
                                   int32_t n_nodes, int32_t *__restrict__ out) {
    out[0] = first_unit[level_ptr[ASNN_CLASSES]];
    out[1] = first_unit[n_nodes];
}

}  // namespace

struct PackWorkspace {
    int *err;
    int32_t *indeg, *packed_deg, *seg_units, *tmp, *first;
    uint32_t *keys_a, *vals_a, *keys_b, *vals_b;            // the edge sort (and, for small networks, the node sort before it)
    uint32_t *node_keys_a, *node_vals_a, *node_keys_b, *node_vals_b;     // large networks: the node sort has buffers of its own
    size_t bytes;
};

// Connections from which the edges are sorted before the packed order is known (below, the
// in-degree count with one atomic per connection is cheaper than the bookkeeping).
constexpr int64_t kSortFirstEdges = 1 << 21;

static PackWorkspace carve_pack(void *ws, int32_t n_nodes, int64_t n_edges) {
    Carver c(ws);
    PackWorkspace w;
    const size_t n = (size_t)n_nodes, e = (size_t)n_edges;
    const size_t m = (n > e ? n : e) + 1;
    w.err = c.take<int>(64);
    w.indeg = c.take<int32_t>(n + 1);
    w.packed_deg = c.take<int32_t>(n + 1);
    w.seg_units = c.take<int32_t>((size_t)ASNN_CLASSES * n + 2);     // n_levels <= n_nodes
    w.keys_a = c.take<uint32_t>(m);
    w.vals_a = c.take<uint32_t>(m);
    w.keys_b = c.take<uint32_t>(m);
    w.vals_b = c.take<uint32_t>(m);
    const size_t own = n_edges >= kSortFirstEdges ? n + 1 : 0;
    w.node_keys_a = c.take<uint32_t>(own);
    w.node_vals_a = c.take<uint32_t>(own);
    w.node_keys_b = c.take<uint32_t>(own);
    w.node_vals_b = c.take<uint32_t>(own);
    w.first = c.take<int32_t>(own);
    const size_t t1 = radix_tmp_ints(m), t2 = scan_tmp_ints(n + 1);
    w.tmp = c.take<int32_t>(t1 > t2 ? t1 : t2);
    w.bytes = c.off;
    return w;
}

}  // namespace asnn

using namespace asnn;

extern "C" size_t asnn_pack_workspace_bytes(int32_t n_nodes, int64_t n_edges) {
    if (n_nodes < 0 || n_edges < 0) return 0;
    return carve_pack(nullptr, n_nodes, n_edges).bytes;
}

extern "C" int asnn_pack_csr(const int32_t *src, const int32_t *dst, const float *w, const int32_t *level,
                             asnn_packed *packed, void *workspace, size_t workspace_bytes, void *stream) {
    if (!packed) return ASNN_ERR_NULL;
    const int32_t n_nodes = packed->n_nodes, n_levels = packed->n_levels;
    const int64_t n_edges = packed->n_edges;
    int32_t *level_ptr = packed->level_ptr, *level_ptr_host = packed->level_ptr_host, *perm = packed->perm,
            *inv_perm = packed->inv_perm, *row_ptr = packed->row_ptr, *col = packed->col, *unit_ptr = packed->unit_ptr;
    float *w_packed = packed->w;
    if (n_nodes <= 0 || n_edges < 0 || n_edges > (int64_t)ASNN_MAX_EDGES || n_levels <= 0 ||
        n_levels > n_nodes || n_levels >= (1 << 28))
        return ASNN_ERR_SIZE;
    if (!level || !level_ptr || !level_ptr_host || !perm || !inv_perm || !row_ptr || !unit_ptr || !workspace)
        return ASNN_ERR_NULL;
    if (n_edges > 0 && (!src || !dst || !w || !col || !w_packed)) return ASNN_ERR_NULL;
    if (((uintptr_t)workspace & 255u) != 0 || workspace_bytes < asnn_pack_workspace_bytes(n_nodes, n_edges))
        return ASNN_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    PackWorkspace ws = carve_pack(workspace, n_nodes, n_edges);
    const size_t n = (size_t)n_nodes;
    const int32_t n_keys = ASNN_CLASSES * n_levels;

    ASNN_HIP_TRY(hipMemsetAsync(ws.err, 0, (size_t)((char *)ws.packed_deg - (char *)ws.err), s));   // err + indeg
    const bool sort_first = n_edges >= kSortFirstEdges;
    const unsigned eb = blocks_for((size_t)(n_edges > 0 ? n_edges : 1), kThreads, 65535);
    uint32_t *edge_keys = nullptr, *edge_ids = nullptr;      // sort_first: connections sorted by original destination
    if (sort_first) {
        hipLaunchKernelGGL(edge_key_by_id_kernel, dim3(eb), dim3(kThreads), 0, s, src, dst, level, n_edges, n_nodes,
                           n_levels, ws.keys_a, ws.vals_a, ws.err);
        ASNN_HIP_TRY(hipGetLastError());
        ASNN_TRY(radix_sort_pairs_u32(ws.keys_a, ws.vals_a, ws.keys_b, ws.vals_b, (size_t)n_edges,
                                      bits_for((uint64_t)n_nodes - 1), ws.tmp, s, &edge_keys, &edge_ids));
        ASNN_TRY(sorted_run_lengths(edge_keys, (size_t)n_edges, ws.first, ws.indeg, s));
    } else if (n_edges > 0) {
        hipLaunchKernelGGL(indegree_kernel, dim3(eb), dim3(kThreads), 0, s, src, dst, level, n_edges, n_nodes, n_levels,
                           ws.indeg, ws.err);
        ASNN_HIP_TRY(hipGetLastError());
    }
    // nodes: stable sort by (level, in-degree class) key
    uint32_t *nka = sort_first ? ws.node_keys_a : ws.keys_a, *nva = sort_first ? ws.node_vals_a : ws.vals_a;
    uint32_t *nkb = sort_first ? ws.node_keys_b : ws.keys_b, *nvb = sort_first ? ws.node_vals_b : ws.vals_b;
    hipLaunchKernelGGL(node_key_kernel, dim3(blocks_for(n, kThreads)), dim3(kThreads), 0, s, level,
                       (const int32_t *)ws.indeg, n_nodes, n_levels, (int32_t)(n_edges / n_nodes), nka, nva, ws.err);
    ASNN_HIP_TRY(hipGetLastError());
    uint32_t *ks, *vs;
    ASNN_TRY(radix_sort_pairs_u32(nka, nva, nkb, nvb, n, bits_for((uint64_t)n_keys << kRankBits), ws.tmp, s, &ks, &vs));
    hipLaunchKernelGGL(permutation_kernel, dim3(blocks_for(n + 1, kThreads)), dim3(kThreads), 0, s,
                       (const uint32_t *)vs, (const int32_t *)ws.indeg, n_nodes, perm, inv_perm, ws.packed_deg);
    ASNN_HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(level_ptr_kernel, dim3(blocks_for((size_t)n_keys + 1, kThreads)), dim3(kThreads), 0, s,
                       (const uint32_t *)ks, n_nodes, n_keys, level_ptr);
    ASNN_HIP_TRY(hipGetLastError());
    ASNN_TRY(exclusive_scan_i32(ws.packed_deg, row_ptr, n + 1, ws.tmp, s));
    // work units (uses the sorted node keys, so before the edge sort recycles the buffers)
    hipLaunchKernelGGL(row_units_kernel, dim3(blocks_for(n + 1, kThreads)), dim3(kThreads), 0, s, (const uint32_t *)ks,
                       (const int32_t *)level_ptr, (const int32_t *)ws.packed_deg, n_nodes, ws.seg_units, ws.err + 4);
    ASNN_HIP_TRY(hipGetLastError());
    ASNN_TRY(exclusive_scan_i32(ws.seg_units, ws.seg_units, n + 1, ws.tmp, s));
    hipLaunchKernelGGL(unit_ptr_kernel, dim3(blocks_for(n + 1, kThreads)), dim3(kThreads), 0, s,
                       (const int32_t *)ws.seg_units, n_nodes, unit_ptr);
    ASNN_HIP_TRY(hipGetLastError());
    int32_t host_units[3] = {0, 0, 0};   // {first unit above level 0, number of units, largest heavy in-degree}
    hipLaunchKernelGGL(unit_counts_kernel, dim3(1), dim3(1), 0, s, (const int32_t *)ws.seg_units,
                       (const int32_t *)level_ptr, n_nodes, ws.err + 2);
    ASNN_HIP_TRY(hipGetLastError());
    ASNN_HIP_TRY(hipMemcpyAsync(host_units, ws.err + 2, 3 * sizeof(int32_t), hipMemcpyDeviceToHost, s));

    // edges: stable sort by packed destination keeps each node's edge-list order
    if (sort_first) {
        hipLaunchKernelGGL(place_edges_kernel, dim3(eb), dim3(kThreads), 0, s, (const uint32_t *)edge_keys,
                           (const uint32_t *)edge_ids, (const int32_t *)ws.first, (const int32_t *)row_ptr, src, w,
                           (const int32_t *)inv_perm, n_edges, n_nodes, col, w_packed);
        ASNN_HIP_TRY(hipGetLastError());
    } else if (n_edges > 0) {
        hipLaunchKernelGGL(edge_key_kernel, dim3(eb), dim3(kThreads), 0, s, dst, (const int32_t *)inv_perm, n_edges,
                           n_nodes, ws.keys_a, ws.vals_a);
        ASNN_HIP_TRY(hipGetLastError());
        ASNN_TRY(radix_sort_pairs_u32(ws.keys_a, ws.vals_a, ws.keys_b, ws.vals_b, (size_t)n_edges,
                                      bits_for((uint64_t)n_nodes - 1), ws.tmp, s, &ks, &vs));
        hipLaunchKernelGGL(gather_edges_kernel, dim3(eb), dim3(kThreads), 0, s, (const uint32_t *)vs, src, w,
                           (const int32_t *)inv_perm, n_edges, n_nodes, col, w_packed);
        ASNN_HIP_TRY(hipGetLastError());
    }
    int host_err = 0;
    ASNN_HIP_TRY(hipMemcpyAsync(&host_err, ws.err, sizeof(int), hipMemcpyDeviceToHost, s));
    ASNN_HIP_TRY(hipMemcpyAsync(level_ptr_host, level_ptr, sizeof(int32_t) * ((size_t)n_keys + 1),
                                hipMemcpyDeviceToHost, s));
    ASNN_HIP_TRY(hipStreamSynchronize(s));
    packed->first_unit = host_units[0];
    packed->n_units = host_units[1];
    packed->max_heavy_indegree = host_units[2];
    return host_err;
}
