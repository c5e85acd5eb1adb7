/*
 * libasnn -- full forward activation of arbitrary-structure sparse neural
 * networks (ASNNs) on one AMD MI355X (gfx950).  C ABI.
 *
 * An ASNN is a directed acyclic graph: N nodes, E weighted connections
 * (src[e] -> dst[e], w[e]), a set of input ("sensor") nodes.  The library
 *   1. assigns every node its dependency layer ("level"): the paper's
 *      network segmentation (Sec. "Sequential activation", segmentation
 *      algorithm) -- a node enters the next layer once its entire input set is
 *      assigned, i.e. level = longest path from any node without incoming
 *      connections; the input layer is level 0 (Sec. "Parallel GPU activation");
 *   2. packs the network into a destination-sorted CSR whose nodes are ordered
 *      by level (the paper sorts its node array by layer number and keeps the
 *      per-layer node counts NNL, Sec. "Parallel GPU activation");
 *   3. activates the network level by level for a batch of B input vectors:
 *      sensors output sigmoid(x), every other node outputs
 *      sigmoid(sum_i w_i * value(in_i)) with sigmoid(x) = 1/(1+e^(-4.97 x))
 *      (Introduction, display equation; activation kernel listing).  A node
 *      with no incoming connection that is no sensor outputs sigmoid(0) = 0.5.
 *
 * Conventions
 *   - "device" pointers are HIP device memory on the current device; "host"
 *     pointers are ordinary host memory.  The library never takes ownership of
 *     a caller's buffer and never returns memory the caller must free.
 *   - stream is a hipStream_t passed as void* (NULL = the default stream).
 *     asnn_build_levels and asnn_pack_csr synchronise that stream before they
 *     return (they hand scalars / small arrays back to the host).
 *     asnn_activate only enqueues work and returns.
 *   - every function returns ASNN_OK (0) or a negative ASNN_ERR_* code; nothing
 *     is printed, thrown or aborted.  asnn_last_hip_error() holds the hipError_t
 *     behind the most recent ASNN_ERR_HIP on the calling thread.
 *   - parallel connections (a,b) are legal and their contributions add; a self
 *     loop is a cycle; node ids need not be in topological order.
 *   - batch layout is node-major with the batch contiguous: X[k*B + b],
 *     V[i*B + b], Y[o*B + b].
 *
 * Shape of the boundary.  The three calls take the paper's problem statement
 * (connections, inputs, outputs; layers; activation of the sorted node array)
 * in this form:
 *   - the packed network travels as ONE record (asnn_packed: sizes plus the
 *     caller-allocated arrays) from asnn_pack_csr to asnn_activate, not as a
 *     list of a dozen array arguments repeated in both signatures;
 *   - a population of networks is passed as their disjoint union: the caller
 *     offsets the node ids of network k by the number of nodes before it and
 *     concatenates the connection lists, input ids, output ids and the rows
 *     of X.  No per-network offset arrays cross the boundary: levels, packing
 *     and activation of a union are those of its components;
 *   - the default arithmetic is the one that meets the parity bar on every
 *     workload (fp64 sums and sigmoid, one rounding to float);
 *     ASNN_FLAG_ACC_F32 selects float arithmetic, not the other way round;
 *   - results restricted to the required set R are obtained by filtering (and,
 *     for a value matrix of |R| rows, compacting) the network beforehand
 *     (asnn_required_set / asnn_filter_required / asnn_compact_required) rather
 *     than by a flag of asnn_activate;
 *   - the library keeps no cache of graphs or launches between calls, so there
 *     is nothing to clear: every buffer, workspaces included, is the caller's.
 */
#ifndef ASNN_H
#define ASNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ASNN_OK 0
#define ASNN_ERR_NULL (-1)               /* a required pointer is NULL */
#define ASNN_ERR_SIZE (-2)               /* negative / zero / too large size argument */
#define ASNN_ERR_INDEX (-3)              /* src, dst, input or level value out of range */
#define ASNN_ERR_INPUT_HAS_INEDGE (-4)   /* a connection ends in an input node */
#define ASNN_ERR_DUP_INPUT (-5)          /* an input id is listed twice */
#define ASNN_ERR_CYCLE (-6)              /* the connections contain a cycle */
#define ASNN_ERR_WORKSPACE (-7)          /* workspace too small or misaligned */
#define ASNN_ERR_HIP (-8)                /* a HIP runtime call failed */
#define ASNN_ERR_LEVEL_ORDER (-9)        /* level[] is not increasing along a connection */
#define ASNN_ERR_NO_DEVICE (-10)         /* no HIP device available */
#define ASNN_ERR_TIMEOUT (-11)           /* a dataflow wait exceeded its time limit */
#define ASNN_ERR_SCRATCH (-12)           /* asnn_activate_static: the network and batch need more scratch than it holds */

/* asnn_activate flags */
#define ASNN_FLAG_RAW_INPUTS 1u  /* store sensor inputs unsquashed (the paper squashes them) */
#define ASNN_FLAG_ACC_F32 2u     /* accumulate and squash in fp32 (default: fp64 accumulate and
                                    fp64 sigmoid, rounded once to fp32 on store) */
#define ASNN_FLAG_LEVEL_LAUNCHES 4u  /* force one launch per level */
#define ASNN_FLAG_DATAFLOW 8u        /* force the persistent dataflow launch (needs the workspace) */
#define ASNN_FLAG_WORKGROUP 16u      /* force one workgroup per tile of batch columns */

/* In-degree classes.  Inside a level the packed order lists the heavy nodes
 * (in-degree >= ASNN_HEAVY_INDEGREE) first, then the medium ones
 * (>= ASNN_MEDIUM_INDEGREE), then the light ones (see asnn_pack_csr): the
 * activation gives a heavy row 16 wavefronts (and, in the dataflow schedule,
 * several workgroups), a medium row 4, 8 or 16, a light row 1 (a lane group of
 * it, or a team of 16 lanes, in the workgroup schedule). */
#define ASNN_HEAVY_INDEGREE 256
#define ASNN_MEDIUM_INDEGREE 32
#define ASNN_CLASSES 3

/* Largest connection count any call takes (32-bit positions, with headroom for
 * the kernels' look-ahead past a position): 2^31 - 65536.  More: ASNN_ERR_SIZE. */
#define ASNN_MAX_EDGES 2147418112LL

const char *asnn_strerror(int code);
int asnn_last_hip_error(void);
int asnn_version(void);

/* ---- 1. levels ---------------------------------------------------------
 * Segmentation into dependency layers (segmentation algorithm; reading: every
 * node without incoming connections is in layer 0, sensor or not).
 *   src, dst     device int32[n_edges]   connection e goes src[e] -> dst[e]
 *   input_ids    device int32[n_inputs]  the sensor nodes (may be NULL if n_inputs == 0)
 *   level_out    device int32[n_nodes]   receives the level of every node
 *   n_levels_out host   int32*           receives max level + 1 (0 if n_nodes == 0)
 *   workspace    device, >= asnn_levels_workspace_bytes(), 256-byte aligned
 * Errors: NULL, SIZE (n_nodes < 0, n_edges < 0 or > ASNN_MAX_EDGES), INDEX,
 * INPUT_HAS_INEDGE, DUP_INPUT, CYCLE (level_out is then unspecified),
 * WORKSPACE, HIP.  Blocks until the result is known. */
size_t asnn_levels_workspace_bytes(int32_t n_nodes, int64_t n_edges);
int asnn_build_levels(int32_t n_nodes, int64_t n_edges,
                      const int32_t *src, const int32_t *dst,
                      const int32_t *input_ids, int32_t n_inputs,
                      int32_t *level_out, int32_t *n_levels_out,
                      void *workspace, size_t workspace_bytes, void *stream);

/* ---- 1b. required set (optional) -----------------------------------------
 * The segmentation algorithm only layers "required" nodes: those needed to
 * compute the outputs (its argument R).  asnn_required_set marks every node
 * from which an output can be reached (outputs included); asnn_filter_required
 * drops the connections that end in a node outside R, keeping the order of the
 * others.  Running asnn_build_levels / asnn_pack_csr / asnn_activate on the
 * kept connections (same n_nodes) gives bit-identical activations for every
 * node of R; nodes outside R become isolated level-0 rows whose value is not
 * meaningful, and no connection work is spent on them.
 *   output_ids     device int32[n_outputs]
 *   required_out   device int32[n_nodes]   1 = in R, 0 = not
 *   n_required_out host   int32*           |R|
 *   src_out, dst_out, w_out  device, n_edges entries each (n_kept_out of them used)
 *   n_kept_out     host   int64*
 *   workspaces     device, >= the matching *_workspace_bytes(), 256-byte aligned
 * Errors: NULL, SIZE, INDEX, WORKSPACE, HIP.  Both block until the host values are known. */
size_t asnn_required_workspace_bytes(int32_t n_nodes, int64_t n_edges);
int asnn_required_set(int32_t n_nodes, int64_t n_edges, const int32_t *src, const int32_t *dst,
                      const int32_t *output_ids, int32_t n_outputs,
                      int32_t *required_out, int32_t *n_required_out,
                      void *workspace, size_t workspace_bytes, void *stream);
size_t asnn_filter_workspace_bytes(int64_t n_edges);
int asnn_filter_required(int32_t n_nodes, int64_t n_edges, const int32_t *src, const int32_t *dst, const float *w,
                         const int32_t *required,
                         int32_t *src_out, int32_t *dst_out, float *w_out, int64_t *n_kept_out,
                         void *workspace, size_t workspace_bytes, void *stream);

/* ---- 1c. outputs-only networks (optional) -----------------------------------
 * After asnn_required_set / asnn_filter_required the nodes outside R still
 * occupy rows of the value matrix.  asnn_compact_required numbers the nodes of
 * R densely (0 .. |R|-1, in the order of their old ids) and asnn_relabel_ids
 * carries id lists over to that numbering, so that the network can be built,
 * packed and activated on |R| nodes: nothing outside R is allocated, written
 * or read, and V is |R| x B.  A connection kept by asnn_filter_required has
 * both ends in R.  An id outside R (a sensor no output depends on) becomes -1,
 * which asnn_activate skips, so X keeps its rows.
 *   required     device int32[n_nodes]   from asnn_required_set
 *   new_id_out   device int32[n_nodes]   dense id, or -1 outside R
 *   n_required_out host int32*           |R|
 *   workspace    device, >= asnn_compact_workspace_bytes(n_nodes), 256-byte aligned
 *   ids, ids_out device int32[n_ids]     (asnn_relabel_ids; may be the same array;
 *                ids outside [0,n_nodes) become -1)
 * Errors: NULL, SIZE, WORKSPACE, HIP.  asnn_compact_required blocks until the
 * count is known; asnn_relabel_ids is asynchronous. */
size_t asnn_compact_workspace_bytes(int32_t n_nodes);
int asnn_compact_required(int32_t n_nodes, const int32_t *required, int32_t *new_id_out,
                          int32_t *n_required_out, void *workspace, size_t workspace_bytes, void *stream);
int asnn_relabel_ids(const int32_t *ids, int64_t n_ids, const int32_t *new_id, int32_t n_nodes,
                     int32_t *ids_out, void *stream);

/* ---- 2. pack -----------------------------------------------------------
 * Level-contiguous, destination-sorted CSR (replaces the paper's per-node
 * record with its inNodes / inWeights arrays and the array sorted by layer).
 * Packed order: by level; inside a level by in-degree class (heavy, medium,
 * light); inside the light class the short rows (in-degree d with
 * 4*d <= 3*floor(n_edges/n_nodes)) come last, so that a level does not end on
 * long rows; ties by original id.  The connections of one node keep their
 * edge-list order.
 *
 * The packed network is described by an asnn_packed record.  The CALLER
 * allocates every array it points to and fills the pointers (and n_nodes,
 * n_edges, n_levels) before asnn_pack_csr; the call fills the arrays and the
 * remaining scalars.  The record is plain data: the caller may copy it. */
typedef struct asnn_packed {
    int32_t n_nodes;
    int32_t n_levels;
    int64_t n_edges;
    int32_t n_units;            /* out: number of work units (see unit_ptr) */
    int32_t first_unit;         /* out: first unit above level 0 */
    int32_t max_heavy_indegree; /* out: largest in-degree among the heavy nodes (0 if there is none) */
    int32_t reserved;           /* keeps the pointers 8-byte aligned; not used */
    int32_t *level_ptr_host;    /* host   int32[3*n_levels+1]: copy of level_ptr for the host */
    int32_t *level_ptr;         /* device int32[3*n_levels+1]: level l holds packed rows
                                   [level_ptr[3l], level_ptr[3l+1]) heavy, [.. 3l+1, 3l+2) medium, [.. 3l+2, 3l+3) light */
    int32_t *perm;              /* device int32[n_nodes]   packed row -> original id */
    int32_t *inv_perm;          /* device int32[n_nodes]   original id -> packed row */
    int32_t *row_ptr;           /* device int32[n_nodes+1] connections of packed row i are [row_ptr[i], row_ptr[i+1]) */
    int32_t *col;               /* device int32[n_edges]   packed row of the connection's source */
    float *w;                   /* device float[n_edges] */
    int32_t *unit_ptr;          /* device int32[n_nodes + n_edges/512 + 2] (n_units+1 used).  Work units in
                                   packed order, each inside one level and class: up to 16 light rows,
                                   one medium row (up to 4 in a level that has 256 or more of
                                   them), or one heavy row or one chunk of it.  A heavy row
                                   of in-degree d is cut into ceil(d/len) chunks of
                                   len = max(512, ceil(d/16)) connections, one unit per chunk.
                                   unit_ptr[u] = first packed row of unit u (the chunks of one row
                                   repeat it), unit_ptr[n_units] = n_nodes */
} asnn_packed;

/*   src, dst, w  device            the connections, as for asnn_build_levels
 *   level        device int32[n_nodes]  from asnn_build_levels
 *   packed       host record, see above
 *   workspace    device, >= asnn_pack_workspace_bytes(), 256-byte aligned
 * Errors: NULL, SIZE, INDEX (level outside [0,n_levels), id out of range),
 * LEVEL_ORDER, WORKSPACE, HIP.  Blocks until the host fields are filled. */
size_t asnn_pack_workspace_bytes(int32_t n_nodes, int64_t n_edges);
int asnn_pack_csr(const int32_t *src, const int32_t *dst, const float *w, const int32_t *level,
                  asnn_packed *packed, void *workspace, size_t workspace_bytes, void *stream);

/* ---- 3. activate -------------------------------------------------------
 * Full activation of the packed network (or of a packed disjoint union of
 * networks: a population is activated by one call) for B input vectors
 * (activation kernel listing).  Three schedules compute the same bits:
 *   - level launches: one launch per level on the stream; the boundary
 *     between two launches is the paper's layer barrier;
 *   - dataflow: one persistent launch; workgroups claim work units in packed
 *     order and a row waits only for its own source rows (the value itself is
 *     the ready flag), so a deep, narrow network is not paced by a barrier
 *     per layer (the paper names grid-wide synchronisation as future work).
 *     The chunks of a heavy row are gathered by different workgroups; their
 *     partial sums meet in the workspace and are added in chunk order.  A
 *     small launch ahead of it stages the sensors and marks every other row
 *     as not written; the copy to Y is done by the last work items of the
 *     persistent launch itself.  Needs the workspace;
 *   - workgroup: the shape of the paper's kernel, one workgroup walks all
 *     levels with a workgroup barrier between two levels; batch columns are
 *     independent, so there is one such workgroup per tile of up to 64
 *     columns and nothing is exchanged between workgroups.  Sensor staging
 *     and the copy to Y happen in the same launch: an activation is one
 *     launch.  Meant for small networks and narrow batches (the paper's own
 *     regime: one input vector, thousands of connections), where launches
 *     and level hand-overs cost more than the connections.
 * By default: the workgroup schedule up to n_edges = 13000 + 1500*n_levels at B = 1
 * (less for wider batches: about 2800 + 130*n_levels at B = 16, 700 + 45*n_levels
 * at B = 64); else the dataflow schedule when a workspace is given and the levels
 * are small (up to about 20 M connections*samples per level; more when the network
 * has rows with thousands of connections, which a level launch has to wait for; less
 * when the value matrix fits the L2 caches or when a level is many work units with
 * little in each); else level launches.  ASNN_FLAG_LEVEL_LAUNCHES / ASNN_FLAG_DATAFLOW /
 * ASNN_FLAG_WORKGROUP force one (more than one of them: SIZE).
 *   packed      host record filled by asnn_pack_csr
 *   input_ids   device int32[n_inputs]  original ids; X row k feeds input_ids[k]
 *               (the ids given to asnn_build_levels)
 *   output_ids  device int32[n_outputs] original ids (may be NULL if Y is NULL)
 *   X           device float[n_inputs*B].  X and Y are only read and written by kernels
 *               (plain loads and stores, each element once), so pinned host memory
 *               that the device can address serves as well: a caller whose inputs
 *               arrive on the host and whose outputs are wanted there saves both
 *               copies (at one input vector an activation with the two copies takes
 *               about 45 us, with X and Y in pinned memory about half of that)
 *   V           device float[n_nodes*B]  receives the activation of EVERY node, packed
 *               row order (row i = node perm[i]); 16-byte aligned
 *   Y           device float[n_outputs*B] or NULL; receives the rows of output_ids
 *   workspace   device, >= asnn_activate_workspace_bytes(packed, B), 256-byte aligned,
 *               or NULL (no dataflow schedule then).  256 bytes, plus
 *               n_edges*B/32 bytes (B rounded up to whole tiles) when a node has more
 *               than 512 connections.  Contents need not be preserved between calls;
 *               activations that may overlap in time (different streams) need a
 *               workspace each.
 * Ids outside [0,n_nodes) in input_ids / output_ids are skipped (an output row
 * of such an id is filled with NaN).  Errors: NULL, SIZE, WORKSPACE, HIP.
 * Asynchronous.  A dataflow wait that exceeds its time limit (2 s of device
 * wall clock; it cannot with a valid packed record on a device that runs the
 * launch without interruption) stops waiting and raises a flag in the
 * workspace: rows computed from unwritten sources are NaN, the output rows
 * copied to Y after the flag was raised are NaN, and asnn_activate_status
 * reports ASNN_ERR_TIMEOUT.  A caller that cannot rule such a wait out (a
 * device shared with other processes) treats a dataflow result as valid only
 * once asnn_activate_status has returned ASNN_OK. */
size_t asnn_activate_workspace_bytes(const asnn_packed *packed, int32_t B);
/* Which schedule asnn_activate takes for this record, batch width, workspace
 * (given or not) and flags: 0 = one launch per level, 1 = dataflow, 2 = one
 * workgroup per tile, < 0 = the error asnn_activate would return for this
 * choice.  Launches nothing. */
int asnn_activate_schedule(const asnn_packed *packed, int32_t B, int has_workspace, uint32_t flags);
int asnn_activate(const asnn_packed *packed,
                  const int32_t *input_ids, int32_t n_inputs,
                  const int32_t *output_ids, int32_t n_outputs,
                  const float *X, int32_t B, float *V, float *Y,
                  void *workspace, size_t workspace_bytes,
                  uint32_t flags, void *stream);
/* Synchronises the stream and returns ASNN_OK, or ASNN_ERR_TIMEOUT if the last
 * dataflow activation that used this workspace gave up a wait.  NULL workspace: ASNN_OK. */
int asnn_activate_status(const void *workspace, void *stream);

/* ---- 3b. activate without any allocation ------------------------------------
 * For callers that cannot allocate device memory or carry a workspace around:
 * code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  asnn_activate_static is asnn_activate (same arguments, same
 * schedules, same kernels, same bits) with the workspace taken from a
 * file-scope device array of ASNN_STATIC_SCRATCH_BYTES inside the library, one
 * copy per device, which that device holds from the moment the library's code
 * is loaded on it until the process ends.  The call itself allocates and frees
 * nothing and calls no allocating routine; the caller still passes X, V and Y.
 *   - A network and batch width whose asnn_activate_workspace_bytes() exceeds
 *     ASNN_STATIC_SCRATCH_BYTES is refused with ASNN_ERR_SCRATCH, whatever
 *     schedule would have been taken (only networks with rows of more than 512
 *     connections need more than 512 bytes: n_edges*B/32 bytes, B rounded up
 *     to whole tiles).  Nothing is launched then.
 *   - Every call on a device shares that device's array, which still holds the
 *     previous call's contents; the call resets what it uses.  Two calls that
 *     may overlap in time on one device (different streams, different host
 *     threads) race on it: such callers serialise them or use asnn_activate
 *     with a workspace each.
 *   - asnn_activate_status(ASNN_STATIC_SCRATCH, stream) reports an abandoned
 *     dataflow wait of the last such call on the current device.
 * Errors: those of asnn_activate, plus SCRATCH.  Asynchronous. */
#define ASNN_STATIC_SCRATCH_BYTES (32u << 20)
#define ASNN_STATIC_SCRATCH ((const void *)(uintptr_t)1)
int asnn_activate_static(const asnn_packed *packed,
                         const int32_t *input_ids, int32_t n_inputs,
                         const int32_t *output_ids, int32_t n_outputs,
                         const float *X, int32_t B, float *V, float *Y,
                         uint32_t flags, void *stream);

/* ---- yardsticks ----------------------------------------------------------
 * Not part of the method: kernels of known traffic without the method's
 * arithmetic, which the benchmark times beside the activation.  All
 * asynchronous; errors: NULL, SIZE, HIP.
 *
 * asnn_device_copy: plain streaming device-to-device copy of `bytes` bytes (a
 * multiple of 16, both pointers 16-byte aligned, buffers must not overlap):
 * reads `bytes`, writes `bytes`.  Also the kernel of known traffic against
 * which hardware byte counters are calibrated.
 *
 * asnn_device_read: plain streaming read of `bytes` bytes (a multiple of 16,
 * 16-byte aligned); sink is a device float the kernel may write (it does not,
 * for ordinary data).
 *
 * asnn_device_gather: random row gather in the launch shape of one level of
 * the activation over a matrix buf[n_rows][row_floats] (row_floats a multiple
 * of 64): one single-wavefront workgroup per (row, tile of 128 columns -- 64
 * when row_floats is no multiple of 128), rows_per_launch rows, each
 * wavefront loading its tile of `gathers` pseudo-random rows of buf (seeded;
 * all tiles of a row pick the same rows).  Reads
 * rows_per_launch * gathers * row_floats * 4 bytes, writes nothing.
 *
 * asnn_device_gather_store: the same gather, and every wavefront stores its
 * tile of one row of out[rows_per_launch][row_floats] (8-byte aligned, must
 * not overlap buf), as a level of the activation stores the rows it
 * computes: reads the same bytes and writes rows_per_launch * row_floats * 4.
 * Every element of a stored row is the sum of the `gathers` elements of its
 * column that were loaded. */
int asnn_device_copy(void *dst, const void *src, size_t bytes, void *stream);
int asnn_device_read(const void *src, size_t bytes, float *sink, void *stream);
int asnn_device_gather(const float *buf, int32_t n_rows, int32_t row_floats, int32_t rows_per_launch,
                       int32_t gathers, uint32_t seed, float *sink, void *stream);
int asnn_device_gather_store(const float *buf, int32_t n_rows, int32_t row_floats, int32_t rows_per_launch,
                             int32_t gathers, uint32_t seed, float *out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* ASNN_H */
