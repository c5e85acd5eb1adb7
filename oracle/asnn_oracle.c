/*
 * Sequential CPU oracle for full activation of an arbitrary-structure sparse
 * neural network (ASNN).  TEST INFRASTRUCTURE ONLY: tests, the smoke check and
 * the benchmark's cpu_baseline leg may call it; the GPU library never does,
 * and the two share no code.
 *
 * What it computes is the plain definition the paper's method reaches:
 *
 *   level(v) = 0                                  if v has no incoming edge
 *            = 1 + max over edges (u,v) level(u)  otherwise
 *     (Network segmentation algorithm, Sec. "Sequential activation": a node
 *      joins the next layer only when its entire input set is already
 *      assigned; the input layer has number 0, Sec. "Parallel GPU activation".
 *      Reading taken here: every node without incoming edges sits in layer 0,
 *      whether or not it is a sensor.)
 *
 *   val(v)   = sigmoid(x_k)                       if v is the k-th input node
 *            = sigmoid(sum over edges (u,v) of w_uv * val(u))   otherwise
 *     (CUDA activation kernel, Sec. "Parallel GPU activation": sensors squash
 *      their input, other nodes start from sum = 0, so an empty sum gives
 *      sigmoid(0) = 0.5; Sec. "Sequential activation", second paragraph.)
 *
 *   sigmoid(x) = 1 / (1 + e^(-4.97 x))            (Introduction, display eq.)
 *
 * Nodes are visited in Kahn FIFO order (a queue of nodes, not level buckets).
 * A node's incoming edges are summed in the order they appear in the caller's
 * edge list.  Parallel edges (a,b) are legal and their contributions add.
 *
 * Precision: ASNN_ORACLE_F64 accumulates and evaluates the sigmoid in double
 * and rounds once to float when the value is stored; successors read the
 * stored float.  ASNN_ORACLE_F32 does the same arithmetic serially in float
 * (the paper's kernel declares the sum as Float); it exists to measure how
 * much the answer depends on precision and is not the reference for parity.
 *
 * Pins (tests/test_oracle_*.py): closed forms, brute force from the recursive
 * definition and longest-path enumeration on small DAGs, the paper's
 * set-based segmentation written out in oracle/segment_network.py, dense
 * matmul chains for unpruned layered nets, metamorphic relabelling.
 */
#define _POSIX_C_SOURCE 199309L   /* clock_gettime under -std=c11 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <time.h>

#define ASNN_ORACLE_OK 0
#define ASNN_ORACLE_ERR_INDEX -1
#define ASNN_ORACLE_ERR_CYCLE -2
#define ASNN_ORACLE_ERR_INPUT_HAS_INEDGE -3
#define ASNN_ORACLE_ERR_DUP_INPUT -4
#define ASNN_ORACLE_ERR_ALLOC -5

#define ASNN_ORACLE_F64 0
#define ASNN_ORACLE_F32 1

static const double SLOPE = 4.97;

typedef struct {
    int64_t *in_ptr;   /* [n+1] */
    int64_t *in_edge;  /* [e] edge indices grouped by dst, edge-list order kept */
    int64_t *out_ptr;  /* [n+1] */
    int32_t *out_dst;  /* [e] */
    int32_t *indeg;    /* [n] */
} adjacency;

static void adjacency_free(adjacency *a) {
    free(a->in_ptr); free(a->in_edge); free(a->out_ptr); free(a->out_dst); free(a->indeg);
    memset(a, 0, sizeof(*a));
}

static int adjacency_build(adjacency *a, int32_t n, int64_t e, const int32_t *src, const int32_t *dst) {
    memset(a, 0, sizeof(*a));
    for (int64_t i = 0; i < e; ++i)
        if (src[i] < 0 || src[i] >= n || dst[i] < 0 || dst[i] >= n) return ASNN_ORACLE_ERR_INDEX;
    a->in_ptr = calloc((size_t)n + 1, sizeof(int64_t));
    a->out_ptr = calloc((size_t)n + 1, sizeof(int64_t));
    a->in_edge = malloc(sizeof(int64_t) * (size_t)(e > 0 ? e : 1));
    a->out_dst = malloc(sizeof(int32_t) * (size_t)(e > 0 ? e : 1));
    a->indeg = calloc((size_t)n + 1, sizeof(int32_t));
    if (!a->in_ptr || !a->out_ptr || !a->in_edge || !a->out_dst || !a->indeg) {
        adjacency_free(a);
        return ASNN_ORACLE_ERR_ALLOC;
    }
    for (int64_t i = 0; i < e; ++i) { a->in_ptr[dst[i] + 1]++; a->out_ptr[src[i] + 1]++; }
    for (int32_t v = 0; v < n; ++v) {
        a->indeg[v] = (int32_t)a->in_ptr[v + 1];
        a->in_ptr[v + 1] += a->in_ptr[v];
        a->out_ptr[v + 1] += a->out_ptr[v];
    }
    int64_t *in_fill = malloc(sizeof(int64_t) * ((size_t)n + 1));
    int64_t *out_fill = malloc(sizeof(int64_t) * ((size_t)n + 1));
    if (!in_fill || !out_fill) { free(in_fill); free(out_fill); adjacency_free(a); return ASNN_ORACLE_ERR_ALLOC; }
    memcpy(in_fill, a->in_ptr, sizeof(int64_t) * ((size_t)n + 1));
    memcpy(out_fill, a->out_ptr, sizeof(int64_t) * ((size_t)n + 1));
    for (int64_t i = 0; i < e; ++i) {
        a->in_edge[in_fill[dst[i]]++] = i;
        a->out_dst[out_fill[src[i]]++] = dst[i];
    }
    free(in_fill); free(out_fill);
    return ASNN_ORACLE_OK;
}

/* Levels only.  level[n] receives the layer number of every node, *n_levels
 * the number of layers (max level + 1; 0 for an empty network). */
int asnn_oracle_levels(int32_t n, int64_t e, const int32_t *src, const int32_t *dst,
                       int32_t *level, int32_t *n_levels) {
    adjacency a;
    int rc = adjacency_build(&a, n, e, src, dst);
    if (rc) return rc;
    int32_t *queue = malloc(sizeof(int32_t) * ((size_t)n + 1));
    if (!queue) { adjacency_free(&a); return ASNN_ORACLE_ERR_ALLOC; }
    int32_t head = 0, tail = 0, top = -1;
    for (int32_t v = 0; v < n; ++v) {
        level[v] = 0;
        if (a.indeg[v] == 0) queue[tail++] = v;
    }
    while (head < tail) {
        int32_t v = queue[head++];
        if (level[v] > top) top = level[v];
        for (int64_t k = a.out_ptr[v]; k < a.out_ptr[v + 1]; ++k) {
            int32_t u = a.out_dst[k];
            if (level[v] + 1 > level[u]) level[u] = level[v] + 1;
            if (--a.indeg[u] == 0) queue[tail++] = u;
        }
    }
    free(queue);
    adjacency_free(&a);
    if (tail < n) return ASNN_ORACLE_ERR_CYCLE;
    *n_levels = top + 1;
    return ASNN_ORACLE_OK;
}

/* Required set R of the segmentation algorithm (its first argument: the nodes
 * needed to compute the outputs): required[v] = 1 iff some output can be
 * reached from v along connections, outputs included.  Plain reverse
 * traversal from the outputs with an explicit stack. */
int asnn_oracle_required(int32_t n, int64_t e, const int32_t *src, const int32_t *dst,
                         int32_t n_outputs, const int32_t *output_ids, int32_t *required) {
    adjacency a;
    int rc = adjacency_build(&a, n, e, src, dst);
    if (rc) return rc;
    int32_t *stack = malloc(sizeof(int32_t) * ((size_t)n + 1));
    if (!stack) { adjacency_free(&a); return ASNN_ORACLE_ERR_ALLOC; }
    int32_t top = 0;
    for (int32_t v = 0; v < n; ++v) required[v] = 0;
    for (int32_t k = 0; k < n_outputs; ++k) {
        int32_t v = output_ids[k];
        if (v < 0 || v >= n) { free(stack); adjacency_free(&a); return ASNN_ORACLE_ERR_INDEX; }
        if (!required[v]) { required[v] = 1; stack[top++] = v; }
    }
    while (top > 0) {
        int32_t v = stack[--top];
        for (int64_t k = a.in_ptr[v]; k < a.in_ptr[v + 1]; ++k) {
            int32_t u = src[a.in_edge[k]];
            if (!required[u]) { required[u] = 1; stack[top++] = u; }
        }
    }
    free(stack);
    adjacency_free(&a);
    return ASNN_ORACLE_OK;
}

static float squash_f64(double s) { return (float)(1.0 / (1.0 + exp(-SLOPE * s))); }
static float squash_f32(float s) { return 1.0f / (1.0f + expf(-4.97f * s)); }

/* Full activation.  val[n*B] (node-major, batch contiguous, ORIGINAL node
 * ids) receives the activation of every node for every input vector.
 * X[n_inputs*B]: row k feeds input_ids[k].  raw_inputs != 0 stores the input
 * values unsquashed (an option outside the paper, which squashes sensors).
 * activation_seconds (may be NULL) receives the wall time of the node loop
 * alone, i.e. without building the adjacency lists (the paper times its
 * sequential activation after its preprocessing step). */
static double now_seconds(void) {
    struct timespec ts;
    clock_gettime(CLOCK_MONOTONIC, &ts);
    return (double)ts.tv_sec + 1e-9 * (double)ts.tv_nsec;
}

int asnn_oracle_activate(int32_t n, int64_t e, const int32_t *src, const int32_t *dst, const float *w,
                         int32_t n_inputs, const int32_t *input_ids, const float *X, int32_t B,
                         int mode, int raw_inputs, float *val, double *activation_seconds) {
    adjacency a;
    int rc = adjacency_build(&a, n, e, src, dst);
    if (rc) return rc;
    int32_t *slot = malloc(sizeof(int32_t) * ((size_t)n + 1));     /* node -> row of X, or -1 */
    int32_t *queue = malloc(sizeof(int32_t) * ((size_t)n + 1));
    double *acc64 = malloc(sizeof(double) * (size_t)(B > 0 ? B : 1));
    float *acc32 = malloc(sizeof(float) * (size_t)(B > 0 ? B : 1));
    if (!slot || !queue || !acc64 || !acc32) { rc = ASNN_ORACLE_ERR_ALLOC; goto done; }
    for (int32_t v = 0; v < n; ++v) slot[v] = -1;
    for (int32_t k = 0; k < n_inputs; ++k) {
        int32_t v = input_ids[k];
        if (v < 0 || v >= n) { rc = ASNN_ORACLE_ERR_INDEX; goto done; }
        if (slot[v] >= 0) { rc = ASNN_ORACLE_ERR_DUP_INPUT; goto done; }
        if (a.indeg[v] != 0) { rc = ASNN_ORACLE_ERR_INPUT_HAS_INEDGE; goto done; }
        slot[v] = k;
    }
    int32_t head = 0, tail = 0;
    const double t_start = now_seconds();
    for (int32_t v = 0; v < n; ++v)
        if (a.indeg[v] == 0) queue[tail++] = v;
    while (head < tail) {
        int32_t v = queue[head++];
        float *out = val + (size_t)v * (size_t)B;
        if (slot[v] >= 0) {
            const float *x = X + (size_t)slot[v] * (size_t)B;
            for (int32_t b = 0; b < B; ++b)
                out[b] = raw_inputs ? x[b] : (mode == ASNN_ORACLE_F64 ? squash_f64((double)x[b]) : squash_f32(x[b]));
        } else if (mode == ASNN_ORACLE_F64) {
            for (int32_t b = 0; b < B; ++b) acc64[b] = 0.0;
            for (int64_t k = a.in_ptr[v]; k < a.in_ptr[v + 1]; ++k) {
                int64_t ed = a.in_edge[k];
                const double wt = (double)w[ed];
                const float *row = val + (size_t)src[ed] * (size_t)B;
                for (int32_t b = 0; b < B; ++b) acc64[b] += wt * (double)row[b];
            }
            for (int32_t b = 0; b < B; ++b) out[b] = squash_f64(acc64[b]);
        } else {
            for (int32_t b = 0; b < B; ++b) acc32[b] = 0.0f;
            for (int64_t k = a.in_ptr[v]; k < a.in_ptr[v + 1]; ++k) {
                int64_t ed = a.in_edge[k];
                const float wt = w[ed];
                const float *row = val + (size_t)src[ed] * (size_t)B;
                for (int32_t b = 0; b < B; ++b) acc32[b] += wt * row[b];
            }
            for (int32_t b = 0; b < B; ++b) out[b] = squash_f32(acc32[b]);
        }
        for (int64_t k = a.out_ptr[v]; k < a.out_ptr[v + 1]; ++k) {
            int32_t u = a.out_dst[k];
            if (--a.indeg[u] == 0) queue[tail++] = u;
        }
    }
    if (activation_seconds) *activation_seconds = now_seconds() - t_start;
    if (tail < n) rc = ASNN_ORACLE_ERR_CYCLE;
done:
    free(slot); free(queue); free(acc64); free(acc32);
    adjacency_free(&a);
    return rc;
}
