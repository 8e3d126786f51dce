/*
 * CPU oracle for dynamic batching of per-example dynamic architectures.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, one-thing-at-a-time C that states what the
 * batched GPU path must compute.  It shares no code, headers, tables or helpers with the
 * HIP library and is only ever called from tests, the smoke check and the benchmark's
 * CPU-baseline leg.
 *
 * Paper: "Effective Approaches to Batch Parallelization for Dynamic Neural Network
 * Architectures" (Suarez & Zhu).
 *   - Background / Visual Reasoning Programs: a program is a sequence of function ids whose
 *     fixed arities give a unique tree, assembled depth first; a SCENE token outputs the
 *     example's image features; every other function is a neural network.
 *   - Methods / Improved topological sort: label every node by its distance from the root,
 *     pool nodes with the same label, run each pool with at most p network calls.
 *   - Methods / Standard topological sort: flatten each program into a dependency-respecting
 *     queue, view the batch as a b x s grid and run it column by column, at most p calls each.
 *   - Results / IEP: the unbatched original loops over examples and runs one module at a
 *     time; the batched version builds the same network, so outputs must agree.
 *   - Results / Sparsely Gated Mixture of Experts: n experts, k active per example; the
 *     naive version runs the k*b expert uses one by one.
 *   - Background / Visual Reasoning Programs, last step: the executed program's output map goes through a
 *     small classifier (one convolutional and two fully connected layers) that yields a softmax
 *     distribution over answers (oracle_classify).
 *   - Results / IEP also times the backward pass: oracle_iep_backward is the gradient of the executed
 *     programs (weights, biases and input feature maps) by the chain rule, node by node, written as the
 *     transpose of the forward loops.
 *   - Discussion: batching by dependency depth (labels counted up from the argument-free nodes),
 *     and architectures given as a general dependency graph in which a node may have several
 *     consumers (there the label is the MAXIMUM distance from the root, as Methods words it).
 * The module (residual conv block), the noisy top-k gate and all sizes are fixed by the
 * benchmark configurations, not by the paper.
 *
 * All floating point here is fp64 (inputs arrive as fp32 arrays and are widened).
 * Float parity of every function below is pinned by tests against library routines,
 * closed forms and brute force; none is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_OK 0
#define ORC_E_MALFORMED (-2)
#define ORC_E_INVAL (-1)

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ------------------------------------------------------------------------------------------
 * Plan oracle (integers).
 * ---------------------------------------------------------------------------------------- */

typedef struct {
    const int32_t* prog;    /* this example's tokens */
    int32_t len;
    int32_t base;           /* node id of token 0 = prog_off[example] */
    const uint8_t* arity;
    int32_t n_types;
    int32_t* level;         /* indexed by global node id */
    int32_t* child0;
    int32_t* child1;
    int32_t* post;          /* post[j] = global node id of the j-th node in the post-order queue */
    int32_t n_post;
    int bad;
} tree_ctx;

/* Depth-first assembly (Background / Visual Reasoning Programs): the children of the token at
 * `pos` are the sub-programs that follow it, one per argument.  Root distance is recorded on
 * the way down (Methods / Improved topological sort), the dependency-respecting queue on the
 * way up (Methods / Standard topological sort: a node enters the queue after its arguments). */
static int32_t build(tree_ctx* c, int32_t pos, int32_t lvl)
{
    if (pos >= c->len) { c->bad = 1; return pos; }
    int32_t t = c->prog[pos];
    if (t < 0 || t >= c->n_types || c->arity[t] > 2) { c->bad = 1; return c->len + 1; }
    int32_t id = c->base + pos;
    c->level[id] = lvl;
    c->child0[id] = -1;
    c->child1[id] = -1;
    int32_t next = pos + 1;
    for (int a = 0; a < c->arity[t]; ++a) {
        if (next >= c->len) { c->bad = 1; return next; }
        if (a == 0) c->child0[id] = c->base + next; else c->child1[id] = c->base + next;
        next = build(c, next, lvl + 1);
        if (c->bad) return next;
    }
    c->post[c->n_post++] = id;
    return next;
}

/* Dependency depth of a node (Discussion: batching "by dependency depth" as TensorFlow Fold
 * does): a node without arguments has depth 0, any other node is one deeper than its deepest
 * argument.  Plain recursion from the definition, recomputed for every node. */
static int32_t dependency_depth(const int32_t* child0, const int32_t* child1, int32_t id)
{
    int32_t d = 0;
    if (child0[id] >= 0) {
        int32_t a = dependency_depth(child0, child1, child0[id]) + 1;
        if (a > d) d = a;
    }
    if (child1[id] >= 0) {
        int32_t b = dependency_depth(child0, child1, child1[id]) + 1;
        if (b > d) d = b;
    }
    return d;
}

/* mode 0: label = distance from the root, pools run deepest label first (improved sort).
 * mode 1: label = position in the example's post-order queue, pools (grid columns) run in
 *         ascending order (standard sort).
 * mode 2: label = dependency depth (0 for argument-free nodes), pools run in ascending order.
 * Within a label, one pool per function id, ascending; members ascending by node id.
 * Returns ORC_OK, or ORC_E_MALFORMED with *bad_example set.
 * Caller provides: level/type/child0/child1/members/in0/in1/out [N], root [B],
 * bucket_* [N] (worst case one bucket per node).                                            */
int oracle_plan(const int32_t* prog, const int32_t* prog_off, int32_t B, const uint8_t* arity,
                int32_t n_types, int32_t mode,
                int32_t* level, int32_t* type, int32_t* child0, int32_t* child1, int32_t* root,
                int32_t* n_levels, int32_t* n_buckets, int32_t* bucket_level, int32_t* bucket_type,
                int32_t* bucket_start, int32_t* bucket_count, int32_t* members, int32_t* in0,
                int32_t* in1, int32_t* out, int32_t* bad_example)
{
    if (!prog || !prog_off || B <= 0 || !arity || n_types <= 0 || mode < 0 || mode > 2) return ORC_E_INVAL;
    int32_t N = prog_off[B];
    int32_t* rootdist = (int32_t*)malloc(sizeof(int32_t) * (size_t)(N > 0 ? N : 1));
    int32_t* post = (int32_t*)malloc(sizeof(int32_t) * (size_t)(N > 0 ? N : 1));
    int32_t D = 0;
    for (int32_t i = 0; i < B; ++i) {
        tree_ctx c;
        c.prog = prog + prog_off[i];
        c.len = prog_off[i + 1] - prog_off[i];
        c.base = prog_off[i];
        c.arity = arity;
        c.n_types = n_types;
        c.level = rootdist;
        c.child0 = child0;
        c.child1 = child1;
        c.post = post + prog_off[i];
        c.n_post = 0;
        c.bad = 0;
        int32_t end = (c.len > 0) ? build(&c, 0, 0) : -1;
        if (c.bad || end != c.len) {          /* ends early, or tokens left over */
            if (bad_example) *bad_example = i;
            free(rootdist); free(post);
            return ORC_E_MALFORMED;
        }
        root[i] = c.base;
        for (int32_t j = 0; j < c.len; ++j) {
            int32_t id = c.base + j;
            type[id] = c.prog[j];
            if (mode == 0) level[id] = rootdist[id];
        }
        if (mode == 1)
            for (int32_t j = 0; j < c.n_post; ++j) level[post[prog_off[i] + j]] = j;
        if (mode == 2)
            for (int32_t j = 0; j < c.len; ++j) level[c.base + j] = dependency_depth(child0, child1, c.base + j);
        for (int32_t j = 0; j < c.len; ++j)
            if (level[c.base + j] + 1 > D) D = level[c.base + j] + 1;   /* max over the minibatch */
    }
    *n_levels = D;

    int32_t nb = 0, filled = 0;
    for (int32_t step = 0; step < D; ++step) {
        int32_t lvl = (mode == 0) ? D - 1 - step : step;
        for (int32_t t = 0; t < n_types; ++t) {
            int32_t start = filled;
            for (int32_t id = 0; id < N; ++id)
                if (level[id] == lvl && type[id] == t) {
                    members[filled] = id;
                    in0[filled] = child0[id];
                    in1[filled] = child1[id];
                    out[filled] = id;
                    ++filled;
                }
            if (filled > start) {
                bucket_level[nb] = lvl;
                bucket_type[nb] = t;
                bucket_start[nb] = start;
                bucket_count[nb] = filled - start;
                ++nb;
            }
        }
    }
    *n_buckets = nb;
    free(rootdist); free(post);
    return ORC_OK;
}

/* ------------------------------------------------------------------------------------------
 * IEP float oracle: one example at a time, one module at a time, by tree recursion.
 * Feature maps are [H][W][C] (channels innermost); conv weights [Cout][kh][kw][Cin].
 * ---------------------------------------------------------------------------------------- */

typedef struct {
    int C, H, W;
    int n_types;
    const uint8_t* arity;
    const float *w1, *b1, *w3a, *b3a, *w3b, *b3b;   /* [n_types, ...], biases may be NULL */
} modules;

/* cross-correlation, zero padding 1, stride 1 */
static void conv3x3(const double* in, const float* w, const float* b, double* out, int C, int H, int W)
{
    for (int y = 0; y < H; ++y)
        for (int x = 0; x < W; ++x)
            for (int co = 0; co < C; ++co) {
                double acc = b ? (double)b[co] : 0.0;
                for (int kh = 0; kh < 3; ++kh) {
                    int iy = y + kh - 1;
                    if (iy < 0 || iy >= H) continue;
                    for (int kw = 0; kw < 3; ++kw) {
                        int ix = x + kw - 1;
                        if (ix < 0 || ix >= W) continue;
                        const double* px = in + ((size_t)iy * W + ix) * C;
                        const float* wk = w + (((size_t)co * 3 + kh) * 3 + kw) * C;
                        for (int ci = 0; ci < C; ++ci) acc += px[ci] * (double)wk[ci];
                    }
                }
                out[((size_t)y * W + x) * C + co] = acc;
            }
}

static void relu_inplace(double* a, size_t n)
{
    for (size_t i = 0; i < n; ++i) if (!(a[i] > 0.0)) a[i] = 0.0;
}

/* Res_t(u) = ReLU(u + conv3x3_b(ReLU(conv3x3_a(u) + b_a)) + b_b) */
static void residual_block(const modules* m, int t, const double* u, double* y)
{
    size_t n = (size_t)m->H * m->W * m->C;
    size_t w3 = (size_t)m->C * 9 * m->C;
    double* mid = (double*)malloc(n * sizeof(double));
    conv3x3(u, m->w3a + t * w3, m->b3a ? m->b3a + (size_t)t * m->C : NULL, mid, m->C, m->H, m->W);
    relu_inplace(mid, n);
    conv3x3(mid, m->w3b + t * w3, m->b3b ? m->b3b + (size_t)t * m->C : NULL, y, m->C, m->H, m->W);
    for (size_t i = 0; i < n; ++i) y[i] += u[i];
    relu_inplace(y, n);
    free(mid);
}

/* u = ReLU(conv1x1_{2C->C}(concat_C(a, b)) + b1): first argument feeds input channels [0,C) */
static void join1x1(const modules* m, int t, const double* a, const double* b, double* u)
{
    int C = m->C;
    const float* w = m->w1 + (size_t)t * C * 2 * C;
    for (size_t p = 0; p < (size_t)m->H * m->W; ++p)
        for (int co = 0; co < C; ++co) {
            double acc = m->b1 ? (double)m->b1[(size_t)t * C + co] : 0.0;
            for (int ci = 0; ci < C; ++ci) acc += a[p * C + ci] * (double)w[(size_t)co * 2 * C + ci];
            for (int ci = 0; ci < C; ++ci) acc += b[p * C + ci] * (double)w[(size_t)co * 2 * C + C + ci];
            u[p * C + co] = acc > 0.0 ? acc : 0.0;
        }
}

/* Evaluates the sub-program starting at *pos and advances *pos past it. Returns a malloc'd map. */
static double* eval_node(const modules* m, const int32_t* prog, int32_t* pos, const float* feat)
{
    size_t n = (size_t)m->H * m->W * m->C;
    int t = prog[(*pos)++];
    double* y = (double*)malloc(n * sizeof(double));
    if (m->arity[t] == 0) {                     /* SCENE: the example's image features */
        for (size_t i = 0; i < n; ++i) y[i] = (double)feat[i];
    } else if (m->arity[t] == 1) {
        double* u = eval_node(m, prog, pos, feat);
        residual_block(m, t, u, y);
        free(u);
    } else {
        double* a = eval_node(m, prog, pos, feat);
        double* b = eval_node(m, prog, pos, feat);
        double* u = (double*)malloc(n * sizeof(double));
        join1x1(m, t, a, b, u);
        residual_block(m, t, u, y);
        free(a); free(b); free(u);
    }
    return y;
}

/* Programs must be well formed (check with oracle_plan first). out: double [B,H,W,C]. */
int oracle_iep_forward(const int32_t* prog, const int32_t* prog_off, int32_t B, const uint8_t* arity,
                       int32_t n_types, int32_t C, int32_t H, int32_t W, const float* feats,
                       const float* w1, const float* b1, const float* w3a, const float* b3a,
                       const float* w3b, const float* b3b, double* out)
{
    if (!prog || !prog_off || B <= 0 || !feats || !out || !w3a || !w3b) return ORC_E_INVAL;
    modules m = { C, H, W, n_types, arity, w1, b1, w3a, b3a, w3b, b3b };
    size_t n = (size_t)H * W * C;
    /* examples are independent: the only parallelism is across them */
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t i = 0; i < B; ++i) {
        int32_t pos = 0;
        double* y = eval_node(&m, prog + prog_off[i], &pos, feats + (size_t)i * n);
        memcpy(out + (size_t)i * n, y, n * sizeof(double));
        free(y);
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------------------------
 * General dependency graphs (Discussion: the method applies to any architecture whose dependency
 * graph is known before execution; Methods / Improved topological sort labels a node with its
 * MAXIMUM distance from the root, which only differs from the plain distance when a node has
 * several consumers).  An example is a list of nodes with explicit argument indices (local to the
 * example, -1 = none) and one root; a node may feed several consumers and is evaluated once.
 * ---------------------------------------------------------------------------------------- */

typedef struct {
    const int32_t *type, *arg0, *arg1;   /* this example's nodes */
    int32_t n, root;
    int32_t* memo;                       /* -2 unknown, -3 being computed (a cycle if met again) */
    int bad;
} dag_ctx;

/* Longest path from the root down to node id: 0 for the root, else one more than the largest
 * value among the nodes that take id as an argument; -1 if no chain of consumers reaches the root. */
static int32_t max_root_distance(dag_ctx* c, int32_t id)
{
    if (c->memo[id] == -3) { c->bad = 1; return -1; }
    if (c->memo[id] != -2) return c->memo[id];
    if (id == c->root) { c->memo[id] = 0; return 0; }
    c->memo[id] = -3;
    int32_t best = -1;
    for (int32_t q = 0; q < c->n && !c->bad; ++q)
        if (c->arg0[q] == id || c->arg1[q] == id) {
            int32_t dq = max_root_distance(c, q);
            if (dq >= 0 && dq + 1 > best) best = dq + 1;
        }
    c->memo[id] = best;
    return best;
}

/* Dependency depth with a cycle guard: 0 without arguments, else one more than the deepest argument. */
static int32_t dag_dependency_depth(dag_ctx* c, int32_t id)
{
    if (c->memo[id] == -3) { c->bad = 1; return 0; }
    if (c->memo[id] != -2) return c->memo[id];
    c->memo[id] = -3;
    int32_t d = 0;
    if (c->arg0[id] >= 0) { int32_t a = dag_dependency_depth(c, c->arg0[id]) + 1; if (a > d) d = a; }
    if (c->arg1[id] >= 0 && !c->bad) { int32_t b = dag_dependency_depth(c, c->arg1[id]) + 1; if (b > d) d = b; }
    c->memo[id] = d;
    return d;
}

/* mode 0: label = maximum distance from the root, pools deepest label first.
 * mode 2: label = dependency depth, pools in ascending order.
 * An example is malformed if a function id or argument index is out of range, the number of
 * arguments differs from the function's arity, the graph has a cycle, the root is out of range,
 * or some node does not contribute to the root.  Outputs as oracle_plan (child0/child1 = global
 * ids of the arguments, root = global id).                                                    */
int oracle_plan_dag(const int32_t* type_in, const int32_t* arg0, const int32_t* arg1, const int32_t* node_off,
                    const int32_t* root_local, int32_t B, const uint8_t* arity, int32_t n_types, int32_t mode,
                    int32_t* level, int32_t* type, int32_t* child0, int32_t* child1, int32_t* root,
                    int32_t* n_levels, int32_t* n_buckets, int32_t* bucket_level, int32_t* bucket_type,
                    int32_t* bucket_start, int32_t* bucket_count, int32_t* members, int32_t* in0,
                    int32_t* in1, int32_t* out, int32_t* bad_example)
{
    if (!type_in || !arg0 || !arg1 || !node_off || !root_local || B <= 0 || !arity || n_types <= 0 ||
        (mode != 0 && mode != 2))
        return ORC_E_INVAL;
    int32_t N = node_off[B], D = 0;
    int32_t* memo = (int32_t*)malloc(sizeof(int32_t) * (size_t)(N > 0 ? N : 1));
    for (int32_t i = 0; i < B; ++i) {
        int32_t base = node_off[i], n = node_off[i + 1] - base;
        int bad = (n <= 0 || root_local[i] < 0 || root_local[i] >= n);
        for (int32_t j = 0; j < n && !bad; ++j) {
            int32_t t = type_in[base + j], a = arg0[base + j], b = arg1[base + j];
            if (t < 0 || t >= n_types || arity[t] > 2 || a < -1 || a >= n || b < -1 || b >= n) { bad = 1; break; }
            int given = (a >= 0) + (b >= 0);
            if (given != arity[t] || (b >= 0 && a < 0)) bad = 1;
        }
        dag_ctx c = { type_in + base, arg0 + base, arg1 + base, n, bad ? 0 : root_local[i], memo + base, 0 };
        if (!bad) {
            /* a cycle anywhere makes the example malformed: walk the argument edges first */
            for (int32_t j = 0; j < n; ++j) c.memo[j] = -2;
            for (int32_t j = 0; j < n && !c.bad; ++j) dag_dependency_depth(&c, j);
            bad = c.bad;
        }
        if (!bad && mode == 0) {
            for (int32_t j = 0; j < n; ++j) c.memo[j] = -2;
            for (int32_t j = 0; j < n; ++j) level[base + j] = max_root_distance(&c, j);
        } else if (!bad) {
            for (int32_t j = 0; j < n; ++j) level[base + j] = c.memo[j];
            /* reachability is judged on root distances in both modes */
            int32_t* dist = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
            dag_ctx r = { c.type, c.arg0, c.arg1, n, c.root, dist, 0 };
            for (int32_t j = 0; j < n; ++j) dist[j] = -2;
            for (int32_t j = 0; j < n; ++j) if (max_root_distance(&r, j) < 0) bad = 1;
            free(dist);
        }
        for (int32_t j = 0; j < n && !bad; ++j) if (level[base + j] < 0) bad = 1;   /* feeds nothing */
        if (bad) {
            if (bad_example) *bad_example = i;
            free(memo);
            return ORC_E_MALFORMED;
        }
        root[i] = base + root_local[i];
        for (int32_t j = 0; j < n; ++j) {
            type[base + j] = type_in[base + j];
            child0[base + j] = arg0[base + j] >= 0 ? base + arg0[base + j] : -1;
            child1[base + j] = arg1[base + j] >= 0 ? base + arg1[base + j] : -1;
            if (level[base + j] + 1 > D) D = level[base + j] + 1;
        }
    }
    free(memo);
    *n_levels = D;
    int32_t nb = 0, filled = 0;
    for (int32_t step = 0; step < D; ++step) {
        int32_t lvl = (mode == 0) ? D - 1 - step : step;
        for (int32_t t = 0; t < n_types; ++t) {
            int32_t start = filled;
            for (int32_t id = 0; id < N; ++id)
                if (level[id] == lvl && type[id] == t) {
                    members[filled] = id;
                    in0[filled] = child0[id];
                    in1[filled] = child1[id];
                    out[filled] = id;
                    ++filled;
                }
            if (filled > start) {
                bucket_level[nb] = lvl;
                bucket_type[nb] = t;
                bucket_start[nb] = start;
                bucket_count[nb] = filled - start;
                ++nb;
            }
        }
    }
    *n_buckets = nb;
    return ORC_OK;
}

/* Value of node id of one example; every node is computed once and kept in val[] (NULL = not yet). */
static const double* eval_dag_node(const modules* m, const int32_t* type, const int32_t* arg0, const int32_t* arg1,
                                   int32_t id, const float* feat, double** val)
{
    if (val[id]) return val[id];
    size_t n = (size_t)m->H * m->W * m->C;
    int t = type[id];
    double* y = (double*)malloc(n * sizeof(double));
    if (m->arity[t] == 0) {
        for (size_t i = 0; i < n; ++i) y[i] = (double)feat[i];
    } else if (m->arity[t] == 1) {
        residual_block(m, t, eval_dag_node(m, type, arg0, arg1, arg0[id], feat, val), y);
    } else {
        const double* a = eval_dag_node(m, type, arg0, arg1, arg0[id], feat, val);
        const double* b = eval_dag_node(m, type, arg0, arg1, arg1[id], feat, val);
        double* u = (double*)malloc(n * sizeof(double));
        join1x1(m, t, a, b, u);
        residual_block(m, t, u, y);
        free(u);
    }
    val[id] = y;
    return y;
}

/* Graphs must be well formed (check with oracle_plan_dag first). out: double [B,H,W,C]. */
int oracle_iep_forward_dag(const int32_t* type, const int32_t* arg0, const int32_t* arg1, const int32_t* node_off,
                           const int32_t* root_local, int32_t B, const uint8_t* arity, int32_t n_types,
                           int32_t C, int32_t H, int32_t W, const float* feats, const float* w1, const float* b1,
                           const float* w3a, const float* b3a, const float* w3b, const float* b3b, double* out)
{
    if (!type || !arg0 || !arg1 || !node_off || !root_local || B <= 0 || !feats || !out || !w3a || !w3b)
        return ORC_E_INVAL;
    modules m = { C, H, W, n_types, arity, w1, b1, w3a, b3a, w3b, b3b };
    size_t n = (size_t)H * W * C;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t i = 0; i < B; ++i) {
        int32_t base = node_off[i], cnt = node_off[i + 1] - base;
        double** val = (double**)calloc((size_t)cnt, sizeof(double*));
        const double* y = eval_dag_node(&m, type + base, arg0 + base, arg1 + base, root_local[i],
                                        feats + (size_t)i * n, val);
        memcpy(out + (size_t)i * n, y, n * sizeof(double));
        for (int32_t j = 0; j < cnt; ++j) free(val[j]);
        free(val);
    }
    return ORC_OK;
}

/* single convolution entry points, exported so tests can pin them against library routines */
void oracle_conv3x3(const float* in, const float* w, const float* b, double* out, int C, int H, int W)
{
    size_t n = (size_t)H * W * C;
    double* d = (double*)malloc(n * sizeof(double));
    for (size_t i = 0; i < n; ++i) d[i] = (double)in[i];
    conv3x3(d, w, b, out, C, H, W);
    free(d);
}

/* ------------------------------------------------------------------------------------------
 * Mixture-of-experts oracle: token by token.
 * ---------------------------------------------------------------------------------------- */

static double softplus(double z) { return (z > 0.0 ? z : 0.0) + log1p(exp(-fabs(z))); }

/* logit[t,e] = x_t . Wg[:,e] + noise[t,e] * softplus(x_t . Wn[:,e]);  Wg, Wn are [d,E]. */
void oracle_moe_logits(const float* x, const float* Wg, const float* Wn, const float* noise,
                       int32_t T, int32_t d, int32_t E, double* logits)
{
#pragma omp parallel for schedule(static)
    for (int32_t t = 0; t < T; ++t)
        for (int32_t e = 0; e < E; ++e) {
            double g = 0.0, s = 0.0;
            for (int32_t c = 0; c < d; ++c) {
                g += (double)x[(size_t)t * d + c] * (double)Wg[(size_t)c * E + e];
                if (noise) s += (double)x[(size_t)t * d + c] * (double)Wn[(size_t)c * E + e];
            }
            logits[(size_t)t * E + e] = noise ? g + (double)noise[(size_t)t * E + e] * softplus(s) : g;
        }
}

/* Routing from fp32 logits (decisions are taken on the fp32 values, so they are exact):
 * k largest per token, equal logits -> lower expert id first; softmax over the k kept logits;
 * then the grouping of the k*T known expert uses by expert, stable in the flat use id a = t*k+j:
 * counts[E], offsets[E+1], perm[A] (sorted position -> use id), inv[A] (use id -> position).     */
int oracle_moe_route(const float* logits, int32_t T, int32_t E, int32_t k, int32_t* topk_idx,
                     double* topk_w, int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv)
{
    if (k <= 0 || k > E) return ORC_E_INVAL;
    for (int32_t t = 0; t < T; ++t) {
        const float* row = logits + (size_t)t * E;
        for (int32_t j = 0; j < k; ++j) {
            int32_t best = -1;
            for (int32_t e = 0; e < E; ++e) {
                int taken = 0;
                for (int32_t q = 0; q < j; ++q) if (topk_idx[(size_t)t * k + q] == e) taken = 1;
                if (taken) continue;
                if (best < 0 || row[e] > row[best]) best = e;     /* strict >: lower id wins ties */
            }
            topk_idx[(size_t)t * k + j] = best;
        }
        double mx = (double)row[topk_idx[(size_t)t * k]];
        double den = 0.0;
        for (int32_t j = 0; j < k; ++j) den += exp((double)row[topk_idx[(size_t)t * k + j]] - mx);
        for (int32_t j = 0; j < k; ++j)
            topk_w[(size_t)t * k + j] = exp((double)row[topk_idx[(size_t)t * k + j]] - mx) / den;
    }
    int32_t A = T * k, pos = 0;
    for (int32_t e = 0; e < E; ++e) {
        offsets[e] = pos;
        for (int32_t a = 0; a < A; ++a)
            if (topk_idx[a] == e) { perm[pos] = a; inv[a] = pos; ++pos; }
        counts[e] = pos - offsets[e];
    }
    offsets[E] = pos;
    return ORC_OK;
}

/* One token through its k experts: out = sum_j w[j] * W2_j . ReLU(W1_j . x)  (no biases: the
 * paper counts 2*h*n*d parameters).  W1_j is [h,d], W2_j is [d,h] (one output unit per row). */
void oracle_moe_token(const float* x, int32_t d, int32_t h, int32_t k, const double* w,
                      const float* const* W1, const float* const* W2, double* out)
{
    double* hid = (double*)malloc(sizeof(double) * (size_t)h);
    for (int32_t c = 0; c < d; ++c) out[c] = 0.0;
    for (int32_t j = 0; j < k; ++j) {
        for (int32_t u = 0; u < h; ++u) {
            double acc = 0.0;
            for (int32_t c = 0; c < d; ++c) acc += (double)W1[j][(size_t)u * d + c] * (double)x[c];
            hid[u] = acc > 0.0 ? acc : 0.0;
        }
        for (int32_t c = 0; c < d; ++c) {
            double acc = 0.0;
            for (int32_t u = 0; u < h; ++u) acc += (double)W2[j][(size_t)c * h + u] * hid[u];
            out[c] += w[j] * acc;
        }
    }
    free(hid);
}

/* All tokens, experts stored contiguously: W1 [E,h,d], W2 [E,d,h]. out: double [T,d]. */
void oracle_moe_experts(const float* x, const int32_t* topk_idx, const double* topk_w,
                        const float* W1, const float* W2, int32_t T, int32_t d, int32_t h,
                        int32_t k, double* out)
{
#pragma omp parallel for schedule(dynamic, 16)
    for (int32_t t = 0; t < T; ++t) {
        const float* p1[64];
        const float* p2[64];
        for (int32_t j = 0; j < k && j < 64; ++j) {
            int32_t e = topk_idx[(size_t)t * k + j];
            p1[j] = W1 + (size_t)e * h * d;
            p2[j] = W2 + (size_t)e * d * h;
        }
        oracle_moe_token(x + (size_t)t * d, d, h, k, topk_w + (size_t)t * k, p1, p2, out + (size_t)t * d);
    }
}

/* ----------------------------------------------------------------------------------------
 * Classifier head (Background / Visual Reasoning Programs: the root map passes through one convolutional
 * and two fully connected layers, then a softmax over the answers).  The paper gives no sizes or kernel
 * shape; the reading taken: a 1x1 convolution C -> Cc with ReLU, the map flattened in [H][W][Cc] order,
 * a fully connected layer to F units with ReLU, a fully connected layer to A answers, softmax.
 *   x    [B][H][W][C]        root maps
 *   wc   [Cc][C], bc [Cc]    convolution (bias NULL = none)
 *   wf1  [F][H*W*Cc], bf1 [F]
 *   wf2  [A][F], bf2 [A]
 *   probs [B][A]  (double), logits [B][A] (double, may be NULL)
 * One example at a time, every sum written out. */
int oracle_classify(const float* x, int32_t B, int32_t C, int32_t H, int32_t W, int32_t Cc, int32_t F, int32_t A,
                    const float* wc, const float* bc, const float* wf1, const float* bf1,
                    const float* wf2, const float* bf2, double* probs, double* logits)
{
    if (!x || !wc || !wf1 || !wf2 || !probs || B <= 0 || C <= 0 || H <= 0 || W <= 0 || Cc <= 0 || F <= 0 || A <= 0)
        return ORC_E_INVAL;
    const size_t P = (size_t)H * W, J = P * (size_t)Cc;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t i = 0; i < B; ++i) {
        double* z = (double*)malloc(sizeof(double) * J);
        double* h1 = (double*)malloc(sizeof(double) * (size_t)F);
        double* lg = (double*)malloc(sizeof(double) * (size_t)A);
        const float* xi = x + (size_t)i * P * C;
        for (size_t p = 0; p < P; ++p)
            for (int32_t cc = 0; cc < Cc; ++cc) {
                double acc = bc ? (double)bc[cc] : 0.0;
                for (int32_t c = 0; c < C; ++c) acc += (double)xi[p * C + c] * (double)wc[(size_t)cc * C + c];
                z[p * Cc + cc] = acc > 0.0 ? acc : 0.0;
            }
        for (int32_t f = 0; f < F; ++f) {
            double acc = bf1 ? (double)bf1[f] : 0.0;
            for (size_t j = 0; j < J; ++j) acc += z[j] * (double)wf1[(size_t)f * J + j];
            h1[f] = acc > 0.0 ? acc : 0.0;
        }
        double mx = -INFINITY;
        for (int32_t a = 0; a < A; ++a) {
            double acc = bf2 ? (double)bf2[a] : 0.0;
            for (int32_t f = 0; f < F; ++f) acc += h1[f] * (double)wf2[(size_t)a * F + f];
            lg[a] = acc;
            if (acc > mx) mx = acc;
        }
        double den = 0.0;
        for (int32_t a = 0; a < A; ++a) den += exp(lg[a] - mx);
        for (int32_t a = 0; a < A; ++a) {
            probs[(size_t)i * A + a] = exp(lg[a] - mx) / den;
            if (logits) logits[(size_t)i * A + a] = lg[a];
        }
        free(z); free(h1); free(lg);
    }
    return ORC_OK;
}

/* ----------------------------------------------------------------------------------------
 * Backward pass of the executed programs (Results / IEP times it next to inference).
 * With dout[i] the gradient of a scalar loss with respect to example i's root map, this computes the
 * gradient with respect to every module parameter (summed over all nodes that use the function, in all
 * examples) and with respect to every example's input feature map (summed over its SCENE leaves).
 * Per example: the tree is evaluated once keeping every node's u (input of the residual block), mid
 * (after the first ReLU) and y; then the chain rule walks from the root down, each step the literal
 * transpose of the forward loop nest it differentiates.
 * ---------------------------------------------------------------------------------------- */
typedef struct bnode {
    int t;
    struct bnode *a, *b;          /* arguments (NULL for SCENE / unary's second) */
    double *y, *u, *mid;          /* y owned; u owned for binary nodes, else an alias of a->y; mid owned */
} bnode;

typedef struct {
    double *dw1, *db1, *dw3a, *db3a, *dw3b, *db3b;   /* shapes of the parameters, [n_types, ...] */
} grads;

/* Nearest bfloat16 (round to nearest even) of a double, as a double. */
static double to_bf16(double v)
{
    float f = (float)v;
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return v;              /* NaN */
    u += 0x7fffu + ((u >> 16) & 1u);
    u &= 0xffff0000u;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* round_bf16 != 0: every stored activation (the 1x1 output u, mid, y) is rounded to bfloat16 where a bf16
 * implementation stores it, so that the ReLU decisions of the backward pass are taken on the values such an
 * implementation holds; the arithmetic in between stays fp64. */
static int g_round_bf16 = 0;
#pragma omp threadprivate(g_round_bf16)

static void store_round(double* a, size_t n)
{
    if (!g_round_bf16) return;
    for (size_t i = 0; i < n; ++i) a[i] = to_bf16(a[i]);
}

static bnode* bfwd(const modules* m, const int32_t* prog, int32_t* pos, const float* feat)
{
    size_t n = (size_t)m->H * m->W * m->C, w3 = (size_t)m->C * 9 * m->C;
    bnode* nd = (bnode*)calloc(1, sizeof(bnode));
    nd->t = prog[(*pos)++];
    nd->y = (double*)malloc(n * sizeof(double));
    if (m->arity[nd->t] == 0) {
        for (size_t i = 0; i < n; ++i) nd->y[i] = (double)feat[i];
        return nd;
    }
    nd->a = bfwd(m, prog, pos, feat);
    if (m->arity[nd->t] == 2) {
        nd->b = bfwd(m, prog, pos, feat);
        nd->u = (double*)malloc(n * sizeof(double));
        join1x1(m, nd->t, nd->a->y, nd->b->y, nd->u);
        store_round(nd->u, n);
    } else {
        nd->u = nd->a->y;
    }
    nd->mid = (double*)malloc(n * sizeof(double));
    conv3x3(nd->u, m->w3a + nd->t * w3, m->b3a ? m->b3a + (size_t)nd->t * m->C : NULL, nd->mid, m->C, m->H, m->W);
    relu_inplace(nd->mid, n);
    store_round(nd->mid, n);
    conv3x3(nd->mid, m->w3b + nd->t * w3, m->b3b ? m->b3b + (size_t)nd->t * m->C : NULL, nd->y, m->C, m->H, m->W);
    for (size_t i = 0; i < n; ++i) nd->y[i] += nd->u[i];
    relu_inplace(nd->y, n);
    store_round(nd->y, n);
    return nd;
}

static void bfree(const modules* m, bnode* nd)
{
    if (!nd) return;
    bfree(m, nd->a); bfree(m, nd->b);
    if (m->arity[nd->t] == 2) free(nd->u);
    free(nd->mid); free(nd->y); free(nd);
}

/* Transpose of conv3x3: given gout = dL/d(out), adds dL/dw to dw and dL/db to db, and writes gin = dL/d(in). */
static void conv3x3_backward(const double* gout, const double* in, const float* w, double* gin, double* dw, double* db,
                             int C, int H, int W)
{
    memset(gin, 0, sizeof(double) * (size_t)H * W * C);
    for (int y = 0; y < H; ++y)
        for (int x = 0; x < W; ++x)
            for (int co = 0; co < C; ++co) {
                const double g = gout[((size_t)y * W + x) * C + co];
                db[co] += g;                                   /* out = b[co] + ... */
                for (int kh = 0; kh < 3; ++kh) {
                    int iy = y + kh - 1;
                    if (iy < 0 || iy >= H) continue;
                    for (int kw = 0; kw < 3; ++kw) {
                        int ix = x + kw - 1;
                        if (ix < 0 || ix >= W) continue;
                        const double* px = in + ((size_t)iy * W + ix) * C;
                        double* gpx = gin + ((size_t)iy * W + ix) * C;
                        const size_t wo = (((size_t)co * 3 + kh) * 3 + kw) * C;
                        for (int ci = 0; ci < C; ++ci) {       /* out += px[ci] * w[wo + ci] */
                            dw[wo + ci] += g * px[ci];
                            gpx[ci] += g * (double)w[wo + ci];
                        }
                    }
                }
            }
}

static void bbwd(const modules* m, const grads* gr, const bnode* nd, const double* dy, double* dfeat)
{
    const int C = m->C;
    const size_t P = (size_t)m->H * m->W, n = P * C, w3 = (size_t)C * 9 * C;
    const int t = nd->t;
    if (m->arity[t] == 0) {                        /* SCENE: y = feat */
        for (size_t i = 0; i < n; ++i) dfeat[i] += dy[i];
        return;
    }
    double* g = (double*)malloc(n * sizeof(double));       /* through y = ReLU(s), s = u + conv_b(mid) + b_b */
    for (size_t i = 0; i < n; ++i) g[i] = nd->y[i] > 0.0 ? dy[i] : 0.0;
    double* dmid = (double*)malloc(n * sizeof(double));
    conv3x3_backward(g, nd->mid, m->w3b + t * w3, dmid, gr->dw3b + t * w3, gr->db3b + (size_t)t * C, C, m->H, m->W);
    for (size_t i = 0; i < n; ++i) if (!(nd->mid[i] > 0.0)) dmid[i] = 0.0;    /* mid = ReLU(conv_a(u) + b_a) */
    double* du = (double*)malloc(n * sizeof(double));
    conv3x3_backward(dmid, nd->u, m->w3a + t * w3, du, gr->dw3a + t * w3, gr->db3a + (size_t)t * C, C, m->H, m->W);
    for (size_t i = 0; i < n; ++i) du[i] += g[i];          /* the residual path: s = u + ... */
    free(g); free(dmid);
    if (m->arity[t] == 1) {
        bbwd(m, gr, nd->a, du, dfeat);
    } else {                                       /* u = ReLU(c), c[p][co] = b1[co] + sum_ci cat[p][ci] * w1[co][ci] */
        const float* w = m->w1 + (size_t)t * C * 2 * C;
        double* dw = gr->dw1 + (size_t)t * C * 2 * C;
        double* da = (double*)calloc(n, sizeof(double));
        double* dbm = (double*)calloc(n, sizeof(double));
        for (size_t p = 0; p < P; ++p)
            for (int co = 0; co < C; ++co) {
                const double dc = nd->u[p * C + co] > 0.0 ? du[p * C + co] : 0.0;
                gr->db1[(size_t)t * C + co] += dc;
                for (int ci = 0; ci < C; ++ci) {
                    dw[(size_t)co * 2 * C + ci] += dc * nd->a->y[p * C + ci];
                    da[p * C + ci] += dc * (double)w[(size_t)co * 2 * C + ci];
                    dw[(size_t)co * 2 * C + C + ci] += dc * nd->b->y[p * C + ci];
                    dbm[p * C + ci] += dc * (double)w[(size_t)co * 2 * C + C + ci];
                }
            }
        bbwd(m, gr, nd->a, da, dfeat);
        bbwd(m, gr, nd->b, dbm, dfeat);
        free(da); free(dbm);
    }
    free(du);
}

/* Programs must be well formed.  dout: float [B,H,W,C].  Outputs (double, overwritten): dfeats [B,H,W,C] and the
 * parameter gradients in the shapes of the parameters; dw1/db1 may be NULL if no function is binary; roots
 * (may be NULL) receives the root maps of the forward evaluation the gradients belong to. */
int oracle_iep_backward(const int32_t* prog, const int32_t* prog_off, int32_t B, const uint8_t* arity,
                        int32_t n_types, int32_t C, int32_t H, int32_t W, const float* feats,
                        const float* w1, const float* b1, const float* w3a, const float* b3a,
                        const float* w3b, const float* b3b, const float* dout, int32_t round_bf16, double* dfeats,
                        double* dw1, double* db1, double* dw3a, double* db3a, double* dw3b, double* db3b, double* roots)
{
    if (!prog || !prog_off || B <= 0 || !feats || !dout || !dfeats || !w3a || !w3b || !dw3a || !db3a || !dw3b || !db3b)
        return ORC_E_INVAL;
    modules m = { C, H, W, n_types, arity, w1, b1, w3a, b3a, w3b, b3b };
    const size_t n = (size_t)H * W * C, s3 = (size_t)n_types * C * 9 * C, s1 = (size_t)n_types * C * 2 * C, sb = (size_t)n_types * C;
    memset(dfeats, 0, sizeof(double) * n * B);
    memset(dw3a, 0, sizeof(double) * s3); memset(dw3b, 0, sizeof(double) * s3);
    memset(db3a, 0, sizeof(double) * sb); memset(db3b, 0, sizeof(double) * sb);
    if (dw1) memset(dw1, 0, sizeof(double) * s1);
    if (db1) memset(db1, 0, sizeof(double) * sb);
#pragma omp parallel
    {
        g_round_bf16 = round_bf16;
        grads gr;                                   /* this thread's sums, added to the result at the end */
        gr.dw3a = (double*)calloc(s3, sizeof(double)); gr.dw3b = (double*)calloc(s3, sizeof(double));
        gr.db3a = (double*)calloc(sb, sizeof(double)); gr.db3b = (double*)calloc(sb, sizeof(double));
        gr.dw1 = (double*)calloc(s1, sizeof(double)); gr.db1 = (double*)calloc(sb, sizeof(double));
#pragma omp for schedule(dynamic, 1)
        for (int32_t i = 0; i < B; ++i) {
            int32_t pos = prog_off[i];
            bnode* root = bfwd(&m, prog, &pos, feats + (size_t)i * n);
            if (roots) memcpy(roots + (size_t)i * n, root->y, n * sizeof(double));
            double* dy = (double*)malloc(n * sizeof(double));
            for (size_t e = 0; e < n; ++e) dy[e] = (double)dout[(size_t)i * n + e];
            bbwd(&m, &gr, root, dy, dfeats + (size_t)i * n);
            free(dy);
            bfree(&m, root);
        }
#pragma omp critical
        {
            for (size_t e = 0; e < s3; ++e) { dw3a[e] += gr.dw3a[e]; dw3b[e] += gr.dw3b[e]; }
            for (size_t e = 0; e < sb; ++e) { db3a[e] += gr.db3a[e]; db3b[e] += gr.db3b[e]; }
            if (dw1) for (size_t e = 0; e < s1; ++e) dw1[e] += gr.dw1[e];
            if (db1) for (size_t e = 0; e < sb; ++e) db1[e] += gr.db1[e];
        }
        free(gr.dw3a); free(gr.dw3b); free(gr.db3a); free(gr.db3b); free(gr.dw1); free(gr.db1);
    }
    return ORC_OK;
}
