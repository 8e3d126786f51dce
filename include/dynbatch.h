/*
 * dynbatch — dynamic batching of per-example dynamic architectures on one AMD MI355X (gfx950).
 *
 * C ABI of the library.  Two paths, both from "Effective Approaches to Batch Parallelization for
 * Dynamic Neural Network Architectures" (Suarez & Zhu):
 *
 *   1. Program-tree execution engine (Background / Visual Reasoning Programs; Methods):
 *      dynbatch_plan()    host  — prefix programs + arities -> trees -> labels -> pools with
 *                                 gather/scatter index lists
 *      dynbatch_plan_dag() host — the same for dependency graphs whose nodes may have several
 *                                 consumers (Discussion)
 *      dynbatch_execute() GPU   — runs the pools: gather the arguments, one batched residual
 *                                 conv module per pool, scatter the results; root maps come back
 *   2. Sparsely gated mixture of experts (Results / Sparsely Gated Mixture of Experts):
 *      moe_forward()      GPU   — noisy top-k gate, grouping of the k*b known expert uses by
 *                                 expert, one grouped FFN per expert, weighted combine
 *
 * Conventions
 *   - Every function returns DYNB_OK (0) or a negative DYNB_E_* code; dynb_last_error() gives a
 *     thread-local, library-owned message for the last failure on the calling thread.
 *   - "host" / "device" in a parameter comment says where the memory must live.  All pointers are
 *     borrowed: the library never frees or keeps caller memory beyond what is stated, and never
 *     allocates device memory — the caller brings workspaces.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  GPU entry points
 *     only enqueue work on it; they do not synchronise.
 *   - Feature maps are [H][W][C] (channels innermost).  Conv weights are [Cout][kh][kw][Cin].
 *   - DYNB_BF16 tensors hold bfloat16 bit patterns (uint16_t); accumulation is always fp32.
 */
#ifndef DYNBATCH_H
#define DYNBATCH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    DYNB_OK = 0,
    DYNB_E_INVAL = -1,        /* NULL pointer, non-positive size, k > E, ...                    */
    DYNB_E_MALFORMED = -2,    /* a program is not a complete prefix tree                        */
    DYNB_E_NOMEM = -3,        /* host allocation failed                                         */
    DYNB_E_WORKSPACE = -4,    /* a caller-provided buffer is too small / plan not uploaded      */
    DYNB_E_UNSUPPORTED = -5,  /* arity > 2, unknown dtype or flag, shape beyond kernel limits   */
    DYNB_E_HIP = -6           /* a HIP runtime call failed                                      */
};

enum { DYNB_F32 = 0, DYNB_BF16 = 1 };

/* Scheduling modes for dynbatch_plan (flags & DYNB_SCHED_MASK). */
enum {
    /* Methods / "Improved topological sort": label = distance from the root, equal labels are
     * pooled over the whole minibatch and pools run deepest label first.                        */
    DYNB_SCHED_IMPROVED = 0,
    /* Methods / "Standard topological sort": each program is flattened into a queue that lists
     * every node after its arguments; the minibatch is a b x s grid run column by column.      */
    DYNB_SCHED_STANDARD = 1,
    /* Results / IEP, the unbatched original: an explicit loop over examples, one module per
     * call.  Same kernels, one launch per node; the comparison row for the speed-up.           */
    DYNB_SCHED_NAIVE = 2,
    /* Discussion / batching "by dependency depth" (the TensorFlow Fold scheme the paper compares
     * with): label = 0 for argument-free nodes, else one more than the deepest argument; equal
     * labels are pooled over the minibatch and pools run in ascending label order.  Same number
     * of labels as DYNB_SCHED_IMPROVED; every node runs as early as its arguments allow.        */
    DYNB_SCHED_DEPTH = 3,
    DYNB_SCHED_MASK = 3,
    /* Optional, with DYNB_SCHED_IMPROVED only (ignored otherwise): balance the launch groups.  The
     * label of a node is the latest group it can run in; nodes whose arguments are ready earlier are
     * pulled forward out of groups wider than the chip's 256 CUs into earlier groups with idle CUs
     * (the Discussion notes that the order of dependency execution could be optimised and does
     * not pursue it).  The logical plan (labels, pools)
     * is unchanged; only node_launch and the executor's work lists differ.                       */
    DYNB_PLAN_BALANCE = 4,
    /* Optional, any scheduling mode: the caller keeps several independent batches in flight (one
     * HIP stream and workspace each) and wants chip throughput rather than the latency of one
     * batch.  dynbatch_execute then always uses the kernel layout with the most work per CU (one
     * node per workgroup, two workgroups sharing a CU) instead of spreading narrow launch groups
     * over idle CUs; kernels of the batches in flight fill the chip together.  Results are
     * bit-identical either way.                                                                 */
    DYNB_PLAN_THROUGHPUT = 8,
    /* Optional, any scheduling mode but DYNB_SCHED_NAIVE (ignored there): dynbatch_execute issues ONE
     * launch for the whole minibatch instead of one per label (Results / IEP expects the stacking and
     * calling overhead to be reducible further).  Resident workgroups claim units of work (a node, or the
     * upper / lower half of a node for labels that would leave half of the chip idle) in the plan's
     * execution order from one device counter and wait, with a bounded spin, until the arguments'
     * results have been published; a label no longer ends with the whole chip draining.  Arguments
     * always precede their consumer in the claim order and a claimed unit belongs to a workgroup that
     * is already running, so the waits always end.  Implies the grouping of DYNB_PLAN_BALANCE; every
     * node gets a result slot of its own (larger workspace).  Only the fast path (bf16, C = 128,
     * 14 x 14) has this kernel; other shapes run one launch per label as usual.  Results are
     * bit-identical either way.  See dynbatch_execute_check for the bounded waits.                 */
    DYNB_PLAN_PERSISTENT = 16,
    /* Optional, any scheduling mode: keep every node's result (a slot of its own in the workspace, no
     * reuse) so that dynbatch_backward can run after dynbatch_execute.  On the fast path (bf16, C = 128,
     * 14 x 14) dynbatch_execute also saves the two intermediate maps of every node (the output of the 1x1
     * convolution of two-argument functions and of the first 3x3 convolution) in the workspace, and a plan
     * that also carries DYNB_PLAN_PERSISTENT runs one launch per label.  Larger workspace (three maps per
     * node).  The plan view then lists the tables the backward pass works from.                     */
    DYNB_PLAN_KEEP = 32
};

const char* dynb_last_error(void);

/* ------------------------------------------------------------------------------------------- */
/* Planner (host only; no GPU needed)                                                           */
/* ------------------------------------------------------------------------------------------- */

typedef struct dynb_plan dynb_plan;

/* Logical plan, independent of how the executor lays out memory.  Node id = prog_off[example] +
 * position in that example's prefix sequence.  Pools ("buckets") are listed in execution order:
 * IMPROVED — label descending, then function id ascending; STANDARD — column ascending, then
 * function id ascending; DEPTH — label ascending, then function id ascending; NAIVE — one bucket
 * per node, example by example in queue order.
 * Members of a bucket are ascending node ids.  in0/in1 are the node ids of the members'
 * arguments (-1 if absent), out is the member itself.  SCENE buckets (arity 0) are listed but
 * cost no network call.  All arrays are owned by the plan and valid until dynbatch_plan_free. */
typedef struct {
    int32_t n_examples;
    int32_t n_nodes;
    int32_t n_levels;         /* number of distinct labels = 1 + max label over the minibatch   */
    int32_t n_buckets;
    int32_t n_compute_nodes;  /* nodes with arity > 0 = module evaluations                      */
    int32_t n_launches;       /* kernel launch groups dynbatch_execute will issue               */
    int32_t max_launch_nodes; /* largest number of compute nodes in one launch group            */
    int32_t n_slots;          /* feature-map slots the executor needs in its workspace          */
    const int32_t* node_level;   /* [n_nodes] label                                             */
    const int32_t* node_type;    /* [n_nodes]                                                   */
    const int32_t* child0;       /* [n_nodes] first argument or -1                              */
    const int32_t* child1;       /* [n_nodes] second argument or -1                             */
    const int32_t* root;         /* [n_examples]                                                */
    const int32_t* bucket_level; /* [n_buckets]                                                 */
    const int32_t* bucket_type;  /* [n_buckets]                                                 */
    const int32_t* bucket_start; /* [n_buckets] offset into members/in0/in1/out                 */
    const int32_t* bucket_count; /* [n_buckets]                                                 */
    const int32_t* members;      /* [n_nodes]                                                   */
    const int32_t* in0;          /* [n_nodes]                                                   */
    const int32_t* in1;          /* [n_nodes]                                                   */
    const int32_t* out;          /* [n_nodes]                                                   */
    const int32_t* node_launch;  /* [n_nodes] launch group that executes the node, -1 for SCENE   */
    const int32_t* item_node;    /* [n_compute_nodes] node evaluated by every work item, in execution
                                    order                                                        */
    int32_t n_tickets;           /* DYNB_PLAN_PERSISTENT: units of work of the single launch, else 0 */
    const int32_t* tickets;      /* [n_tickets] in claim order: 4 * item + part; part 0 = the whole
                                    node, 1 / 2 = its upper / lower half                         */
    /* DYNB_PLAN_KEEP: what the backward pass works from (NULL / 0 otherwise).                     */
    const int32_t* grad_dst0;    /* [n_compute_nodes] where the gradient of an item's first argument goes:
                                    >= 0 the item that evaluates the argument, -1 - l the SCENE leaf number l
                                    (leaves are numbered example by example in node order)         */
    const int32_t* grad_dst1;    /* [n_compute_nodes] same for the second argument (0 if there is none) */
    const int32_t* fn_first;     /* [n_types + 1] the items of function t are fn_items[fn_first[t] ..
                                    fn_first[t+1]), ascending                                      */
    const int32_t* fn_items;     /* [n_compute_nodes]                                             */
    int32_t n_types;
    int32_t n_wg_units;          /* units of work of the parameter-gradient kernel                */
    const int32_t* wg_units;     /* [n_wg_units][8]: mode (0 second conv3x3, 1 first conv3x3, 2 conv1x1),
                                    function, part (kernel row, or argument for mode 2), begin, end (a chunk
                                    fn_items[begin .. end) of at most 16 items), 3 unused            */
    const int32_t* wg_order;     /* [n_wg_units] unit taken by every workgroup of that kernel     */
} dynb_plan_view;

/* Builds the plan for a minibatch of programs (Background / Visual Reasoning Programs: the fixed
 * arities make the tree unique, it is assembled depth first; Methods: labelling and pooling).
 *   prog      host  concatenated prefix sequences of function ids
 *   prog_off  host  [B+1], prog_off[0] = 0, example i owns prog[prog_off[i] .. prog_off[i+1])
 *   arity     host  [n_types] values 0, 1 or 2; any id with arity 0 is a SCENE-like leaf that
 *                   outputs the example's feature map
 *   flags     one DYNB_SCHED_* value, optionally | DYNB_PLAN_BALANCE | DYNB_PLAN_THROUGHPUT
 *   out       receives a library-owned plan; release with dynbatch_plan_free
 * Errors: DYNB_E_INVAL (NULL, B <= 0, n_types <= 0, offsets not increasing from 0),
 * DYNB_E_UNSUPPORTED (arity > 2, unknown flag), DYNB_E_MALFORMED (function id out of range, a
 * sequence that ends before its tree is complete or has tokens left over, an empty sequence;
 * the message names the first offending example), DYNB_E_NOMEM.  On error *out is NULL.         */
int dynbatch_plan(const int32_t* prog, const int32_t* prog_off, int32_t B, const uint8_t* arity,
                  int32_t n_types, uint32_t flags, dynb_plan** out);

/* The same for architectures given as general dependency graphs (Discussion: any architecture
 * whose dependencies are known before execution; a node may have several consumers and is
 * evaluated once).  Example i owns nodes [node_off[i], node_off[i+1]) in any order.
 *   type      host  [N]   function id of every node
 *   arg0/1    host  [N]   index INSIDE the example of the node that produces the first / second
 *                         argument, -1 if the function takes none; arg1 >= 0 requires arg0 >= 0
 *   node_off  host  [B+1] node_off[0] = 0
 *   root      host  [B]   index inside the example of the node whose map is the example's output
 *   flags     DYNB_SCHED_IMPROVED (label = MAXIMUM distance from the root, Methods / Improved
 *             topological sort) or DYNB_SCHED_DEPTH, optionally | DYNB_PLAN_THROUGHPUT;
 *             DYNB_PLAN_BALANCE is accepted and ignored
 * The plan behaves like one from dynbatch_plan (view, upload, execute, free); in its view node id
 * = node_off[example] + index and child0/child1 are the arguments' node ids.
 * Errors as dynbatch_plan; DYNB_E_MALFORMED also for an argument index out of range, an argument
 * count that differs from the arity, a cycle, a root out of range, or a node that the root does
 * not depend on; DYNB_E_UNSUPPORTED for the standard and naive schedules.                       */
int dynbatch_plan_dag(const int32_t* type, const int32_t* arg0, const int32_t* arg1,
                      const int32_t* node_off, const int32_t* root, int32_t B, const uint8_t* arity,
                      int32_t n_types, uint32_t flags, dynb_plan** out);

int dynbatch_plan_view(const dynb_plan* plan, dynb_plan_view* view);

void dynbatch_plan_free(dynb_plan* plan);

/* Bytes of device memory the plan's index lists need. */
size_t dynbatch_plan_device_bytes(const dynb_plan* plan);

/* Copies the index lists (and, for DYNB_PLAN_KEEP plans, the backward pass's tables) to `dev_buf` (device,
 * >= dynbatch_plan_device_bytes, 16-byte aligned) on `stream` with one copy, once per plan.  The plan
 * remembers dev_buf; it must stay valid and unmodified while the plan is executed.  The copy reads a host
 * image that the plan owns: do not free the plan, or upload it again, before the work enqueued on
 * `stream` up to this call has finished.
 * Errors: DYNB_E_INVAL, DYNB_E_WORKSPACE (too small), DYNB_E_HIP.                               */
int dynbatch_plan_upload(dynb_plan* plan, void* dev_buf, size_t bytes, void* stream);

/* ------------------------------------------------------------------------------------------- */
/* Executor                                                                                      */
/* ------------------------------------------------------------------------------------------- */

typedef struct {
    int32_t C, H, W;
    int32_t dtype;            /* DYNB_F32 or DYNB_BF16: element type of feats, out, workspace
                                 slots and conv weights                                         */
} dynb_shape;

/* Per-function parameters, one block per function id (blocks of SCENE ids are never read).
 * Unary function t:  y = ReLU(u + conv3x3_b(ReLU(conv3x3_a(u) + b3a)) + b3b),  u = its argument.
 * Binary function t: same with u = ReLU(conv1x1(concat_C(arg0, arg1)) + b1); the first argument
 * feeds input channels [0,C).  Convolutions are cross-correlations, stride 1, zero padding 1.   */
typedef struct {
    const void* w1;           /* device [n_types][C][2C]        dtype; may be NULL if no binary  */
    const float* b1;          /* device [n_types][C]            fp32;  NULL = no bias            */
    const void* w3a;          /* device [n_types][C][3][3][C]   dtype                            */
    const float* b3a;         /* device [n_types][C]            fp32;  NULL = no bias            */
    const void* w3b;          /* device [n_types][C][3][3][C]   dtype                            */
    const float* b3b;         /* device [n_types][C]            fp32;  NULL = no bias            */
    const void* packed;       /* device, optional: the three weight tensors in the fast path's
                                 MFMA fragment order, written by dynbatch_pack_weights for the same
                                 n_types and shape.  NULL: dynbatch_execute repacks w1, w3a, w3b into
                                 its workspace on every call (about 20 us for 41 functions).
                                 Ignored by shapes without a fast path.  The caller keeps it in
                                 step with the weights: repack after they change.               */
} dynb_module_weights;

/* Bytes of the packed copy for n_types functions (0 if the shape has no fast path or on bad input). */
size_t dynbatch_packed_weights_bytes(const dynb_shape* shape, int32_t n_types);

/* One-time preparation of constant weights (the paper's modules are fixed at inference time):
 * writes w->w1 (if not NULL), w->w3a and w->w3b in fragment order into `packed`, asynchronously on
 * `stream`.  Biases are not part of the packed copy.
 *   packed   device, >= dynbatch_packed_weights_bytes, 256-byte aligned, caller-owned
 * Errors: DYNB_E_INVAL (NULL, n_types <= 0, misaligned), DYNB_E_UNSUPPORTED (shape without a fast
 * path), DYNB_E_WORKSPACE (too small), DYNB_E_HIP.                                              */
int dynbatch_pack_weights(const dynb_shape* shape, int32_t n_types, const dynb_module_weights* w,
                          void* packed, size_t packed_bytes, void* stream);

/* Bytes of device workspace dynbatch_execute needs for this plan and shape (0 on bad input).   */
size_t dynbatch_workspace_bytes(const dynb_plan* plan, const dynb_shape* shape);

/* Executes the plan (Methods: each pool is run at once, one batched network call per function;
 * Results / IEP: the "data stacking" that builds a pool's batch and returns its results is part
 * of this call).  One launch group per label; inside it every workgroup looks up its node's
 * function and parameter block.
 *   feats      device [B][H][W][C]  the SCENE output of each example
 *   out        device [B][H][W][C]  receives each example's root map
 *   workspace  device, >= dynbatch_workspace_bytes, 256-byte aligned; contents are scratch, and
 *              nothing else may read or write it until the call's work on `stream` has finished
 *              (calls in flight on different streams need a workspace each)
 * The fast path (bf16, C = 128, 14 x 14) runs fused MFMA kernels; every other shape runs generic
 * kernels with the same semantics.  Errors: DYNB_E_INVAL, DYNB_E_WORKSPACE (workspace too small
 * or plan not uploaded), DYNB_E_UNSUPPORTED (dtype; w1 NULL with binary functions), DYNB_E_HIP. */
int dynbatch_execute(const dynb_plan* plan, const dynb_shape* shape, const dynb_module_weights* w,
                     const void* feats, void* out, void* workspace, size_t workspace_bytes,
                     void* stream);

/* After a dynbatch_execute of a DYNB_PLAN_PERSISTENT plan on the fast path: waits for `stream`,
 * then reads the status word that call left in `workspace`.  DYNB_OK; DYNB_E_HIP if a workgroup's
 * bounded wait for an argument expired (the kernel then drains without computing and `out` is
 * invalid: with a correct plan this means the device was not making progress); DYNB_E_INVAL for
 * NULL arguments or a plan that is not DYNB_PLAN_PERSISTENT.                                     */
int dynbatch_execute_check(const dynb_plan* plan, const dynb_shape* shape, const void* workspace, void* stream);

/* Polls a workgroup makes before it gives up waiting for an argument (default 1 << 22, about a
 * second); 0 makes a workgroup give up at once if an argument is not ready.  Process-wide; for tests
 * of the error path.  Returns the previous value.                                               */
int32_t dynb_set_spin_limit(int32_t polls);

/* ------------------------------------------------------------------------------------------- */
/* Backward pass of an executed plan                                                             */
/* ------------------------------------------------------------------------------------------- */

/* Gradients, all device fp32, in the shapes of the tensors they belong to; overwritten by the call. */
typedef struct {
    float* dfeats;            /* [B][H][W][C]            gradient of every example's input feature map */
    float* dw1;               /* [n_types][C][2C]        may be NULL if no function takes two arguments */
    float* db1;               /* [n_types][C]            may be NULL if no function takes two arguments */
    float* dw3a;              /* [n_types][C][3][3][C]                                                 */
    float* db3a;              /* [n_types][C]                                                          */
    float* dw3b;              /* [n_types][C][3][3][C]                                                 */
    float* db3b;              /* [n_types][C]                                                          */
} dynb_module_grads;

/* Bytes of device workspace dynbatch_backward needs (0 on bad input or a plan without DYNB_PLAN_KEEP). */
size_t dynbatch_backward_workspace_bytes(const dynb_plan* plan, const dynb_shape* shape);

/* Backward pass of the programs a dynbatch_execute call ran (Results / IEP times it beside inference; the
 * batching is the same: the plan's launch groups in reverse order, parameter gradients summed pool by pool).
 * With dout[i] = dL/d(root map of example i) for some scalar loss L it writes dL/d(feature maps) and
 * dL/d(every module parameter), the latter summed over all nodes that use the function.
 *   plan               made with DYNB_PLAN_KEEP by dynbatch_plan (not dynbatch_plan_dag), uploaded
 *   w, feats           as passed to dynbatch_execute (w->packed is not used)
 *   out                device [B][H][W][C] dtype: what dynbatch_execute wrote
 *   forward_workspace  device: the workspace of that dynbatch_execute call, unchanged since
 *   dout               device [B][H][W][C] fp32
 *   grads              host struct of device pointers
 *   workspace          device, >= dynbatch_backward_workspace_bytes, 256-byte aligned, scratch
 * Any shape and both dtypes.  bf16 with C = 128 and 14 x 14 maps (the shape of the fused forward kernels) runs on
 * MFMAs: gradients travel between nodes as fp32 maps and enter the contractions rounded to bf16, like every other
 * operand of that path.  Other shapes run plain FMA kernels (one thread per output element, fp32 gradients
 * throughout).  Every sum has a fixed order, so two calls give the same bits.  Errors: DYNB_E_INVAL, DYNB_E_WORKSPACE (too small, plan
 * not uploaded), DYNB_E_UNSUPPORTED (plan without DYNB_PLAN_KEEP, dependency graphs, dtype), DYNB_E_HIP. */
int dynbatch_backward(const dynb_plan* plan, const dynb_shape* shape, const dynb_module_weights* w, const void* feats,
                      const void* out, const void* forward_workspace, const float* dout, const dynb_module_grads* grads,
                      void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------- */
/* Classifier head                                                                               */
/* ------------------------------------------------------------------------------------------- */

/* Background / Visual Reasoning Programs: the output of the executed program passes through a small
 * classifier, one convolutional and two fully connected layers, that yields a softmax distribution
 * over the answers.  The paper gives neither sizes nor the kernel shape; this library takes
 *   z  = ReLU(conv1x1_{C -> Cc}(root) + bc)         per pixel
 *   h1 = ReLU(wf1 . flatten(z) + bf1)               flatten in [H][W][Cc] order, F units
 *   p  = softmax(wf2 . h1 + bf2)                    n_answers entries                           */
typedef struct {
    int32_t C, H, W;
    int32_t dtype;            /* DYNB_F32 or DYNB_BF16: element type of the root maps and the three
                                 weight tensors (z and h1 are kept in it too); sums are fp32    */
    int32_t Cc;               /* channels after the convolution                                  */
    int32_t F;                /* units of the first fully connected layer                        */
    int32_t n_answers;
} dynb_head_shape;

typedef struct {
    const void* wc;           /* device [Cc][C]             dtype                                 */
    const float* bc;          /* device [Cc]                fp32; NULL = no bias                  */
    const void* wf1;          /* device [F][H*W*Cc]         dtype                                 */
    const float* bf1;         /* device [F]                 fp32; NULL = no bias                  */
    const void* wf2;          /* device [n_answers][F]      dtype                                 */
    const float* bf2;         /* device [n_answers]         fp32; NULL = no bias                  */
} dynb_head_weights;

/* Bytes of device workspace dynbatch_classify needs for B root maps (0 on bad input). */
size_t dynbatch_classify_workspace_bytes(const dynb_head_shape* shape, int32_t B);

/* Runs the classifier on B root maps, asynchronously on `stream`.
 *   roots      device [B][H][W][C] dtype: what dynbatch_execute wrote to its `out`
 *   probs      device [B][n_answers] fp32
 *   logits     device [B][n_answers] fp32 or NULL: the inputs of the softmax, if wanted
 *   workspace  device, >= dynbatch_classify_workspace_bytes, 256-byte aligned, scratch
 * Any sizes are accepted; bf16 layers whose inner extent (C, H*W*Cc, F) is a multiple of 8 run on
 * MFMAs, the others on plain FMAs.  B = 0 succeeds without work.  Errors: DYNB_E_INVAL (NULL,
 * sizes <= 0, misaligned), DYNB_E_WORKSPACE, DYNB_E_UNSUPPORTED (dtype, batch too large), DYNB_E_HIP. */
int dynbatch_classify(const dynb_head_shape* shape, const dynb_head_weights* w, const void* roots, int32_t B,
                      float* probs, float* logits, void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------- */
/* Mixture of experts                                                                            */
/* ------------------------------------------------------------------------------------------- */

typedef struct {
    int32_t T;                /* tokens (the paper's b)                                         */
    int32_t d;                /* model width                                                    */
    int32_t h;                /* hidden units per expert                                        */
    int32_t E;                /* experts (the paper's n)                                        */
    int32_t k;                /* experts per token, 1 <= k <= E                                 */
    int32_t dtype;            /* DYNB_BF16 only                                                 */
    uint32_t flags;           /* 0, or MOE_SEPARATE_PERMUTE                                     */
} moe_shape;

/* moe_shape.flags.  By default the stacking of the tokens by expert (Results / Sparsely Gated Mixture
 * of Experts counts it as "data stacking" next to the expert calls) happens inside the first expert
 * layer's operand load: the permuted copy of x is never written.  With MOE_SEPARATE_PERMUTE it is a
 * kernel of its own that writes the copy (an HBM-bound scatter that can be timed and profiled alone);
 * the results are bit-identical.                                                                   */
enum { MOE_SEPARATE_PERMUTE = 1 };

/* Optional outputs of the routing stages; any pointer may be NULL.  All device memory.          */
typedef struct {
    float* logits;            /* [T][E]                                                         */
    int32_t* topk_idx;        /* [T][k]  descending logit, equal logits -> lower expert first   */
    float* topk_w;            /* [T][k]  softmax over the k kept logits                         */
    int32_t* counts;          /* [E]                                                            */
    int32_t* offsets;         /* [E+1]   exclusive prefix sum of counts                         */
    int32_t* perm;            /* [T*k]   sorted position -> flat use id a = t*k + j             */
    int32_t* inv;             /* [T*k]   flat use id -> sorted position                         */
} moe_aux;

size_t moe_workspace_bytes(const moe_shape* shape);

/* One sparsely gated MoE layer (Results / Sparsely Gated Mixture of Experts: the k*b known expert
 * uses are grouped so that only n expert calls are made; experts are one-hidden-layer networks
 * without biases, 2*h*n*d parameters in all).
 *   logit[t][e] = x_t . Wg[e] + noise[t][e] * softplus(x_t . Wn[e])
 *   keep the k largest logits per token, softmax over them
 *   group the uses by expert with a stable counting sort (order inside a group = ascending t*k+j)
 *   y = ReLU(xs . W1_e^T) . W2_e^T for each group; out_t = sum_j w[t][j] * y[use (t,j)]
 *   x      device [T][d]      bf16
 *   Wg,Wn  device [E][d]      bf16   (row e is expert e's gate vector; Wn may be NULL iff noise is)
 *   noise  device [T][E]      fp32 or NULL (noiseless gate)
 *   W1     device [E][h][d]   bf16   (row j of W1_e produces hidden unit j)
 *   W2     device [E][d][h]   bf16   (row c of W2_e produces output channel c)
 *   out    device [T][d]      bf16
 *   aux    host struct of device pointers, or NULL
 *   workspace device, >= moe_workspace_bytes, 256-byte aligned; it holds the routing tables of the
 *             call, so nothing else may write it until the call's work on `stream` has finished
 *             (calls in flight on different streams need a workspace each)
 * T = 0 succeeds without work.  Errors: DYNB_E_INVAL (NULL, k > E, sizes <= 0), DYNB_E_WORKSPACE,
 * DYNB_E_UNSUPPORTED (dtype; d or h not a multiple of 8: rows move in 16-byte pieces; more than
 * 2^30 expert uses), DYNB_E_HIP.  All shape errors are reported before any work is enqueued.      */
int moe_forward(const moe_shape* shape, const void* x, const void* Wg, const void* Wn,
                const float* noise, const void* W1, const void* W2, void* out, const moe_aux* aux,
                void* workspace, size_t workspace_bytes, void* stream);

/* moe_forward for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): same layer, same kernels, same results, but no
 * workspace argument.  The routing tables and the permuted / hidden / expert-output rows live in a
 * device array of MOE_STATIC_SCRATCH_BYTES that is part of the library's code object (each GPU the
 * library runs on holds it until the process ends).  The call allocates nothing and frees nothing.
 *   other arguments as moe_forward (aux pointers, if given, are still the caller's memory)
 * All calls on one GPU share that GPU's array: calls that overlap on one GPU (different streams or
 * threads) race on it; issue them on one stream or serialise them.  Nothing is kept between calls.
 * Errors as moe_forward; DYNB_E_WORKSPACE if moe_workspace_bytes(shape) exceeds
 * MOE_STATIC_SCRATCH_BYTES (the 4096-token, 256-expert benchmark layer needs 38 MB and fits; the
 * 16384-token, 1024-expert one needs 607 MB and does not: use moe_forward for it).               */
#define MOE_STATIC_SCRATCH_BYTES (48u << 20)
int moe_forward_static(const moe_shape* shape, const void* x, const void* Wg, const void* Wn,
                       const float* noise, const void* W1, const void* W2, void* out, const moe_aux* aux,
                       void* stream);

/* The unbatched comparison row of Results / Sparsely Gated Mixture of Experts (the naive version
 * there runs each of the k*b expert uses on its own, in a loop): gate, top-k, grouping and
 * permute as in moe_forward, then one expert call (both layers, same kernels, one row) per use,
 * issued from a host loop, then combine.  Synchronises the stream once to read the group sizes.
 *   use_stride  >= 1; 1 executes every use and gives the same `out` as moe_forward; a larger
 *               value executes only every use_stride-th use (a timing sample: `out` is then
 *               not meaningful).
 * Other arguments and errors as moe_forward; DYNB_E_INVAL for use_stride < 1.                     */
int moe_forward_naive(const moe_shape* shape, const void* x, const void* Wg, const void* Wn,
                      const float* noise, const void* W1, const void* W2, void* out,
                      const moe_aux* aux, void* workspace, size_t workspace_bytes, void* stream,
                      int32_t use_stride);

/* ------------------------------------------------------------------------------------------- */
/* Per-stage timing (the paper reports "neural cell execution time" and "data stacking" apart   */
/* from the whole forward pass: Results / IEP, Results / Sparsely Gated Mixture of Experts)      */
/* ------------------------------------------------------------------------------------------- */

typedef struct {
    int32_t tag;    /* dynbatch_execute: index of the launch group, -2 for set-up; moe_forward: stage id
                       0 gate, 1 top-k, 2 grouping (counting sort), 3 permute, 4 expert layer 1,
                       5 expert layer 2, 6 combine                                               */
    int32_t units;  /* dynbatch_execute: module evaluations in the launch group; moe_forward: 0   */
    float ms;       /* GPU time between the HIP events that bracket the stage                    */
} dynb_stage_time;

/* Switches event recording for the calling thread: 0 off (the default), 1 one HIP event per
 * launch group (dynbatch_execute) or stage (moe_forward) on the caller's stream, 2 as 1 for
 * moe_forward but a single pair of events around all launch groups of dynbatch_execute (one
 * stage, tag 0, units = all module evaluations), which keeps the event records themselves out of
 * the measured interval.  In both modes dynbatch_execute first reports its set-up work (weight
 * repacking, copies of single-leaf programs) as a stage with tag -2.  An event costs a few
 * microseconds, so leave timing off when measuring throughput.  Errors: DYNB_E_INVAL.           */
int dynb_timing_enable(int on);

/* Waits for the last timed call of this thread to finish on the GPU and returns its stages.
 *   out       host [capacity]
 *   n_out     host, receives the number of stages of the call (may exceed capacity)
 * Errors: DYNB_E_INVAL, DYNB_E_HIP.                                                             */
int dynb_timing_read(dynb_stage_time* out, int32_t capacity, int32_t* n_out);

/* ------------------------------------------------------------------------------------------- */
/* Measurement helpers: what the card sustains, from the simplest possible kernels.  Not part of */
/* the method; a benchmark reports these next to the published peaks and times them itself       */
/* (events on `stream`).                                                                         */
/* ------------------------------------------------------------------------------------------- */

/* Enqueues a register-only loop of independent 32x32x16 bf16 MFMAs: `workgroups` workgroups of four
 * waves, `iters` x 8 MFMAs per wave, no memory traffic.
 *   sink   device, one float (written only if an impossible sum comes out: keeps the loop alive)
 *   flops  host, receives the flop count of the launch (2 * 32 * 32 * 16 per MFMA)
 * Errors: DYNB_E_INVAL, DYNB_E_HIP.                                                             */
int dynb_probe_mfma_bf16(int32_t iters, int32_t workgroups, float* sink, void* stream, double* flops);

/* Enqueues a plain copy kernel (16-byte loads and stores, grid-stride): `bytes` read + `bytes`
 * written.  dst, src device, 16-byte aligned, not overlapping; bytes a multiple of 16.
 * Errors: DYNB_E_INVAL, DYNB_E_HIP.                                                             */
int dynb_probe_copy(void* dst, const void* src, size_t bytes, void* stream);

/* Reads `bytes` of device memory with 16-byte loads, every workgroup a contiguous share of the buffer, and stores
 * nothing (`sink`: device, at least 4 bytes, practically never written): the bandwidth a kernel that only streams
 * operands in can expect at best.
 * Errors: DYNB_E_INVAL (NULL, size or pointer not a multiple of 16), DYNB_E_HIP.                          */
int dynb_probe_read(const void* src, size_t bytes, void* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DYNBATCH_H */
