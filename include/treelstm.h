/*
 * treelstm.h - batched forward evaluation of recursive tree networks on one AMD
 * MI355X (gfx950).  C ABI; every pointer is a plain pointer, marked below as HOST or
 * DEVICE memory.
 *
 * What is computed.  A batch of full binary trees is evaluated bottom-up: a leaf's
 * state comes from the embedding of its word, an internal node's state from the
 * states of its two children (the recursive definition of the paper's Figure 2).
 * A node's cell runs as soon as its children are done, so independent subtrees and
 * independent trees proceed concurrently (Section 4.1, "Recursive Execution": ready
 * queue fed by unresolved-input counters), instead of one node at a time in a
 * topologically sorted order (Figure 1).  The result is the same set of numbers
 * either way (Section 6.2, "Convergence").
 *
 * The paper names its cells (Section 6.1: TreeLSTM, TreeRNN, RNTN) without printing
 * them; this library uses the standard binary forms.  With s(t) = 1/(1+exp(-t)),
 * x = embedding row of a leaf's word, a = [h_left ; h_right] (length 2H):
 *
 *   TL_TREELSTM  leaf      [gi|go|gu] = x W_leaf + b_leaf         (each block H wide)
 *                          c = s(gi)*tanh(gu);  h = s(go)*tanh(c)
 *                internal  [gi|gfl|gfr|go|gu] = a U + b
 *                          c = s(gi)*tanh(gu) + s(gfl)*c_left + s(gfr)*c_right
 *                          h = s(go)*tanh(c)
 *   TL_TREERNN   leaf h = x (embed_dim == hidden);  internal h = tanh(a U + b)
 *   TL_RNTN      leaf h = x;  internal h_k = tanh(sum_pq a_p V[k][p][q] a_q + (a U)_k + b_k)
 *
 * Tree encoding (the paper's tree.children[idx] / tree.leaves[idx] index arrays of
 * Figures 1-2, flattened over the batch): tree t owns nodes tree_off[t] ..
 * tree_off[t+1]-1; left[n] / right[n] are GLOBAL node indices of n's children inside
 * the same tree, or -1 at a leaf; word[n] is the word id of a leaf (ignored at
 * internal nodes).  Nodes of a tree may be numbered in ANY order - no topological
 * sorting is required (Section 2.1 explains that only the iterative form needs it).
 * A single-node tree (the root is a leaf) is legal.
 *
 * Threading: a context is not thread safe; one forward may be in flight per context.
 * TL_SCHED_READY (also in its _PRIORITY variant, which is meant wherever TL_SCHED_READY is
 * named below), TL_SCHED_LEVEL_DEVICE and TL_SCHED_DATAFLOW evaluate the internal nodes in one
 * kernel whose workgroups wait for each other, so all of them must be resident together.
 * tl_forward sizes the grid to what the device holds of the very kernel it launches (asked of
 * the runtime per kernel variant) and returns TL_EHIP at once if not even one set of workgroups
 * fits; with the device to itself such a forward therefore always completes.  What the library
 * cannot see is other work on the device: while such a forward runs, nothing else that holds
 * compute units for long (another context's forward on a second stream, say) may run beside it.
 * Forwards of several contexts are therefore put on one stream or ordered with events (tested
 * with two contexts on two streams); breaking this does not hang - every wait is bounded by
 * spin_limit - but the forward may then end with TL_ESTALL.  TL_SCHED_LEVEL_HOST has no such
 * requirement.  The default of the ABI (scheduler = 0) is TL_SCHED_READY, the plainest device
 * form of the paper's mechanism; TL_SCHED_DATAFLOW is the fastest on every workload measured in
 * fp32, TL_SCHED_LEVEL_DEVICE on wide batches with bf16 operands.
 * Errors: functions return TL_OK (0) or a negative tl_error.
 */
#ifndef TREELSTM_H
#define TREELSTM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tl_ctx tl_ctx;

enum tl_cell { TL_TREELSTM = 0, TL_TREERNN = 1, TL_RNTN = 2 };

/* TL_F32: fp32 operands, fp32 accumulation.  TL_BF16_IN: weights, embeddings and the
 * gathered child h are rounded to bfloat16 (nearest even) as matrix operands;
 * accumulation, gate functions, c and the stored h stay fp32. */
enum tl_precision { TL_F32 = 0, TL_BF16_IN = 1 };

/* How internal nodes are scheduled (Section 4.1 versus the depth-wise batching that
 * Section 6.3, "Comparison with Folding", describes):
 *  TL_SCHED_READY        one persistent kernel; every node has a counter of unfinished
 *                        children; the workgroup that finishes the last child pushes the
 *                        parent on a device ready queue, from which tiles of ready nodes
 *                        are formed.  Needs no heights and no per-level barrier.
 *  TL_SCHED_LEVEL_DEVICE one persistent kernel walks the heights 1, 2, ... with a grid-wide
 *                        barrier between them; the frontier of the next height is built
 *                        from the same counters while the current one is evaluated (no
 *                        separate pass over the trees).
 *  TL_SCHED_LEVEL_HOST   node heights and per-height node lists are built on the device,
 *                        then one kernel launch per height from the host (which reads the
 *                        number of heights back first).  Comparison baseline.
 *  TL_SCHED_READY_PRIORITY  TL_SCHED_READY with the critical path first (what Section 4.1
 *                        leaves as future work: operations that many later ones wait for
 *                        should run before others that are ready).  The structure pass also
 *                        computes every node's distance from its root, i.e. the number of
 *                        dependent steps still above it (counted up to 128; two more small
 *                        launches).  A node is critical when that distance is at least 32
 *                        and at least four times the batch's mean.  Critical nodes that start ready go to the front of
 *                        the ready queue, and a critical parent that becomes ready is handed
 *                        straight back to the gang that finished its last child, as a small
 *                        tile of its own, instead of queueing behind the bulk of the batch;
 *                        that gang takes no other work while it holds such a chain.  Pays
 *                        when a few deep trees share a batch with much shallow work, costs
 *                        the extra launches otherwise.
 *  TL_SCHED_DATAFLOW     the ready counters of Section 4.1 with nothing shared between the
 *                        workers.  The trees are dealt to sets of workgroups (one workgroup per 16
 *                        hidden units) in contiguous ranges of about equal node count; every
 *                        workgroup keeps, for the trees of its set, its own counters of handed-out
 *                        children and its own list of ready nodes, so no queue, record, mailbox or
 *                        grid-wide barrier is exchanged about the schedule.  Whether a child's row
 *                        has been written is read off the row itself: the rows that internal nodes
 *                        will produce are filled with a bit pattern that no cell stores (all ones, a
 *                        NaN) before the kernel starts, and a consumer repeats its request while a
 *                        piece of the row still shows it.  A dependent step costs about one memory
 *                        round trip instead of an acknowledgement, a barrier and a queue read, so
 *                        this is the fastest choice for deep or narrow batches and as fast as
 *                        TL_SCHED_LEVEL_DEVICE on wide ones.  Consequence: if the parameters or
 *                        embeddings hold NaNs whose bits are all ones, a forward ends with
 *                        TL_ESTALL instead of NaN results.  Where the weight-stationary cell is not
 *                        used (TL_RNTN, hidden > 512, odd hidden in TL_F32, tl_forward_noalloc)
 *                        TL_SCHED_LEVEL_DEVICE stands in.  Whole trees are dealt to the sets, so a
 *                        batch of fewer trees than the device has sets leaves sets idle; if its trees
 *                        have 256 nodes or more on average, both this kernel and that of
 *                        TL_SCHED_LEVEL_DEVICE are launched and the device picks one by the width of
 *                        the first frontier (more than 16 ready nodes per tree: bushy trees, level by
 *                        level on all sets; otherwise deep narrow ones, data-flow).  A batch in which
 *                        one large bushy tree stands beside many small ones is better served by
 *                        TL_SCHED_LEVEL_DEVICE.  Unreachable nodes: TL_ESTRUCT.
 * Results do not depend on the scheduler: all paths of one precision sum a node's
 * contraction in the same order, so all of them agree bit for bit and repeat their bits from
 * run to run.  One exception: in TL_F32, TL_SCHED_DATAFLOW evaluates the dependent steps of few
 * rows (the last block of up to 12 rows of each piece of its lists) with a narrower matrix
 * instruction that rounds the same sum in another order; which nodes those are is fixed by the
 * batch, so it repeats its own bits from run to run and agrees with the other schedulers to
 * rounding (relative 2e-5 in the tests). */
enum tl_scheduler { TL_SCHED_READY = 0, TL_SCHED_LEVEL_DEVICE = 1, TL_SCHED_LEVEL_HOST = 2, TL_SCHED_READY_PRIORITY = 3,
                    TL_SCHED_DATAFLOW = 4 };

enum tl_error {
    TL_OK = 0,
    TL_EINVAL = -1,    /* null pointer, negative size, unsupported dimension or enum          */
    TL_ENOMEM = -2,    /* device or host allocation failed                                     */
    TL_EHIP = -3,      /* a HIP runtime call failed                                            */
    TL_ESTRUCT = -4,   /* malformed batch: offsets not ascending / child outside its tree /
                          node with two parents / tree without exactly one root / leaf word id
                          outside the vocabulary / node count inconsistent with full binary trees */
    TL_ESTALL = -5,    /* TL_SCHED_READY made no progress within its spin budget (nodes that are
                          unreachable from any leaf, e.g. a cycle); outputs are incomplete.  The
                          level schedulers report such a batch as TL_ESTRUCT.                   */
    TL_ELIMIT = -6     /* tl_forward_noalloc: the batch does not fit the fixed workspace         */
};

typedef struct {
    int cell;          /* enum tl_cell      */
    int precision;     /* enum tl_precision */
    int scheduler;     /* enum tl_scheduler */
    int validate;      /* != 0: additionally prove, before any cell runs, that every node is
                          reachable bottom-up from the leaves (costs one pass whose length is the
                          tree height).  The cheap checks listed under TL_ESTRUCT always run.    */
    int vocab;         /* rows of emb                                                           */
    int embed_dim;     /* E.  TL_TREERNN / TL_RNTN require embed_dim == hidden                  */
    int hidden;        /* H (called d for TreeRNN / RNTN)                                       */
    int spin_limit;    /* 0 = default.  Upper bound on consecutive unsuccessful polls of a
                          waiting workgroup before it gives up with TL_ESTALL.                   */
    /* All parameter arrays: DEVICE pointers, fp32, row-major, read during tl_create only
     * (the library keeps its own re-packed copies; the caller may free them afterwards). */
    const float *emb;     /* [vocab x E]                                                          */
    const float *w_leaf;  /* TL_TREELSTM: [E x 3H], column blocks i | o | u.   Else NULL.         */
    const float *b_leaf;  /* TL_TREELSTM: [3H].                                Else NULL.         */
    const float *u;       /* TL_TREELSTM: [2H x 5H], column blocks i | f_l | f_r | o | u; rows
                             0..H-1 multiply h_left, rows H..2H-1 multiply h_right.
                             TL_TREERNN / TL_RNTN: W [2d x d].                                    */
    const float *b;       /* TL_TREELSTM: [5H];  TL_TREERNN / TL_RNTN: [d]                        */
    const float *v;       /* TL_RNTN: [d x 2d x 2d], index order (k, p, q).    Else NULL.
                             TL_RNTN needs d <= 128 and TL_F32 (else TL_EINVAL).                  */
} tl_config;

/* Creates a context on the current HIP device.  cfg is HOST memory; *out receives the
 * context.  Synchronous (returns after the parameter copies are packed). */
int tl_create(const tl_config *cfg, tl_ctx **out);

/*
 * Evaluates every node of a batch.  Asynchronous: all work is enqueued on hip_stream
 * (a hipStream_t passed as void*, NULL = the default stream), except that
 * TL_SCHED_LEVEL_HOST waits for the structure pass to learn the number of heights,
 * and that the first call with a larger batch than any before (re)allocates the
 * context's workspace, which synchronises the device.
 *
 * With TL_SCHED_READY or TL_SCHED_LEVEL_DEVICE, profiling off, and after one ordinary call
 * with a batch at least as large (so that nothing is allocated), the call makes no host round
 * trip and may be captured in a HIP graph and replayed.
 *
 *   n_trees >= 1, n_nodes >= n_trees                          HOST scalars
 *                         (n_trees = n_nodes = 0, an empty batch, is accepted: nothing is
 *                         launched, read or written, the pointers may be NULL, and
 *                         tl_status reports TL_OK afterwards)
 *   tree_off [n_trees+1]  int32, tree_off[0]=0, ascending,
 *                         tree_off[n_trees]=n_nodes            DEVICE, read-only
 *   left, right, word [n_nodes] int32                          DEVICE, read-only
 *   h [n_nodes x H] fp32 out, row n = state of node n          DEVICE
 *   c [n_nodes x H] fp32 out (TL_TREELSTM; ignored and may be
 *                         NULL for the other cells)            DEVICE
 *   h_root, c_root [n_trees x H] fp32 out, may be NULL         DEVICE
 *   root [n_trees] int32 out: global index of each tree's root,
 *                         may be NULL                          DEVICE
 *
 * Input arrays must stay valid and unmodified until the stream has passed the call.
 * Host-detectable errors are returned at once.  Errors found on the device (TL_ESTRUCT,
 * TL_ESTALL) are latched and reported by tl_status; after such an error no cell kernel
 * reads through a bad index, and the output contents are unspecified.
 */
int tl_forward(tl_ctx *ctx, int n_trees, int n_nodes,
               const int32_t *tree_off, const int32_t *left, const int32_t *right,
               const int32_t *word, float *h, float *c, float *h_root, float *c_root,
               int32_t *root, void *hip_stream);

/*
 * tl_forward for callers that cannot allocate device memory while they run: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * the same results bit for bit as tl_forward, but the scheduler state (parent links, ready
 * counters, ready queue, mailboxes, control block, and the bf16 copy of h that TL_BF16_IN gathers
 * from) lives in one fixed array that is part of the library's device code - about 17.2 MiB of
 * every GPU the library is used on, held until the process ends - instead of a workspace that the
 * context allocates and grows.  The call allocates, creates and frees nothing (no hipMalloc,
 * hipHostMalloc, hipFree, event creation), never synchronises, and only enqueues kernels on
 * hip_stream.  Limits:
 *   n_nodes <= TL_NOALLOC_MAX_NODES, and with TL_BF16_IN also
 *   n_nodes * roundup(H, 8) <= TL_NOALLOC_MAX_NODES * 512     else TL_ELIMIT (nothing is enqueued)
 *   TL_SCHED_LEVEL_HOST contexts                               TL_EINVAL (that scheduler reads
 *                                                              level offsets back to the host)
 * Stage timing (tl_set_profiling) is not recorded and gate activations (tl_set_keep_gates) are not
 * kept by this call.  tl_status and tl_last_stats afterwards report on this call like on a
 * tl_forward.  All contexts of a process share the one array of their GPU, which holds whatever
 * the last call left there (every call resets what it needs): two such calls that overlap in time
 * on one GPU - from two contexts or two streams - race and give wrong results; order them on one
 * stream or with events.  tl_forward calls are not affected (they use the context's own workspace).
 */
enum { TL_NOALLOC_MAX_NODES = 16384 };
int tl_forward_noalloc(tl_ctx *ctx, int n_trees, int n_nodes,
                       const int32_t *tree_off, const int32_t *left, const int32_t *right,
                       const int32_t *word, float *h, float *c, float *h_root, float *c_root,
                       int32_t *root, void *hip_stream);

/* Waits for the stream of the last tl_forward and returns its latched device-side
 * error (TL_OK if none). */
int tl_status(tl_ctx *ctx);

/* Stage timing.  After tl_set_profiling(ctx, 1) every tl_forward records HIP events between
 * its stages on the caller's stream; the events of the last TL_PROFILE_RING forwards are kept.
 * tl_stage_ms waits for the forward that lies `back` calls in the past (0 = the last one) and
 * writes TL_N_STAGES durations in milliseconds to ms (HOST):
 *   [0] structure pass (parents, counters, roots; heights and per-height lists if used)
 *   [1] leaf cells   [2] internal cells incl. scheduling   [3] root gather   [4] total
 * TL_EINVAL if that forward was not recorded. */
enum { TL_N_STAGES = 5, TL_PROFILE_RING = 128 };
int tl_set_profiling(tl_ctx *ctx, int on);
int tl_stage_ms(tl_ctx *ctx, int back, float *ms);

/* Facts about the last forward, for reports and tests (HOST out-parameters, any may be
 * NULL): number of heights seen by a level scheduler (0 for TL_SCHED_READY; with
 * TL_SCHED_LEVEL_DEVICE the number of frontiers it evaluated plus one for the leaves, which
 * exceeds the number of heights by a few when it left the last rows of large frontiers to
 * the next one), number of tiles of ready nodes formed by TL_SCHED_READY (0 otherwise),
 * workgroups launched for the internal-node kernel.  Waits for the stream. */
int tl_last_stats(tl_ctx *ctx, int *n_levels, int *n_tiles, int *n_workgroups);

/*
 * Backward pass of a forward in TL_F32, for all three cells (Section 4.2.2, recursive
 * backpropagation: the gradient of a node's cell is applied from the roots down, each node
 * finding its forward values by node index).  The loss may depend on every node's h:
 * g_h[n] = dL/dh[n] (zero rows where it does not).  h and c are the rows tl_forward wrote for
 * the same batch.
 *   tree_off, left, right, word, h, c   as in tl_forward (h, c read-only; c NULL for
 *             TL_TREERNN)                                                         DEVICE
 *   g_h       [n_nodes x H] fp32                                                  DEVICE, read-only
 *   d_u       [2H x 5H], d_b [5H], d_w_leaf [E x 3H], d_b_leaf [3H]  fp32 out,
 *             sums over all nodes of the batch, same layouts as the parameters    DEVICE
 *             (TL_TREERNN: d_u [2H x H], d_b [H]; d_w_leaf, d_b_leaf unused, may be NULL.
 *             TL_RNTN: d_u [2d x d] for W, d_b [d], and d_w_leaf receives the gradient of the
 *             tensor V, [d x 2d x 2d]; d_b_leaf unused.)
 *   d_x       [n_nodes x E] fp32 out: row n = dL/d(embedding row used by leaf n);
 *             rows of internal nodes are zero (the caller scatter-adds by word)    DEVICE
 * fp32 arithmetic; the TreeLSTM gate activations are recomputed from h / c unless the forward
 * kept them (tl_set_keep_gates); TreeRNN and RNTN need nothing but h.  The RNTN path is a first
 * version: it materialises a row of d * 2d + d values per internal node (workspace of that size).
 * Work is enqueued on hip_stream, but the call waits for the structure pass and returns the deferred
 * structure status: TL_OK, TL_ESTRUCT, ... (where the heights are walked by launches, one pair per height,
 * it needs their number and sizes first; where one persistent kernel walks them, it has enqueued all its
 * work by then and the device is not held up).  With tl_set_async_backward(ctx, 1) it does not wait.
 * The first call for a larger batch than any before allocates workspace (TL_ENOMEM if the RNTN
 * rows would take more than 64 GiB).  TL_BF16_IN: TL_EINVAL.
 */
int tl_backward(tl_ctx *ctx, int n_trees, int n_nodes, const int32_t *tree_off, const int32_t *left,
                const int32_t *right, const int32_t *word, const float *h, const float *c, const float *g_h,
                float *d_u, float *d_b, float *d_w_leaf, float *d_b_leaf, float *d_x, void *hip_stream);

/*
 * One step of plain stochastic gradient descent on the parameters the context holds (the
 * training runs of Section 6 update the model after every batch; the paper does not print its
 * optimiser, the plainest one is taken): theta <- theta - lr * gradient for U, b, W_leaf,
 * b_leaf, and emb[word[n]] <- emb[word[n]] - lr * d_x[n] for every leaf n.  The gradient arrays
 * are those tl_backward wrote (DEVICE, read-only); left / word / n_nodes are the batch's arrays.
 * d_x may be NULL: the embedding table then stays as it is.  Afterwards everything derived from
 * the parameters (packed weights of the forward and backward kernels) is rebuilt; all of it is
 * enqueued on hip_stream and nothing is allocated.  Dense parameters change exactly as the
 * formula says in fp32 (product rounded, then difference); embedding rows shared by several
 * leaves are updated with atomics.  Calls on one context must be ordered with its forwards
 * and backwards (same stream, or synchronised).  TL_F32 only, else TL_EINVAL; TL_TREERNN has
 * u, b and the embedding only (d_w_leaf, d_b_leaf may be NULL), TL_RNTN takes the gradient of
 * V in d_w_leaf, as tl_backward writes it.
 */
int tl_sgd_update(tl_ctx *ctx, float lr, int n_nodes, const int32_t *left, const int32_t *word, const float *d_u,
                  const float *d_b, const float *d_w_leaf, const float *d_b_leaf, const float *d_x, void *hip_stream);

/*
 * Copies the context's current parameters to the caller's DEVICE buffers (any of them may be
 * NULL): u [2H x 5H], b [5H], w_leaf [E x 3H], b_leaf [3H], emb [vocab x E], fp32, the layouts
 * tl_create takes (TL_TREERNN: u [2H x H], b [H]; w_leaf and b_leaf must be NULL.  TL_RNTN:
 * u = W [2d x d], b [d], w_leaf receives V [d x 2d x 2d], b_leaf must be NULL).
 * Asynchronous on hip_stream.  TL_F32 only, else TL_EINVAL.
 */
int tl_get_params(tl_ctx *ctx, float *u, float *b, float *w_leaf, float *b_leaf, float *emb, void *hip_stream);

/*
 * Training mode of tl_forward (Section 4.2.2: the backward pass of a recursive call looks up the
 * forward values of the same call instance).  With on != 0, every later tl_forward of a TreeLSTM /
 * TL_F32 context also keeps the gate activations of every node (5H floats per node, in a
 * workspace the context owns and grows like its others), and a tl_backward whose h argument and
 * n_nodes are those of that forward takes them from there instead of recomputing the forward
 * contraction.  The caller must not change h, c or the batch between the two calls.  Results of
 * tl_forward are unchanged bit for bit; those of tl_backward agree with the recomputing path to
 * rounding (the same activations, computed once instead of twice).  Other cells / precisions:
 * accepted, no effect.  Off by default.
 */
int tl_set_keep_gates(tl_ctx *ctx, int on);

/*
 * For callers that must not be held up by tl_backward (the recursion of Section 4.2.2 walked without the host):
 * with on > 0, a tl_backward that needs no contraction for its gate gradients - TreeLSTM from kept gate
 * activations (tl_set_keep_gates), TreeRNN - walks all heights in one persistent kernel that finds the
 * per-height lists on the device (TreeLSTM and TreeRNN with H = 128, 256, 384 or 512: the operand gradient on weight-stationary
 * workgroups).  Nothing is read back and the call returns without waiting; a malformed batch is then reported
 * by tl_status (TL_ESTRUCT, gradients undefined), not by tl_backward.  Same results as the per-height launches
 * (same contractions in the same order).
 * on == 0, the default: tl_backward returns the structure pass's status itself, as described there.  Where the
 * weight-stationary form applies it is the fastest form whatever the shape of the trees (H = 512, 256 trees:
 * 1.26 ms per call against 1.27 with launches per height; 64 trees of 1 024 heights: 13.9 against 16.9 ms), so
 * the call enqueues all its work and then waits only for the copy of that status, which sits in front of that
 * kernel.  Otherwise (other hidden sizes: the persistent kernel with the streaming cell is 5 % slower
 * than the launches on shallow batches and faster on deep ones) the call waits for the number of heights and
 * takes the persistent kernel for more than 64 of them, launches per height up to there.
 * on < 0: always launches per height.  Like the persistent schedulers of tl_forward, the kernel needs all its
 * workgroups resident.  Recomputed gates and TL_RNTN always take the launches per height and wait.
 */
int tl_set_async_backward(tl_ctx *ctx, int on);

/*
 * Per-node classifier head (Section 6.1: the evaluated networks label all nodes of a parse
 * tree; the paper does not print the head, the usual form is taken):
 *     probs[n] = softmax(h[n] W_s + b_s)          for n = 0 .. n_rows-1
 * Asynchronous on hip_stream; call it after tl_forward on the same stream to label a batch.
 *   h     [n_rows x H] fp32, H = cfg.hidden of ctx       DEVICE, read-only
 *   w_s   [H x n_classes] fp32, row-major                 DEVICE, read-only
 *   b_s   [n_classes] fp32                                DEVICE, read-only
 *   probs [n_rows x n_classes] fp32 out                   DEVICE
 * fp32 arithmetic throughout (one pass over h; bound by memory bandwidth).
 * 1 <= n_classes <= 32 and n_classes * H <= 24576, else TL_EINVAL.  Nothing is allocated and
 * nothing of the context changes.
 */
int tl_classify(tl_ctx *ctx, int n_rows, const float *h, const float *w_s, const float *b_s, int n_classes,
                float *probs, void *hip_stream);

/*
 * Backward pass of the classifier head under a cross-entropy loss summed over the labelled
 * rows (the training objective of the sentiment networks of Section 6.1, where every node of a
 * parse tree carries a label; the paper does not print it, the usual form is taken):
 *     loss      = - sum_n log probs[n][label[n]]            probs as in tl_classify
 *     d_logits[n] = probs[n] - onehot(label[n])
 *     g_h[n]    = d_logits[n] W_s^T          (the g_h argument of tl_backward)
 *     d_w_s     = sum_n h[n]^T d_logits[n]       d_b_s = sum_n d_logits[n]
 * A row whose label is outside [0, n_classes) has no label: its d_logits and g_h rows are
 * zero and it adds nothing to the sums.
 *   h, w_s, b_s   as in tl_classify                                   DEVICE, read-only
 *   label     [n_rows] int32                                           DEVICE, read-only
 *   d_logits  [n_rows x n_classes] fp32 out                            DEVICE
 *   g_h       [n_rows x H] fp32 out                                    DEVICE
 *   d_w_s     [H x n_classes], d_b_s [n_classes], loss [1]  fp32 out   DEVICE
 * fp32 arithmetic; the sums over rows are accumulated with atomics, so their last bits can
 * differ from run to run.  Asynchronous on hip_stream, allocates nothing, same limits on
 * n_classes as tl_classify.  n_rows = 0 zeroes the three sums.
 */
int tl_classify_backward(tl_ctx *ctx, int n_rows, const float *h, const float *w_s, const float *b_s, int n_classes,
                         const int32_t *label, float *d_logits, float *g_h, float *d_w_s, float *d_b_s, float *loss,
                         void *hip_stream);

/*
 * Top-down generation of dynamically structured trees (Section 6.3, "Dynamically Structured
 * Models": whether a node gets children is decided from the value computed for that node, so the
 * trees are not known before they are evaluated).  The paper names such models and prints no
 * equations; the form taken is an LSTM step along every parent -> child edge with weights per
 * side and a linear stopping rule:
 *     score(n) = w_stop . h[n] + b_stop        n gets two children iff score(n) > 0,
 *                                               depth(n) < max_depth and two rows are free
 *     child on side s:  g = h[n] U_s + b_s = [gi|gf|go|gu]
 *                       c_s = sigmoid(gf) c[n] + sigmoid(gi) tanh(gu),  h_s = sigmoid(go) tanh(c_s)
 *
 * tl_td_create: copies and re-packs the parameters.
 *   u_td   [H x 8H] fp32 row-major, columns [iL|fL|oL|uL|iR|fR|oR|uR]   DEVICE, read during the call
 *   b_td   [8H], w_stop [H] fp32                                         DEVICE, read during the call
 *   b_stop, spin_limit (0: default; bound of every wait inside the kernel)
 * TL_OK, TL_EINVAL (null pointer, hidden < 1 or > 16384), TL_ENOMEM, TL_EHIP.
 */
typedef struct tl_td_ctx tl_td_ctx;
int tl_td_create(int hidden, const float *u_td, const float *b_td, const float *w_stop, float b_stop, int spin_limit,
                 tl_td_ctx **out);

/*
 * Grows n_trees trees in one persistent kernel, asynchronously on hip_stream: batches of up to 32 roots (H a
 * multiple of 4, rows 16-byte aligned) without frontiers - a node is expanded as soon as its own parent has been
 * decided, and its children are computed while it is still being scored -, larger ones breadth first, frontier by
 * frontier, with two grid barriers per depth.
 *   h, c     [max_nodes x H] fp32: rows 0 .. n_trees-1 hold the root states on entry (node t is
 *            the root of tree t); every other used row is written                       DEVICE
 *   parent, left, right, depth  [max_nodes] int32 out: links (-1: none) and depth       DEVICE
 *   score    [max_nodes] fp32 out                                                       DEVICE
 *   counts   [4] int32 out: nodes, nodes that would have expanded but found no two free
 *            rows, frontiers walked, 0                                                  DEVICE
 * Rows beyond counts[0] hold no result (the call may have overwritten them: of h and c up to 16 MiB, of the
 * int32 arrays all max_nodes entries).  The two children of a node are consecutive rows, left
 * first; which rows they are depends on timing and differs from run to run, the trees (and each
 * node's state, bit for bit) do not.  Nothing is allocated.  fp32 arithmetic on the matrix units.
 * The kernel needs the device to itself (all its workgroups resident), like the persistent
 * schedulers of tl_forward; calls on one context must not overlap.
 * TL_OK, TL_EINVAL (null pointer, n_trees < 1, max_nodes < n_trees, max_depth < 0), TL_EHIP.
 * tl_td_status waits for the stream and returns what the kernel latched: TL_OK, or TL_ESTALL if
 * a wait inside the kernel ran out of spins.
 */
int tl_td_generate(tl_td_ctx *ctx, int n_trees, int max_nodes, int max_depth, float *h, float *c, int32_t *parent,
                   int32_t *left, int32_t *right, int32_t *depth, float *score, int32_t *counts, void *hip_stream);
int tl_td_status(tl_td_ctx *ctx);
int tl_td_destroy(tl_td_ctx *ctx);

const char *tl_strerror(int code);

/* Frees the context and everything it owns.  Waits for the device. */
int tl_destroy(tl_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* TREELSTM_H */
