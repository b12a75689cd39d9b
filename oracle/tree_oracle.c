/*
 * CPU checker for batched forward evaluation of recursive tree networks.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the GPU
 * library is compared against.  It shares no code with the GPU library and must
 * never be linked into, imported by, or called from the product path.
 *
 * What it follows:
 *  - Evaluation order "recursive": the recursive definition of the paper's
 *    Figure 2 (a node is a leaf -> embed + cell; otherwise evaluate both
 *    children, then the two-input cell).
 *  - Evaluation order "topological": the iterative formulation of Figure 1
 *    (all leaves, then internal nodes in an order in which children precede
 *    parents).  Section 6.2 ("Convergence") states both give numerically
 *    identical results; here they are bit-identical because each node's
 *    arithmetic is the same sequence of operations.
 *  - The paper names the cells (TreeLSTM, TreeRNN, RNTN; Section 6.1) without
 *    printing equations.  The forms used are the standard binary ones:
 *
 *    TreeLSTM leaf     g = x W_x + b_x, g = [gi|go|gu] each H wide
 *                      i = s(gi) o = s(go) u = tanh(gu);  c = i*u;  h = o*tanh(c)
 *    TreeLSTM internal a = [h_l ; h_r];  g = a U + b, g = [gi|gfl|gfr|go|gu]
 *                      c = s(gi)*tanh(gu) + s(gfl)*c_l + s(gfr)*c_r;  h = s(go)*tanh(c)
 *    TreeRNN           leaf h = x;  internal h = tanh(a W + b)
 *    RNTN              leaf h = x;  internal h_k = tanh(sum_pq a_p V[k][p][q] a_q + (a W)_k + b_k)
 *
 *    with s(t) = 1/(1+exp(-t)).
 *
 * Arithmetic: inputs are fp32; every sum is accumulated in double in ascending
 * index order; s() and tanh() are libm in double; each stored h / c element is
 * rounded to fp32 once.  A parent consumes the *stored* fp32 h / c of its children.
 * With round_bf16 != 0 the gathered operand vector (embedding row or [h_l;h_r]) is
 * rounded to bfloat16 (round to nearest even) before it enters a contraction, which
 * models a matrix unit fed with bf16 operands; the caller passes weights that are
 * already bf16-representable.  c is never rounded to bf16.
 *
 * Parity status: the cell equations are pinned by tests against closed forms,
 * hand-worked small trees, torch.nn.RNN / torch.nn.LSTM special cases and an
 * independent numpy evaluation.  Agreement with the *paper authors'* own TreeLSTM
 * variant (leaf treatment, bias sharing, hyper-parameters) is PARITY UNPINNED: the
 * paper prints no equations, weights or activations.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { CELL_TREELSTM = 0, CELL_TREERNN = 1, CELL_RNTN = 2 };

typedef struct {
    int cell, vocab, E, H, round_bf16;
    const float *emb, *w_leaf, *b_leaf, *u, *b, *v;
    const int32_t *left, *right, *word;
    float *h, *c;
} model_t;

static double sigm(double t) { return 1.0 / (1.0 + exp(-t)); }

/* fp32 -> nearest bfloat16 (ties to even), returned as fp32. Finite inputs only. */
static float to_bf16(float x)
{
    uint32_t bits;
    memcpy(&bits, &x, 4);
    uint32_t lsb = (bits >> 16) & 1u;
    bits += 0x7FFFu + lsb;
    bits &= 0xFFFF0000u;
    memcpy(&x, &bits, 4);
    return x;
}

static void load_operand(const model_t *m, double *dst, const float *src, int n)
{
    for (int k = 0; k < n; ++k)
        dst[k] = m->round_bf16 ? (double)to_bf16(src[k]) : (double)src[k];
}

/* g[j] = bias[j] + sum_k a[k] * W[k][j],  W row-major [K x ncol] */
static void affine(const double *a, int K, const float *W, const float *bias, int ncol, double *g)
{
    for (int j = 0; j < ncol; ++j) g[j] = 0.0;
    for (int k = 0; k < K; ++k) {
        const double ak = a[k];
        const float *row = W + (size_t)k * ncol;
        for (int j = 0; j < ncol; ++j) g[j] += ak * (double)row[j];
    }
    for (int j = 0; j < ncol; ++j) g[j] += (double)bias[j];
}

static void leaf_cell(const model_t *m, int n, double *a, double *g)
{
    const int H = m->H, E = m->E;
    const float *x = m->emb + (size_t)m->word[n] * E;
    float *h = m->h + (size_t)n * H;
    if (m->cell == CELL_TREELSTM) {
        float *c = m->c + (size_t)n * H;
        load_operand(m, a, x, E);
        affine(a, E, m->w_leaf, m->b_leaf, 3 * H, g);
        for (int j = 0; j < H; ++j) {
            double i = sigm(g[j]), o = sigm(g[H + j]), u = tanh(g[2 * H + j]);
            double cc = i * u;
            c[j] = (float)cc;
            h[j] = (float)(o * tanh(cc));
        }
    } else {
        for (int j = 0; j < H; ++j) h[j] = x[j];   /* E == H for these cells */
    }
}

static void internal_cell(const model_t *m, int n, double *a, double *g)
{
    const int H = m->H;
    const int l = m->left[n], r = m->right[n];
    float *h = m->h + (size_t)n * H;
    load_operand(m, a, m->h + (size_t)l * H, H);
    load_operand(m, a + H, m->h + (size_t)r * H, H);
    if (m->cell == CELL_TREELSTM) {
        const float *cl = m->c + (size_t)l * H, *cr = m->c + (size_t)r * H;
        float *c = m->c + (size_t)n * H;
        affine(a, 2 * H, m->u, m->b, 5 * H, g);
        for (int j = 0; j < H; ++j) {
            double i = sigm(g[j]), fl = sigm(g[H + j]), fr = sigm(g[2 * H + j]);
            double o = sigm(g[3 * H + j]), u = tanh(g[4 * H + j]);
            double cc = i * u + fl * (double)cl[j] + fr * (double)cr[j];
            c[j] = (float)cc;
            h[j] = (float)(o * tanh(cc));
        }
    } else {
        affine(a, 2 * H, m->u, m->b, H, g);
        if (m->cell == CELL_RNTN) {
            const int D2 = 2 * H;
            for (int k = 0; k < H; ++k) {
                const float *Vk = m->v + (size_t)k * D2 * D2;
                double s = 0.0;
                for (int p = 0; p < D2; ++p) {
                    double t = 0.0;
                    for (int q = 0; q < D2; ++q) t += (double)Vk[(size_t)p * D2 + q] * a[q];
                    s += a[p] * t;
                }
                g[k] += s;
            }
        }
        for (int j = 0; j < H; ++j) h[j] = (float)tanh(g[j]);
    }
}

static void eval_recursive(const model_t *m, int n, double *a, double *g)
{
    if (m->left[n] < 0) {
        leaf_cell(m, n, a, g);
    } else {
        eval_recursive(m, m->left[n], a, g);
        eval_recursive(m, m->right[n], a, g);
        internal_cell(m, n, a, g);
    }
}

static int height_of(const int32_t *left, const int32_t *right, int n, int32_t *height)
{
    if (left[n] < 0) { height[n] = 0; return 0; }
    int hl = height_of(left, right, left[n], height);
    int hr = height_of(left, right, right[n], height);
    height[n] = 1 + (hl > hr ? hl : hr);
    return height[n];
}

/*
 * Plain traversal of the batch structure.
 *   parent[n] : global index of n's parent, -1 for roots
 *   root[t]   : the node of tree t that is nobody's child
 *   height[n] : 0 at leaves, 1 + max(children) otherwise
 * Returns 0, or -1 if a tree does not have exactly one root / a child index leaves
 * its tree's range / a node has two parents.
 */
int oracle_structure(int n_trees, int n_nodes, const int32_t *tree_off, const int32_t *left,
                     const int32_t *right, int32_t *parent, int32_t *root, int32_t *height)
{
    for (int n = 0; n < n_nodes; ++n) parent[n] = -1;
    for (int t = 0; t < n_trees; ++t) {
        for (int n = tree_off[t]; n < tree_off[t + 1]; ++n) {
            if ((left[n] < 0) != (right[n] < 0)) return -1;
            if (left[n] < 0) continue;
            const int ch[2] = { left[n], right[n] };
            for (int s = 0; s < 2; ++s) {
                if (ch[s] < tree_off[t] || ch[s] >= tree_off[t + 1]) return -1;
                if (parent[ch[s]] != -1) return -1;
                parent[ch[s]] = n;
            }
        }
    }
    for (int t = 0; t < n_trees; ++t) {
        int found = -1;
        for (int n = tree_off[t]; n < tree_off[t + 1]; ++n)
            if (parent[n] == -1) { if (found >= 0) return -1; found = n; }
        if (found < 0) return -1;
        root[t] = found;
        height_of(left, right, found, height);
    }
    return 0;
}

/*
 * Forward evaluation of every node of every tree.
 *   order 0: recursive (Figure 2).  order 1: leaves first, then internal nodes by
 *   ascending height, ties in index order (Figure 1 with a valid topological order).
 *   n_threads: trees are independent, so they may be spread over threads; the
 *   per-node arithmetic is unaffected.
 * h, c: [n_nodes x H] row-major outputs (c is ignored for TreeRNN / RNTN and may be NULL).
 * h_root, c_root: [n_trees x H], may be NULL.  Returns 0 or -1 on a malformed batch.
 */
int oracle_forward(int cell, int vocab, int E, int H, int round_bf16,
                   const float *emb, const float *w_leaf, const float *b_leaf,
                   const float *u, const float *b, const float *v,
                   int n_trees, int n_nodes, const int32_t *tree_off,
                   const int32_t *left, const int32_t *right, const int32_t *word,
                   int order, int n_threads,
                   float *h, float *c, float *h_root, float *c_root)
{
    model_t m = { cell, vocab, E, H, round_bf16, emb, w_leaf, b_leaf, u, b, v, left, right, word, h, c };
    int32_t *parent = malloc(sizeof(int32_t) * (size_t)(n_nodes > 0 ? n_nodes : 1));
    int32_t *height = malloc(sizeof(int32_t) * (size_t)(n_nodes > 0 ? n_nodes : 1));
    int32_t *root = malloc(sizeof(int32_t) * (size_t)(n_trees > 0 ? n_trees : 1));
    int rc = oracle_structure(n_trees, n_nodes, tree_off, left, right, parent, root, height);
    for (int n = 0; rc == 0 && n < n_nodes; ++n)
        if (left[n] < 0 && (word[n] < 0 || word[n] >= vocab)) rc = -1;
    if (rc == 0) {
        const int K = (2 * H > E ? 2 * H : E), G = 5 * H;
        if (n_threads < 1) n_threads = 1;
        #pragma omp parallel for schedule(dynamic, 1) num_threads(n_threads)
        for (int t = 0; t < n_trees; ++t) {
            double *a = malloc(sizeof(double) * (size_t)K);
            double *g = malloc(sizeof(double) * (size_t)G);
            if (order == 0) {
                eval_recursive(&m, root[t], a, g);
            } else {
                const int lo = tree_off[t], hi = tree_off[t + 1];
                for (int lvl = 0; lvl <= height[root[t]]; ++lvl)
                    for (int n = lo; n < hi; ++n)
                        if (height[n] == lvl) {
                            if (lvl == 0) leaf_cell(&m, n, a, g); else internal_cell(&m, n, a, g);
                        }
            }
            for (int j = 0; j < H; ++j) {
                if (h_root) h_root[(size_t)t * H + j] = h[(size_t)root[t] * H + j];
                if (c_root && cell == CELL_TREELSTM) c_root[(size_t)t * H + j] = c[(size_t)root[t] * H + j];
            }
            free(a); free(g);
        }
    }
    free(parent); free(height); free(root);
    return rc;
}

/*
 * Per-node classifier head.  Section 6.1 states that a trained network labels all nodes of the
 * parse trees; the paper does not print the head.  The reading taken is the usual one of the
 * cited models: probs[n] = softmax(h[n] W_s + b_s), W_s is [H x C] row-major.  Logits are
 * accumulated in double (bias first, then k ascending), the softmax subtracts the row maximum
 * and is evaluated in double; each probability is rounded to fp32 once.
 * Pinned by tests against closed forms (zero weights, two classes = logistic function),
 * scipy.special.softmax on a double matmul, shift invariance and a brute-force loop.
 */
int oracle_classify(int n_rows, int H, int C, const float *h, const float *w_s, const float *b_s, float *probs)
{
    if (n_rows < 0 || H < 1 || C < 1) return -1;
    double *z = malloc(sizeof(double) * (size_t)C);
    for (int n = 0; n < n_rows; ++n) {
        for (int c = 0; c < C; ++c) {
            double s = b_s[c];
            for (int k = 0; k < H; ++k) s += (double)h[(size_t)n * H + k] * (double)w_s[(size_t)k * C + c];
            z[c] = s;
        }
        double m = z[0];
        for (int c = 1; c < C; ++c) if (z[c] > m) m = z[c];
        double sum = 0.0;
        for (int c = 0; c < C; ++c) { z[c] = exp(z[c] - m); sum += z[c]; }
        for (int c = 0; c < C; ++c) probs[(size_t)n * C + c] = (float)(z[c] / sum);
    }
    free(z);
    return 0;
}

/*
 * Backward pass of the TreeLSTM forward above (Section 4.2.2, "Recursive Backpropagation": the
 * gradient of a recursive call is the recursive application of the gradient of its body, with
 * the forward values of each call instance kept for it - here the stored h / c rows, found by
 * node index).
 *
 * The loss is any function of the node states; the caller passes g_h[n] = dL/dh[n] for every
 * node (zero rows where a node's state does not enter the loss directly).  With the forward
 * definitions above, going from a node to its children (dh_n = g_h[n] + what the parent sent,
 * dc_n = what the parent sent, zero at roots):
 *   t = tanh(c_n)      do = dh_n * t        dct = dc_n + dh_n * o * (1 - t^2)
 *   internal:  dgi = dct*u*i(1-i)   dgfl = dct*c_l*fl(1-fl)   dgfr = dct*c_r*fr(1-fr)
 *              dgo = do*o(1-o)      dgu = dct*i*(1-u^2)
 *              dc_l = dct*fl        dc_r = dct*fr
 *              [dh_l ; dh_r] (sent to the children) = dG U^T      dU += a^T dG     db += dG
 *   leaf:      dgi = dct*u*i(1-i)   dgo = do*o(1-o)   dgu = dct*i*(1-u^2)
 *              dx = dG W_x^T        dW_x += x^T dG    db_x += dG
 * Gates are recomputed in double from the stored fp32 child states (the same values the forward
 * cell consumed); all sums are accumulated in double and rounded to fp32 once at the end.
 * d_x is [n_nodes x E]: row n is dL/d(embedding row used by leaf n); rows of internal nodes are zero.
 * TreeLSTM only.  Returns 0, or -1 on a malformed batch.
 * Pinned by tests against torch autograd on an independent float64 evaluation, finite
 * differences, and closed forms.
 */
typedef struct {
    int E, H;
    const float *emb, *w_leaf, *b_leaf, *u, *b, *h, *c, *g_h;
    const int32_t *left, *right, *word;
    double *d_u, *d_b, *d_w_leaf, *d_b_leaf;   /* accumulators */
    float *d_x;
} bwd_t;

static void backward_node(const bwd_t *m, int n, const double *dh, const double *dc, double *scratch)
{
    const int H = m->H, E = m->E;
    const float *c = m->c + (size_t)n * H;
    if (m->left[n] < 0) {
        double *x = scratch, *g = x + E, *dg = g + 3 * H;
        const float *xr = m->emb + (size_t)m->word[n] * E;
        for (int k = 0; k < E; ++k) x[k] = xr[k];
        affine(x, E, m->w_leaf, m->b_leaf, 3 * H, g);
        for (int j = 0; j < H; ++j) {
            const double i = sigm(g[j]), o = sigm(g[H + j]), u = tanh(g[2 * H + j]);
            const double t = tanh((double)c[j]);
            const double d_o = dh[j] * t, dct = dc[j] + dh[j] * o * (1.0 - t * t);
            dg[j] = dct * u * i * (1.0 - i);
            dg[H + j] = d_o * o * (1.0 - o);
            dg[2 * H + j] = dct * i * (1.0 - u * u);
        }
        for (int k = 0; k < E; ++k) {
            const float *row = m->w_leaf + (size_t)k * 3 * H;
            double s = 0.0;
            for (int j = 0; j < 3 * H; ++j) {
                s += dg[j] * (double)row[j];
                m->d_w_leaf[(size_t)k * 3 * H + j] += x[k] * dg[j];
            }
            m->d_x[(size_t)n * E + k] = (float)s;
        }
        for (int j = 0; j < 3 * H; ++j) m->d_b_leaf[j] += dg[j];
        return;
    }
    const int l = m->left[n], r = m->right[n];
    double *a = scratch, *g = a + 2 * H, *dg = g + 5 * H, *dhl = dg + 5 * H, *dhr = dhl + H, *dcl = dhr + H, *dcr = dcl + H;
    double *next = dcr + H;
    const float *cl = m->c + (size_t)l * H, *cr = m->c + (size_t)r * H;
    for (int k = 0; k < H; ++k) { a[k] = m->h[(size_t)l * H + k]; a[H + k] = m->h[(size_t)r * H + k]; }
    affine(a, 2 * H, m->u, m->b, 5 * H, g);
    for (int j = 0; j < H; ++j) {
        const double i = sigm(g[j]), fl = sigm(g[H + j]), fr = sigm(g[2 * H + j]);
        const double o = sigm(g[3 * H + j]), u = tanh(g[4 * H + j]);
        const double t = tanh((double)c[j]);
        const double d_o = dh[j] * t, dct = dc[j] + dh[j] * o * (1.0 - t * t);
        dg[j] = dct * u * i * (1.0 - i);
        dg[H + j] = dct * (double)cl[j] * fl * (1.0 - fl);
        dg[2 * H + j] = dct * (double)cr[j] * fr * (1.0 - fr);
        dg[3 * H + j] = d_o * o * (1.0 - o);
        dg[4 * H + j] = dct * i * (1.0 - u * u);
        dcl[j] = dct * fl;
        dcr[j] = dct * fr;
    }
    for (int k = 0; k < 2 * H; ++k) {
        const float *row = m->u + (size_t)k * 5 * H;
        double s = 0.0;
        for (int j = 0; j < 5 * H; ++j) {
            s += dg[j] * (double)row[j];
            m->d_u[(size_t)k * 5 * H + j] += a[k] * dg[j];
        }
        if (k < H) dhl[k] = s + (double)m->g_h[(size_t)l * H + k];
        else dhr[k - H] = s + (double)m->g_h[(size_t)r * H + (k - H)];
    }
    for (int j = 0; j < 5 * H; ++j) m->d_b[j] += dg[j];
    backward_node(m, l, dhl, dcl, next);
    backward_node(m, r, dhr, dcr, next);
}

int oracle_backward(int vocab, int E, int H,
                    const float *emb, const float *w_leaf, const float *b_leaf, const float *u, const float *b,
                    int n_trees, int n_nodes, const int32_t *tree_off,
                    const int32_t *left, const int32_t *right, const int32_t *word,
                    const float *h, const float *c, const float *g_h,
                    float *d_u, float *d_b, float *d_w_leaf, float *d_b_leaf, float *d_x)
{
    int32_t *parent = malloc(sizeof(int32_t) * (size_t)(n_nodes > 0 ? n_nodes : 1));
    int32_t *height = malloc(sizeof(int32_t) * (size_t)(n_nodes > 0 ? n_nodes : 1));
    int32_t *root = malloc(sizeof(int32_t) * (size_t)(n_trees > 0 ? n_trees : 1));
    int rc = oracle_structure(n_trees, n_nodes, tree_off, left, right, parent, root, height);
    for (int n = 0; rc == 0 && n < n_nodes; ++n)
        if (left[n] < 0 && (word[n] < 0 || word[n] >= vocab)) rc = -1;
    if (rc == 0) {
        const size_t nu = (size_t)2 * H * 5 * H, nw = (size_t)E * 3 * H;
        bwd_t m = { E, H, emb, w_leaf, b_leaf, u, b, h, c, g_h, left, right, word,
                    calloc(nu, sizeof(double)), calloc((size_t)5 * H, sizeof(double)),
                    calloc(nw, sizeof(double)), calloc((size_t)3 * H, sizeof(double)), d_x };
        memset(d_x, 0, sizeof(float) * (size_t)n_nodes * E);
        int max_h = 0;
        for (int t = 0; t < n_trees; ++t) if (height[root[t]] > max_h) max_h = height[root[t]];
        /* scratch of one node: 2H + 5H + 5H + 4H doubles (or E + 6H at a leaf); one such frame per level of the recursion */
        const size_t frame = (size_t)(16 * H > E + 6 * H ? 16 * H : E + 6 * H);
        double *scratch = malloc(sizeof(double) * frame * (size_t)(max_h + 2));
        double *dh = malloc(sizeof(double) * (size_t)H), *dc = calloc((size_t)H, sizeof(double));
        for (int t = 0; t < n_trees; ++t) {
            for (int j = 0; j < H; ++j) dh[j] = (double)g_h[(size_t)root[t] * H + j];
            backward_node(&m, root[t], dh, dc, scratch);
        }
        for (size_t i = 0; i < nu; ++i) d_u[i] = (float)m.d_u[i];
        for (int j = 0; j < 5 * H; ++j) d_b[j] = (float)m.d_b[j];
        for (size_t i = 0; i < nw; ++i) d_w_leaf[i] = (float)m.d_w_leaf[i];
        for (int j = 0; j < 3 * H; ++j) d_b_leaf[j] = (float)m.d_b_leaf[j];
        free(m.d_u); free(m.d_b); free(m.d_w_leaf); free(m.d_b_leaf); free(scratch); free(dh); free(dc);
    }
    free(parent); free(height); free(root);
    return rc;
}

/*
 * Backward pass of the classifier head with a cross-entropy loss summed over the labelled nodes:
 *   L = - sum_{n : label[n] >= 0} log probs[n][label[n]],   probs as in oracle_classify.
 * With g[n] = probs[n] - onehot(label[n]) (zero for unlabelled nodes):
 *   g_h[n] = g[n] W_s^T     d_w_s = sum_n h[n]^T g[n]     d_b_s = sum_n g[n]
 * All sums in double, rounded to fp32 once.  g_h is what the tree backward pass takes as the
 * upstream gradient of every node.  Returns 0, or -1 on bad dimensions / labels.
 * Pinned by tests against torch's cross_entropy autograd in float64 and closed forms.
 */
int oracle_classify_backward(int n_rows, int H, int C, const float *h, const float *w_s, const float *b_s,
                             const int32_t *label, float *g_h, float *d_w_s, float *d_b_s, double *loss)
{
    if (n_rows < 0 || H < 1 || C < 1) return -1;
    double *z = malloc(sizeof(double) * (size_t)C);
    double *dw = calloc((size_t)H * C, sizeof(double)), *db = calloc((size_t)C, sizeof(double));
    double total = 0.0;
    int rc = 0;
    for (int n = 0; n < n_rows && rc == 0; ++n) {
        float *gr = g_h + (size_t)n * H;
        if (label[n] < 0) { for (int k = 0; k < H; ++k) gr[k] = 0.f; continue; }
        if (label[n] >= C) { rc = -1; break; }
        for (int c = 0; c < C; ++c) {
            double s = b_s[c];
            for (int k = 0; k < H; ++k) s += (double)h[(size_t)n * H + k] * (double)w_s[(size_t)k * C + c];
            z[c] = s;
        }
        double m = z[0];
        for (int c = 1; c < C; ++c) if (z[c] > m) m = z[c];
        double sum = 0.0;
        for (int c = 0; c < C; ++c) sum += exp(z[c] - m);
        total += -(z[label[n]] - m - log(sum));
        for (int c = 0; c < C; ++c) z[c] = exp(z[c] - m) / sum - (c == label[n] ? 1.0 : 0.0);
        for (int k = 0; k < H; ++k) {
            double s = 0.0;
            const double hk = h[(size_t)n * H + k];
            for (int c = 0; c < C; ++c) {
                s += z[c] * (double)w_s[(size_t)k * C + c];
                dw[(size_t)k * C + c] += hk * z[c];
            }
            gr[k] = (float)s;
        }
        for (int c = 0; c < C; ++c) db[c] += z[c];
    }
    for (size_t i = 0; i < (size_t)H * C; ++i) d_w_s[i] = (float)dw[i];
    for (int c = 0; c < C; ++c) d_b_s[c] = (float)db[c];
    *loss = total;
    free(z); free(dw); free(db);
    return rc;
}

/*
 * Top-down generation of trees whose shape is decided by values computed on the way (Section 6.3,
 * "Dynamically Structured Models": whether a node gets children depends on the node's own
 * computed value, so the tree is not known before it is evaluated).  The paper names such models
 * (TD-TreeLSTM and others) and prints no equations; the form used here is an LSTM step along
 * every parent -> child edge with weights per side, and a linear stopping rule:
 *
 *    score(n) = w_stop . h_n + b_stop                     n expands iff score(n) > 0 and depth(n) < max_depth
 *    child on side s in {L, R}:  g = h_n U_s + b_s,  g = [gi|gf|go|gu] each H wide
 *                                c_s = s(gf)*c_n + s(gi)*tanh(gu);   h_s = s(go)*tanh(c_s)
 *
 * u_td is [H x 8H] row-major with columns [iL|fL|oL|uL|iR|fR|oR|uR], b_td [8H].  Sums in double in
 * ascending index order, stored states rounded to fp32 once; a child consumes the stored fp32
 * state of its parent.  The score is rounded to fp32 before it is compared with zero.
 *
 * oracle_td_step: both children and the score of one node from its stored state.
 *   child_h, child_c: [2 x H] (left, right).
 */
void oracle_td_step(int H, const float *u_td, const float *b_td, const float *w_stop, float b_stop,
                    const float *h, const float *c, float *child_h, float *child_c, float *score)
{
    double s = b_stop;
    for (int k = 0; k < H; ++k) s += (double)w_stop[k] * (double)h[k];
    *score = (float)s;
    for (int side = 0; side < 2; ++side) {
        for (int j = 0; j < H; ++j) {
            double g[4];
            for (int q = 0; q < 4; ++q) {
                const int col = side * 4 * H + q * H + j;
                double acc = b_td[col];
                for (int k = 0; k < H; ++k) acc += (double)h[k] * (double)u_td[(size_t)k * 8 * H + col];
                g[q] = acc;
            }
            const double cc = sigm(g[1]) * (double)c[j] + sigm(g[0]) * tanh(g[3]);
            child_c[side * H + j] = (float)cc;
            child_h[side * H + j] = (float)(sigm(g[2]) * tanh(cc));
        }
    }
}

/*
 * oracle_td_generate: grows n_trees trees breadth first.  Node t < n_trees is the root of tree t with
 * the given state (rows of h_root / c_root); children get the next two free indices, left first, in the
 * order in which their parents are visited (index order).  A node that would expand when fewer than two
 * of the max_nodes rows are free stays a leaf and is counted in *truncated.
 * Outputs, max_nodes rows each: parent (-1 for roots), left / right (-1 for nodes without children),
 * depth, score, h, c.  Returns the number of nodes, or -1 on bad arguments.
 */
int oracle_td_generate(int H, const float *u_td, const float *b_td, const float *w_stop, float b_stop,
                       int n_trees, const float *h_root, const float *c_root, int max_depth, int max_nodes,
                       int32_t *parent, int32_t *left, int32_t *right, int32_t *depth, float *score,
                       float *h, float *c, int32_t *truncated)
{
    if (H < 1 || n_trees < 1 || max_nodes < n_trees || max_depth < 0) return -1;
    float *kid_h = malloc(sizeof(float) * 2 * (size_t)H), *kid_c = malloc(sizeof(float) * 2 * (size_t)H);
    int n = n_trees;
    *truncated = 0;
    for (int t = 0; t < n_trees; ++t) {
        parent[t] = -1;
        depth[t] = 0;
        memcpy(h + (size_t)t * H, h_root + (size_t)t * H, sizeof(float) * (size_t)H);
        memcpy(c + (size_t)t * H, c_root + (size_t)t * H, sizeof(float) * (size_t)H);
    }
    for (int v = 0; v < n; ++v) {                 /* index order is breadth-first order */
        oracle_td_step(H, u_td, b_td, w_stop, b_stop, h + (size_t)v * H, c + (size_t)v * H, kid_h, kid_c, &score[v]);
        left[v] = right[v] = -1;
        if (!(score[v] > 0.0f) || depth[v] >= max_depth) continue;
        if (n + 2 > max_nodes) { *truncated += 1; continue; }
        for (int side = 0; side < 2; ++side) {
            const int k = n + side;
            parent[k] = v;
            depth[k] = depth[v] + 1;
            memcpy(h + (size_t)k * H, kid_h + (size_t)side * H, sizeof(float) * (size_t)H);
            memcpy(c + (size_t)k * H, kid_c + (size_t)side * H, sizeof(float) * (size_t)H);
        }
        left[v] = n;
        right[v] = n + 1;
        n += 2;
    }
    free(kid_h); free(kid_c);
    return n;
}

/*
 * Backward pass of the TreeRNN forward (leaf h = x, internal h = tanh([h_l ; h_r] W + b)) for a loss
 * that may touch every node: g_h[n] = dL/dh[n] from outside; a node's total dh is g_h[n] plus what its
 * parent sends down.  With a = [h_l ; h_r]:
 *   internal:  dpre = dh * (1 - h^2)      [dh_l ; dh_r] (sent down) = dpre W^T      dW += a^T dpre      db += dpre
 *   leaf:      d_x[n] = dh                (the embedding row is the state itself)
 * h is the stored fp32 forward state; sums in double, rounded to fp32 once.  d_x is [n_nodes x H], rows of
 * internal nodes zero.  Returns 0, or -1 on a malformed batch.
 * Pinned by tests against torch autograd on an independent float64 evaluation and finite differences.
 */
typedef struct {
    int H;
    const float *w, *h, *g_h;
    const int32_t *left, *right;
    double *d_w, *d_b;
    float *d_x;
} bwd_rnn_t;

static void backward_rnn_node(const bwd_rnn_t *m, int n, const double *dh, double *scratch)
{
    const int H = m->H;
    if (m->left[n] < 0) {
        for (int j = 0; j < H; ++j) m->d_x[(size_t)n * H + j] = (float)dh[j];
        return;
    }
    const int l = m->left[n], r = m->right[n];
    double *dpre = scratch, *dhl = dpre + H, *dhr = dhl + H, *next = dhr + H;
    for (int j = 0; j < H; ++j) {
        const double hv = m->h[(size_t)n * H + j];
        dpre[j] = dh[j] * (1.0 - hv * hv);
        m->d_b[j] += dpre[j];
    }
    for (int k = 0; k < 2 * H; ++k) {
        const double ak = k < H ? m->h[(size_t)l * H + k] : m->h[(size_t)r * H + (k - H)];
        const float *row = m->w + (size_t)k * H;
        double s = 0.0;
        for (int j = 0; j < H; ++j) {
            s += dpre[j] * (double)row[j];
            m->d_w[(size_t)k * H + j] += ak * dpre[j];
        }
        if (k < H) dhl[k] = s + (double)m->g_h[(size_t)l * H + k];
        else dhr[k - H] = s + (double)m->g_h[(size_t)r * H + (k - H)];
    }
    backward_rnn_node(m, l, dhl, next);
    backward_rnn_node(m, r, dhr, next);
}

int oracle_backward_rnn(int H, const float *w, int n_trees, int n_nodes, const int32_t *tree_off,
                        const int32_t *left, const int32_t *right, const float *h, const float *g_h,
                        float *d_w, float *d_b, float *d_x)
{
    int32_t *parent = malloc(sizeof(int32_t) * (size_t)(n_nodes > 0 ? n_nodes : 1));
    int32_t *height = malloc(sizeof(int32_t) * (size_t)(n_nodes > 0 ? n_nodes : 1));
    int32_t *root = malloc(sizeof(int32_t) * (size_t)(n_trees > 0 ? n_trees : 1));
    int rc = oracle_structure(n_trees, n_nodes, tree_off, left, right, parent, root, height);
    if (rc == 0) {
        const size_t nw = (size_t)2 * H * H;
        bwd_rnn_t m = { H, w, h, g_h, left, right, calloc(nw, sizeof(double)), calloc((size_t)H, sizeof(double)), d_x };
        memset(d_x, 0, sizeof(float) * (size_t)n_nodes * H);
        int max_h = 0;
        for (int t = 0; t < n_trees; ++t) if (height[root[t]] > max_h) max_h = height[root[t]];
        double *scratch = malloc(sizeof(double) * (size_t)3 * H * (size_t)(max_h + 2));
        double *dh = malloc(sizeof(double) * (size_t)H);
        for (int t = 0; t < n_trees; ++t) {
            for (int j = 0; j < H; ++j) dh[j] = (double)g_h[(size_t)root[t] * H + j];
            backward_rnn_node(&m, root[t], dh, scratch);
        }
        for (size_t i = 0; i < nw; ++i) d_w[i] = (float)m.d_w[i];
        for (int j = 0; j < H; ++j) d_b[j] = (float)m.d_b[j];
        free(m.d_w); free(m.d_b); free(scratch); free(dh);
    }
    free(parent); free(height); free(root);
    return rc;
}

/*
 * Backward pass of the RNTN forward (leaf h = x, internal h_k = tanh(a^T V_k a + (a W)_k + b_k), a = [h_l ; h_r],
 * V of shape d x 2d x 2d) for a loss that may touch every node (g_h[n] = dL/dh[n] from outside):
 *   internal:  dz = dh * (1 - h^2)
 *              da_p = sum_k dz_k ( sum_q (V[k][p][q] + V[k][q][p]) a_q + W[p][k] )      sent down to the children
 *              dV[k][p][q] += dz_k a_p a_q       dW[p][k] += a_p dz_k       db_k += dz_k
 *   leaf:      d_x[n] = dh
 * h is the stored fp32 forward state; sums in double, rounded to fp32 once.  d_x is [n_nodes x d], rows of internal
 * nodes zero.  Returns 0, or -1 on a malformed batch.
 * Pinned by tests against torch autograd on an independent float64 evaluation and finite differences.
 */
typedef struct {
    int H;
    const float *w, *v, *h, *g_h;
    const int32_t *left, *right;
    double *d_w, *d_b, *d_v;
    float *d_x;
} bwd_rntn_t;

static void backward_rntn_node(const bwd_rntn_t *m, int n, const double *dh, double *scratch)
{
    const int H = m->H, D2 = 2 * H;
    if (m->left[n] < 0) {
        for (int j = 0; j < H; ++j) m->d_x[(size_t)n * H + j] = (float)dh[j];
        return;
    }
    const int l = m->left[n], r = m->right[n];
    double *dz = scratch, *a = dz + H, *da = a + D2, *next = da + D2;
    for (int k = 0; k < H; ++k) {
        const double hv = m->h[(size_t)n * H + k];
        dz[k] = dh[k] * (1.0 - hv * hv);
        m->d_b[k] += dz[k];
    }
    for (int p = 0; p < D2; ++p) a[p] = p < H ? m->h[(size_t)l * H + p] : m->h[(size_t)r * H + (p - H)];
    for (int p = 0; p < D2; ++p) {
        double s = 0.0;
        for (int k = 0; k < H; ++k) {
            s += dz[k] * (double)m->w[(size_t)p * H + k];
            m->d_w[(size_t)p * H + k] += a[p] * dz[k];
        }
        da[p] = s;
    }
    for (int k = 0; k < H; ++k) {
        const float *Vk = m->v + (size_t)k * D2 * D2;
        double *dVk = m->d_v + (size_t)k * D2 * D2;
        for (int p = 0; p < D2; ++p)
            for (int q = 0; q < D2; ++q) {
                const double vpq = Vk[(size_t)p * D2 + q];
                da[p] += dz[k] * vpq * a[q];
                da[q] += dz[k] * vpq * a[p];
                dVk[(size_t)p * D2 + q] += dz[k] * a[p] * a[q];
            }
    }
    double *dhl = next, *dhr = dhl + H, *deeper = dhr + H;
    for (int j = 0; j < H; ++j) {
        dhl[j] = da[j] + (double)m->g_h[(size_t)l * H + j];
        dhr[j] = da[H + j] + (double)m->g_h[(size_t)r * H + j];
    }
    backward_rntn_node(m, l, dhl, deeper);
    backward_rntn_node(m, r, dhr, deeper);
}

int oracle_backward_rntn(int H, const float *w, const float *v, int n_trees, int n_nodes, const int32_t *tree_off,
                         const int32_t *left, const int32_t *right, const float *h, const float *g_h,
                         float *d_w, float *d_b, float *d_v, float *d_x)
{
    int32_t *parent = malloc(sizeof(int32_t) * (size_t)(n_nodes > 0 ? n_nodes : 1));
    int32_t *height = malloc(sizeof(int32_t) * (size_t)(n_nodes > 0 ? n_nodes : 1));
    int32_t *root = malloc(sizeof(int32_t) * (size_t)(n_trees > 0 ? n_trees : 1));
    int rc = oracle_structure(n_trees, n_nodes, tree_off, left, right, parent, root, height);
    if (rc == 0) {
        const size_t nw = (size_t)2 * H * H, nv = (size_t)H * 2 * H * 2 * H;
        bwd_rntn_t m = { H, w, v, h, g_h, left, right, calloc(nw, sizeof(double)), calloc((size_t)H, sizeof(double)),
                         calloc(nv, sizeof(double)), d_x };
        memset(d_x, 0, sizeof(float) * (size_t)n_nodes * H);
        int max_h = 0;
        for (int t = 0; t < n_trees; ++t) if (height[root[t]] > max_h) max_h = height[root[t]];
        double *scratch = malloc(sizeof(double) * (size_t)7 * H * (size_t)(max_h + 2));     /* dz, a, da, dhl, dhr per level */
        double *dh = malloc(sizeof(double) * (size_t)H);
        for (int t = 0; t < n_trees; ++t) {
            for (int j = 0; j < H; ++j) dh[j] = (double)g_h[(size_t)root[t] * H + j];
            backward_rntn_node(&m, root[t], dh, scratch);
        }
        for (size_t i = 0; i < nw; ++i) d_w[i] = (float)m.d_w[i];
        for (int j = 0; j < H; ++j) d_b[j] = (float)m.d_b[j];
        for (size_t i = 0; i < nv; ++i) d_v[i] = (float)m.d_v[i];
        free(m.d_w); free(m.d_b); free(m.d_v); free(scratch); free(dh);
    }
    free(parent); free(height); free(root);
    return rc;
}
