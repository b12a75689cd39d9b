// C ABI of the tree-network forward library (see include/treelstm.h).
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "treelstm.h"
#include "common.hpp"
#include "pack.hpp"
#include "structure.hpp"
#include "cell_tile.hpp"
#include "schedulers.hpp"
#include "classify.hpp"
#include "backward.hpp"
#include "topdown.hpp"

using namespace tl;

namespace {

constexpr int DEFAULT_SPIN_LIMIT = 1 << 20;
constexpr int LEVELS_AHEAD = 66;                // offsets of the per-height lists read back before the number of heights is known
constexpr int BW_PERSISTENT_MIN_LEVELS = 64;    // heights from which the backward pass walks them in one persistent kernel rather than in launches per height
constexpr int FLOW_LARGE_TREE_NODES = 256;      // mean nodes per tree from which a batch of fewer trees than sets of workgroups has the device pick its kernel

struct DevBuf {
    void *p = nullptr;
    size_t bytes = 0;
};

}  // namespace

struct tl_ctx {
    tl_config cfg{};
    int device = 0;
    int n_cu = 0;
    int n_cg = 0;
    // packed parameters
    float *emb = nullptr;
    void *wp_leaf = nullptr, *wp_inner = nullptr;
    float *bp_leaf = nullptr, *bp_inner = nullptr;
    Gemm g_leaf{}, g_inner{};
    // workspace
    unsigned char *ws = nullptr;
    size_t ws_bytes = 0;
    struct Resident { const void *kernel; size_t lds; int per_cu; };
    std::vector<Resident> resident;    // workgroups per compute unit of the persistent kernel variants launched so far
    unsigned char *flow_ws = nullptr;  // data-flow scheduler: per-column-group counters and lists, for cap_nodes nodes
    unsigned char *scratch = nullptr;  // this device's copy of the fixed workspace of tl_forward_noalloc (not owned)
    int cap_nodes = 0, cap_trees = 0;
    int32_t *host_levels = nullptr;   // pinned, cap_nodes + 2
    Ctl *host_ctl = nullptr;          // pinned
    Fwd last{};                       // pointers of the last forward (workspace part is reused)
    hipStream_t last_stream = nullptr;
    bool ran = false;
    int persistent_grid = 0;          // workgroups of the persistent kernels (streaming cell)
    int spw = 0;                      // k-steps per wave of the weight-stationary cell, 0 = not used
    int ws_grid = 0;                  // workgroups of the persistent kernels (weight-stationary cell)
    size_t ws_lds = 0;                // their LDS bytes
    int spw_leaf = 0;                 // k-steps per wave of the weight-stationary leaf kernel, 0 = streaming tiles
    int leaf_grid = 0;
    int es = 0;                       // row stride of the bf16 copy of the embedding table
    unsigned short *embb = nullptr;
    int hs = 0;                       // row stride of the bf16 copy of h
    unsigned short *hb = nullptr;     // bf16 copy of h, cap_nodes rows (bf16 weight-stationary cell only)
    // backward pass (TreeLSTM, fp32): transposed weights packed like the forward ones, workspace
    void *wp_bwd_inner = nullptr, *wp_bwd_leaf = nullptr, *wp_bwd_inner1 = nullptr;
    float *bp_bwd_inner = nullptr, *bp_bwd_leaf = nullptr, *bp_bwd_inner1 = nullptr;
    int bw_grid = 0;                  // workgroups of the backward kernel that walks all heights (0: per-height launches)
    int bw_ws_grid = 0, bw_spw2 = 0;  // ... of its form with the operand gradient on weight-stationary workgroups (0: none)
    Gemm g_bwd_inner1{};              // U^T once more with one column block per group: more workgroups for heights of few rows
    Gemm g_bwd_inner{}, g_bwd_leaf{};
    int ng_bwd_inner = 1, ng_bwd_leaf = 1;    // blocks of output columns per column group of the operand-gradient contractions
    float *bw = nullptr;              // dh | dc | gate gradients of internal nodes | of leaves
    int bw_nodes = 0;
    float *m_u = nullptr, *m_b = nullptr, *m_w_leaf = nullptr, *m_b_leaf = nullptr;   // fp32 TreeLSTM: the parameters themselves
    float *t_scratch = nullptr, *zero_bias = nullptr;
    float *m_v = nullptr;             // fp32 RNTN: the tensor V as given
    float *rntn_part = nullptr;       // RNTN forward: scratch area of the parts of a tile's sums, see cell_rntn.hpp
    unsigned int *rntn_done = nullptr;
    int rntn_units = 0;
    float *rntn_acc = nullptr;        // RNTN backward: [2d x (d * 2d + d)] weight-gradient contraction and its column sums
    int ws_steps16 = 0;
    bool keep_gates = false;          // tl_set_keep_gates
    int async_backward = 0;           // tl_set_async_backward: 1 never waits, -1 always launches per height, 0 picks by the number of heights
    float *gates = nullptr;           // [gates_cap x 5H] gate activations of the last forward that kept them
    int gates_cap = 0;
    int gates_nodes = 0;              // nodes of that forward, 0: nothing kept
    const float *gates_h = nullptr;   // its h argument: identifies the batch the activations belong to
    int last_grid = 0;
    int last_levels = 0;
    // profiling
    int profiling = 0;
    hipEvent_t ev[TL_PROFILE_RING][TL_N_STAGES]{};   // created on first use
    hipEvent_t ev_ctl = nullptr;      // tl_backward: behind the copy of the structure pass's status, in front of the kernels that do not need the host
    long long n_recorded = 0;                        // forwards recorded since profiling was switched on
};

// Context of the top-down generator (tl_td_*).
struct tl_td_ctx {
    int device = 0, n_cu = 0, H = 0, n_cg = 0, spin_limit = 0;
    int spw = 0;                      // k-steps per wave of the weight-stationary expansion step (0: streaming cell only)
    int flow_grid = 0;                // workgroups of the data-flow form that are resident together (0: that form is not used)
    tl::Gemm side[2]{};
    void *wp[2] = {nullptr, nullptr};
    float *bp[2] = {nullptr, nullptr};
    float *w_stop = nullptr;
    float b_stop = 0.f;
    float *zeros = nullptr;
    tl::Ctl *ctl = nullptr;
    tl::Ctl *host_ctl = nullptr;      // pinned
    hipStream_t last_stream = nullptr;
    bool ran = false;
};

namespace {

#define TL_HIP(call)                                   \
    do {                                               \
        hipError_t e_ = (call);                        \
        if (e_ != hipSuccess) return hip_fail(e_);     \
    } while (0)

int hip_fail(hipError_t e)
{
    if (getenv("TL_DEBUG")) fprintf(stderr, "treelstm: HIP error: %s\n", hipGetErrorString(e));
    return e == hipErrorOutOfMemory ? TL_ENOMEM : TL_EHIP;
}

inline int round_up(int x, int m) { return (x + m - 1) / m * m; }

typedef void (*fwd_kernel)(Fwd);
typedef void (*tiles_kernel)(Fwd, const int32_t *, int, LevelPlan);
typedef void (*wgrad_kernel)(Fwd, const int32_t *, int, const float *, int, const float *, int, float *, float *);

// Steps per wave that the weight-stationary cell is instantiated for; 0 = streaming cell.
const int WS_SIZES[] = {1, 2, 4, 5, 8, 16};
// Same for bf16 operands, in k-steps of 32.
const int WSB_SIZES[] = {1, 2, 3, 4, 6, 8};

template <int EPI> fwd_kernel ready_kernel_epi(bool vec4, int spw, bool bf16)
{
    if (bf16) {
        switch (spw) {
        case 1: return k_ready_persistent<EPI, true, 1, true>;
        case 2: return k_ready_persistent<EPI, true, 2, true>;
        case 3: return k_ready_persistent<EPI, true, 3, true>;
        case 4: return k_ready_persistent<EPI, true, 4, true>;
        case 6: return k_ready_persistent<EPI, true, 6, true>;
        case 8: return k_ready_persistent<EPI, true, 8, true>;
        default: return vec4 ? k_ready_persistent<EPI, true, 0, true> : k_ready_persistent<EPI, false, 0, true>;
        }
    }
    switch (spw) {
    case 1: return vec4 ? k_ready_persistent<EPI, true, 1> : k_ready_persistent<EPI, false, 1>;
    case 2: return vec4 ? k_ready_persistent<EPI, true, 2> : k_ready_persistent<EPI, false, 2>;
    case 4: return vec4 ? k_ready_persistent<EPI, true, 4> : k_ready_persistent<EPI, false, 4>;
    case 5: return vec4 ? k_ready_persistent<EPI, true, 5> : k_ready_persistent<EPI, false, 5>;
    case 8: return vec4 ? k_ready_persistent<EPI, true, 8> : k_ready_persistent<EPI, false, 8>;
    case 16: return vec4 ? k_ready_persistent<EPI, true, 16> : k_ready_persistent<EPI, false, 16>;
    default: return vec4 ? k_ready_persistent<EPI, true, 0> : k_ready_persistent<EPI, false, 0>;
    }
}
template <int EPI> fwd_kernel levels_kernel_epi(bool vec4, int spw, bool bf16)
{
    if (bf16) {
        switch (spw) {
        case 1: return k_levels_persistent<EPI, true, 1, true>;
        case 2: return k_levels_persistent<EPI, true, 2, true>;
        case 3: return k_levels_persistent<EPI, true, 3, true>;
        case 4: return k_levels_persistent<EPI, true, 4, true>;
        case 6: return k_levels_persistent<EPI, true, 6, true>;
        case 8: return k_levels_persistent<EPI, true, 8, true>;
        default: return vec4 ? k_levels_persistent<EPI, true, 0, true> : k_levels_persistent<EPI, false, 0, true>;
        }
    }
    switch (spw) {
    case 1: return vec4 ? k_levels_persistent<EPI, true, 1> : k_levels_persistent<EPI, false, 1>;
    case 2: return vec4 ? k_levels_persistent<EPI, true, 2> : k_levels_persistent<EPI, false, 2>;
    case 4: return vec4 ? k_levels_persistent<EPI, true, 4> : k_levels_persistent<EPI, false, 4>;
    case 5: return vec4 ? k_levels_persistent<EPI, true, 5> : k_levels_persistent<EPI, false, 5>;
    case 8: return vec4 ? k_levels_persistent<EPI, true, 8> : k_levels_persistent<EPI, false, 8>;
    case 16: return vec4 ? k_levels_persistent<EPI, true, 16> : k_levels_persistent<EPI, false, 16>;
    default: return vec4 ? k_levels_persistent<EPI, true, 0> : k_levels_persistent<EPI, false, 0>;
    }
}
template <int EPI> fwd_kernel flow_kernel_epi(bool vec4, int spw, bool bf16)
{
    if (bf16) {
        switch (spw) {
        case 1: return k_flow_persistent<EPI, true, 1, true>;
        case 2: return k_flow_persistent<EPI, true, 2, true>;
        case 3: return k_flow_persistent<EPI, true, 3, true>;
        case 4: return k_flow_persistent<EPI, true, 4, true>;
        case 6: return k_flow_persistent<EPI, true, 6, true>;
        default: return k_flow_persistent<EPI, true, 8, true>;
        }
    }
    switch (spw) {
    case 1: return vec4 ? k_flow_persistent<EPI, true, 1> : k_flow_persistent<EPI, false, 1>;
    case 2: return vec4 ? k_flow_persistent<EPI, true, 2> : k_flow_persistent<EPI, false, 2>;
    case 4: return vec4 ? k_flow_persistent<EPI, true, 4> : k_flow_persistent<EPI, false, 4>;
    case 5: return vec4 ? k_flow_persistent<EPI, true, 5> : k_flow_persistent<EPI, false, 5>;
    case 8: return vec4 ? k_flow_persistent<EPI, true, 8> : k_flow_persistent<EPI, false, 8>;
    default: return vec4 ? k_flow_persistent<EPI, true, 16> : k_flow_persistent<EPI, false, 16>;
    }
}
// spw > 0 and not the RNTN cell
fwd_kernel flow_kernel(int cell, bool vec4, int spw, bool bf16)
{
    return cell == TL_TREELSTM ? flow_kernel_epi<EPI_LSTM_INNER>(vec4, spw, bf16) : flow_kernel_epi<EPI_RNN_INNER>(vec4, spw, bf16);
}
fwd_kernel ready_kernel(int cell, bool vec4, int spw, bool bf16)
{
    if (cell == TL_RNTN) return vec4 ? k_ready_persistent<EPI_RNTN_INNER, true, 0> : k_ready_persistent<EPI_RNTN_INNER, false, 0>;
    return cell == TL_TREELSTM ? ready_kernel_epi<EPI_LSTM_INNER>(vec4, spw, bf16) : ready_kernel_epi<EPI_RNN_INNER>(vec4, spw, bf16);
}
fwd_kernel levels_kernel(int cell, bool vec4, int spw, bool bf16)
{
    if (cell == TL_RNTN) return vec4 ? k_levels_persistent<EPI_RNTN_INNER, true, 0> : k_levels_persistent<EPI_RNTN_INNER, false, 0>;
    return cell == TL_TREELSTM ? levels_kernel_epi<EPI_LSTM_INNER>(vec4, spw, bf16) : levels_kernel_epi<EPI_RNN_INNER>(vec4, spw, bf16);
}
fwd_kernel leaf_ws_kernel(int spw)
{
    switch (spw) {
    case 1: return k_leaf_ws<1>;
    case 2: return k_leaf_ws<2>;
    case 4: return k_leaf_ws<4>;
    case 5: return k_leaf_ws<5>;
    case 8: return k_leaf_ws<8>;
    case 16: return k_leaf_ws<16>;
    default: return nullptr;
    }
}
fwd_kernel leaf_ws_bf_kernel(int s)
{
    switch (s) {
    case 1: return k_leaf_ws_bf<1>;
    case 2: return k_leaf_ws_bf<2>;
    case 3: return k_leaf_ws_bf<3>;
    case 4: return k_leaf_ws_bf<4>;
    case 6: return k_leaf_ws_bf<6>;
    case 8: return k_leaf_ws_bf<8>;
    default: return nullptr;
    }
}
// LDS bytes of the weight-stationary kernels
// LDS of the leaf kernel: the bf16 form has a leaner layout of its own (three gates, no scheduler tables)
size_t leaf_lds_bytes(int spw, bool bf16);
size_t ws_lds_bytes(int spw, bool bf16)
{
    if (bf16) {
        switch (spw) {
        case 1: return sizeof(WsSmemBfT<1>);
        case 2: return sizeof(WsSmemBfT<2>);
        case 3: return sizeof(WsSmemBfT<3>);
        case 4: return sizeof(WsSmemBfT<4>);
        case 6: return sizeof(WsSmemBfT<6>);
        default: return sizeof(WsSmemBfT<8>);
        }
    }
    switch (spw) {
    case 1: return sizeof(WsSmemT<1>);
    case 2: return sizeof(WsSmemT<2>);
    case 4: return sizeof(WsSmemT<4>);
    case 5: return sizeof(WsSmemT<5>);
    case 8: return sizeof(WsSmemT<8>);
    default: return sizeof(WsSmemT<16>);
    }
}
size_t leaf_lds_bytes(int spw, bool bf16)
{
    if (!bf16) return ws_lds_bytes(spw, false);
    switch (spw) {
    case 1: return sizeof(LeafSmemBf<1>);
    case 2: return sizeof(LeafSmemBf<2>);
    case 3: return sizeof(LeafSmemBf<3>);
    case 4: return sizeof(LeafSmemBf<4>);
    case 6: return sizeof(LeafSmemBf<6>);
    default: return sizeof(LeafSmemBf<8>);
    }
}
template <bool BF16> tiles_kernel static_kernel_p(int epi, bool vec4)
{
    switch (epi) {
    case EPI_LSTM_LEAF: return vec4 ? k_tiles_static<EPI_LSTM_LEAF, true, BF16> : k_tiles_static<EPI_LSTM_LEAF, false, BF16>;
    case EPI_LSTM_INNER: return vec4 ? k_tiles_static<EPI_LSTM_INNER, true, BF16> : k_tiles_static<EPI_LSTM_INNER, false, BF16>;
    default: return vec4 ? k_tiles_static<EPI_RNN_INNER, true, BF16> : k_tiles_static<EPI_RNN_INNER, false, BF16>;
    }
}
tiles_kernel backward_kernel(int epi, bool vec4)
{
    switch (epi) {
    case EPI_BWD_INNER_GATES: return vec4 ? k_tiles_static<EPI_BWD_INNER_GATES, true, false> : k_tiles_static<EPI_BWD_INNER_GATES, false, false>;
    case EPI_BWD_INNER_OPERAND: return vec4 ? k_tiles_static<EPI_BWD_INNER_OPERAND, true, false> : k_tiles_static<EPI_BWD_INNER_OPERAND, false, false>;
    case EPI_BWD_LEAF_GATES: return vec4 ? k_tiles_static<EPI_BWD_LEAF_GATES, true, false> : k_tiles_static<EPI_BWD_LEAF_GATES, false, false>;
    case EPI_BWD_INNER_OPERAND4: return vec4 ? k_tiles_static<EPI_BWD_INNER_OPERAND4, true, false> : k_tiles_static<EPI_BWD_INNER_OPERAND4, false, false>;
    case EPI_BWD_LEAF_OPERAND4: return vec4 ? k_tiles_static<EPI_BWD_LEAF_OPERAND4, true, false> : k_tiles_static<EPI_BWD_LEAF_OPERAND4, false, false>;
    default: return vec4 ? k_tiles_static<EPI_BWD_LEAF_OPERAND, true, false> : k_tiles_static<EPI_BWD_LEAF_OPERAND, false, false>;
    }
}
tiles_kernel static_kernel(int epi, bool vec4, bool bf16)
{
    if (epi == EPI_RNTN_INNER) return vec4 ? k_tiles_static<EPI_RNTN_INNER, true, false> : k_tiles_static<EPI_RNTN_INNER, false, false>;
    return bf16 ? static_kernel_p<true>(epi, vec4) : static_kernel_p<false>(epi, vec4);
}

template <typename K> int allow_lds(K kernel, size_t bytes = TILE_SMEM_BYTES)
{
    TL_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
    return TL_OK;
}

// Packs one weight matrix [SEG*L x NG*H] and its bias; fills the Gemm descriptor.
// If *wp_out / *bp_out are set they are packed over (the sizes depend only on the shapes), else allocated.
int pack_gemm(const float *w, const float *b, int NG, int H, int SEG, int L, int n_cg, int min_steps, bool bf16, Gemm *g,
              void **wp_out, float **bp_out, hipStream_t st = nullptr)
{
    // bf16: segments start at multiples of 8 elements (16 bytes of a bf16 row) and the K axis is a
    // multiple of 4 k-steps of 32, so that it splits into four quarters of whole k-steps
    const int Lp = round_up(L, bf16 ? 8 : 4);
    int Kp = round_up(SEG * Lp, bf16 ? 128 : KC);
    if (Kp < min_steps * STEP_K) Kp = min_steps * STEP_K;   // the weight-stationary cell wants exactly 4 * SPW k-steps
    const int n_steps = Kp / STEP_K;
    const size_t n_w = (size_t)n_cg * n_steps * NG * 64 * 4;
    void *wp = *wp_out;
    float *bp = *bp_out;
    if (!wp) TL_HIP(hipMalloc(&wp, n_w * (bf16 ? sizeof(unsigned short) : sizeof(float))));
    *wp_out = wp;
    if (!bp) TL_HIP(hipMalloc(&bp, (size_t)n_cg * NG * HU * sizeof(float)));
    *bp_out = bp;
    if (bf16)
        hipLaunchKernelGGL(k_pack_bf16, dim3(1024), dim3(256), 0, st, w, (unsigned short *)wp, NG, H, SEG, L, Lp, n_steps / 2, n_cg);
    else
        hipLaunchKernelGGL(k_pack_f32, dim3(1024), dim3(256), 0, st, w, (float *)wp, NG, H, SEG, L, Lp, n_steps, n_cg);
    hipLaunchKernelGGL(k_pack_bias, dim3(64), dim3(256), 0, st, b, bp, NG, H, n_cg);
    TL_HIP(hipGetLastError());
    g->wp = wp;
    g->bp = bp;
    g->L = L;
    g->Lp = Lp;
    g->n_chunks = Kp / KC;
    return TL_OK;
}

// (Re-)packs everything that is derived from the fp32 TreeLSTM parameters kept in the context: forward weights of
// leaves and internal nodes, and the transposed weights of the backward pass.  Enqueued on st.
int pack_treelstm_f32(tl_ctx *ctx, hipStream_t st)
{
    const int H = ctx->cfg.hidden, E = ctx->cfg.embed_dim;
    int rc = pack_gemm(ctx->m_w_leaf, ctx->m_b_leaf, 3, H, 1, E, ctx->n_cg, 4 * ctx->spw_leaf, false, &ctx->g_leaf, &ctx->wp_leaf,
                       &ctx->bp_leaf, st);
    if (rc != TL_OK) return rc;
    rc = pack_gemm(ctx->m_u, ctx->m_b, 5, H, 2, H, ctx->n_cg, ctx->ws_steps16, false, &ctx->g_inner, &ctx->wp_inner, &ctx->bp_inner, st);
    if (rc != TL_OK) return rc;
    // backward pass: U^T [5H x 2H] and W_leaf^T [3H x E] as contractions with a zero bias
    float *t = ctx->t_scratch, *zb = ctx->zero_bias;
    hipLaunchKernelGGL(k_transpose, dim3(1024), dim3(256), 0, st, (const float *)ctx->m_u, t, 2 * H, 5 * H);
    rc = pack_gemm(t, zb, ctx->ng_bwd_inner, 2 * H / ctx->ng_bwd_inner, 1, 5 * H, (2 * H / ctx->ng_bwd_inner + HU - 1) / HU, 0, false,
                   &ctx->g_bwd_inner, &ctx->wp_bwd_inner, &ctx->bp_bwd_inner, st);
    if (rc != TL_OK) return rc;
    if (ctx->ng_bwd_inner == 4) {
        rc = pack_gemm(t, zb, 1, 2 * H, 1, 5 * H, (2 * H + HU - 1) / HU, 0, false, &ctx->g_bwd_inner1, &ctx->wp_bwd_inner1,
                       &ctx->bp_bwd_inner1, st);
        if (rc != TL_OK) return rc;
    }
    hipLaunchKernelGGL(k_transpose, dim3(1024), dim3(256), 0, st, (const float *)ctx->m_w_leaf, t, E, 3 * H);   // in stream order after the packs above
    rc = pack_gemm(t, zb, ctx->ng_bwd_leaf, E / ctx->ng_bwd_leaf, 1, 3 * H, (E / ctx->ng_bwd_leaf + HU - 1) / HU, 0, false,
                   &ctx->g_bwd_leaf, &ctx->wp_bwd_leaf, &ctx->bp_bwd_leaf, st);
    if (rc != TL_OK) return rc;
    TL_HIP(hipGetLastError());
    return TL_OK;
}

// One job of k_pack_many for a matrix that pack_gemm has packed before (g says how): [SEG * L x NG * H], from w as it is
// stored (row-major) or, transposed = true, from the stored [NG * H x SEG * L] matrix whose transpose it is.
PackJob repack_job(const Gemm &g, const float *w, const float *b, float *bp, int NG, int H, int SEG, int n_cg, bool transposed)
{
    PackJob j{};
    j.w = w; j.wp = (float *)const_cast<void *>(g.wp); j.b = b; j.bp = bp;
    j.NG = NG; j.H = H; j.SEG = SEG; j.L = g.L; j.Lp = g.Lp; j.n_steps = g.n_chunks * (KC / STEP_K); j.n_cg = n_cg;
    j.rs = transposed ? 1 : (long long)NG * H;
    j.cs = transposed ? (long long)SEG * g.L : 1;
    return j;
}

// After a parameter update of an fp32 TreeLSTM or TreeRNN context: everything pack_treelstm_f32 / pack_treernn_f32 derive
// from the parameters, packed over in one launch.
int repack_f32(tl_ctx *ctx, hipStream_t st)
{
    const int H = ctx->cfg.hidden, E = ctx->cfg.embed_dim;
    const bool lstm = ctx->cfg.cell == TL_TREELSTM;
    const int ng_cell = lstm ? 5 : 1;
    if (!ctx->wp_inner || !ctx->wp_bwd_inner || (lstm && (!ctx->wp_leaf || !ctx->wp_bwd_leaf))) return TL_EINVAL;
    PackList pl{};
    int n = 0;
    if (lstm) pl.job[n++] = repack_job(ctx->g_leaf, ctx->m_w_leaf, ctx->m_b_leaf, ctx->bp_leaf, 3, H, 1, ctx->n_cg, false);
    pl.job[n++] = repack_job(ctx->g_inner, ctx->m_u, ctx->m_b, ctx->bp_inner, ng_cell, H, 2, ctx->n_cg, false);
    // backward pass: U^T [ng_cell H x 2H] and W_leaf^T [3H x E]
    pl.job[n++] = repack_job(ctx->g_bwd_inner, ctx->m_u, nullptr, nullptr, ctx->ng_bwd_inner, 2 * H / ctx->ng_bwd_inner, 1,
                             (2 * H / ctx->ng_bwd_inner + HU - 1) / HU, true);
    if (ctx->ng_bwd_inner == 4)
        pl.job[n++] = repack_job(ctx->g_bwd_inner1, ctx->m_u, nullptr, nullptr, 1, 2 * H, 1, (2 * H + HU - 1) / HU, true);
    if (lstm)
        pl.job[n++] = repack_job(ctx->g_bwd_leaf, ctx->m_w_leaf, nullptr, nullptr, ctx->ng_bwd_leaf, E / ctx->ng_bwd_leaf, 1,
                                 (E / ctx->ng_bwd_leaf + HU - 1) / HU, true);
    pl.n = n;
    hipLaunchKernelGGL(k_pack_many, dim3(2048), dim3(256), 0, st, pl);
    TL_HIP(hipGetLastError());
    return TL_OK;
}

// The same for an fp32 TreeRNN context: forward weights and W^T of the backward pass.
int pack_treernn_f32(tl_ctx *ctx, hipStream_t st)
{
    const int H = ctx->cfg.hidden;
    int rc = pack_gemm(ctx->m_u, ctx->m_b, 1, H, 2, H, ctx->n_cg, ctx->ws_steps16, false, &ctx->g_inner, &ctx->wp_inner, &ctx->bp_inner, st);
    if (rc != TL_OK) return rc;
    float *t = ctx->t_scratch, *zb = ctx->zero_bias;
    hipLaunchKernelGGL(k_transpose, dim3(1024), dim3(256), 0, st, (const float *)ctx->m_u, t, 2 * H, H);
    rc = pack_gemm(t, zb, ctx->ng_bwd_inner, 2 * H / ctx->ng_bwd_inner, 1, H, (2 * H / ctx->ng_bwd_inner + HU - 1) / HU, 0, false,
                   &ctx->g_bwd_inner, &ctx->wp_bwd_inner, &ctx->bp_bwd_inner, st);
    if (rc != TL_OK) return rc;
    if (ctx->ng_bwd_inner == 4) {
        rc = pack_gemm(t, zb, 1, 2 * H, 1, H, (2 * H + HU - 1) / HU, 0, false, &ctx->g_bwd_inner1, &ctx->wp_bwd_inner1,
                       &ctx->bp_bwd_inner1, st);
        if (rc != TL_OK) return rc;
    }
    TL_HIP(hipGetLastError());
    return TL_OK;
}

// The same for an fp32 RNTN context: the forward's packed tensor slices, and the matrix S of the operand gradient
// (see backward.hpp) packed like transposed weights.
int pack_rntn_f32(tl_ctx *ctx, hipStream_t st)
{
    const int H = ctx->cfg.hidden, D2 = 2 * H, L = H * D2 + H;
    const int Lp = round_up(H, 4);
    int Kp = round_up(2 * Lp, KC);
    if (Kp > 128) Kp = 256;
    const size_t n_v = (size_t)ctx->n_cg * (Kp + 1) * (Kp / STEP_K) * 256;
    if (!ctx->wp_inner) TL_HIP(hipMalloc(&ctx->wp_inner, n_v * sizeof(float)));
    if (!ctx->bp_inner) TL_HIP(hipMalloc(&ctx->bp_inner, (size_t)ctx->n_cg * HU * sizeof(float)));
    hipLaunchKernelGGL(k_pack_rntn, dim3(2048), dim3(256), 0, st, (const float *)ctx->m_v, (const float *)ctx->m_u, (float *)ctx->wp_inner,
                       H, Lp, Kp, ctx->n_cg);
    hipLaunchKernelGGL(k_pack_bias, dim3(64), dim3(256), 0, st, (const float *)ctx->m_b, ctx->bp_inner, 1, H, ctx->n_cg);
    TL_HIP(hipGetLastError());
    ctx->g_inner.wp = ctx->wp_inner;
    ctx->g_inner.bp = ctx->bp_inner;
    ctx->g_inner.L = H;
    ctx->g_inner.Lp = Lp;
    ctx->g_inner.n_chunks = Kp / KC;
    hipLaunchKernelGGL(k_rntn_build_s, dim3(2048), dim3(256), 0, st, (const float *)ctx->m_v, (const float *)ctx->m_u, ctx->t_scratch, H);
    int rc = pack_gemm(ctx->t_scratch, ctx->zero_bias, ctx->ng_bwd_inner, D2 / ctx->ng_bwd_inner, 1, L,
                       (D2 / ctx->ng_bwd_inner + HU - 1) / HU, 0, false, &ctx->g_bwd_inner, &ctx->wp_bwd_inner, &ctx->bp_bwd_inner, st);
    if (rc != TL_OK) return rc;
    if (ctx->ng_bwd_inner == 4) {
        rc = pack_gemm(ctx->t_scratch, ctx->zero_bias, 1, D2, 1, L, (D2 + HU - 1) / HU, 0, false, &ctx->g_bwd_inner1, &ctx->wp_bwd_inner1,
                       &ctx->bp_bwd_inner1, st);
        if (rc != TL_OK) return rc;
    }
    TL_HIP(hipGetLastError());
    return TL_OK;
}

// Workgroups of `kernel` (with `lds` bytes of dynamic LDS) that one compute unit holds at a time; asked of the runtime
// once per kernel variant.
int resident_per_cu(tl_ctx *ctx, fwd_kernel kernel, size_t lds, int *out)
{
    for (const auto &r : ctx->resident)
        if (r.kernel == reinterpret_cast<const void *>(kernel) && r.lds == lds) { *out = r.per_cu; return TL_OK; }
    int n = 0;
    TL_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, reinterpret_cast<const void *>(kernel), WG_THREADS, lds));
    ctx->resident.push_back({reinterpret_cast<const void *>(kernel), lds, n});
    *out = n;
    return TL_OK;
}

constexpr size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Bytes of the workspace for batches of up to N nodes / B trees (carve_workspace cuts it up).
constexpr size_t workspace_bytes(size_t N, size_t B)
{
    return align256((N + 2) * 4) * 12 + align256(B * 4) + align256(sizeof(Ctl)) + align256(sizeof(GangBox) * MAX_GANGS) + 4096;
}

// Workspace of tl_forward_noalloc: one array per device, part of the loaded code object, so that the call has
// nothing to allocate.  First the workspace proper for TL_NOALLOC_MAX_NODES nodes (and as many trees), then room
// for the bf16 copy of h that the bf16 weight-stationary cell gathers from.  Host code must not use the name
// `scratch` as an address: tl_create asks the runtime for the array's address on its device (scratch_address).
constexpr size_t NOALLOC_WS_BYTES = workspace_bytes(TL_NOALLOC_MAX_NODES, TL_NOALLOC_MAX_NODES);
constexpr size_t NOALLOC_HB_BYTES = (size_t)TL_NOALLOC_MAX_NODES * 512 * sizeof(unsigned short);
static __device__ __align__(256) unsigned char scratch[NOALLOC_WS_BYTES + NOALLOC_HB_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex scratch_mutex;
unsigned char *scratch_of_device[MAX_DEVICES];

// Address of `scratch` on the current device (which must be `device`); looked up once per device.
int scratch_address(int device, unsigned char **out)
{
    *out = nullptr;
    if (device < 0 || device >= MAX_DEVICES) return TL_EINVAL;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_of_device[device]) {
        void *p = nullptr;
        TL_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return TL_EHIP;
        scratch_of_device[device] = static_cast<unsigned char *>(p);
    }
    *out = scratch_of_device[device];
    return TL_OK;
}

// Data-flow scheduler: counters [n_cg x N] (int32) followed by lists [n_cg x N / 2] of 16-byte entries.
size_t flow_bytes(size_t n_cg, size_t N) { return align256(n_cg * N * sizeof(int32_t)) + n_cg * (N / 2 + 1) * sizeof(int4); }

// Workspace for batches of up to n_nodes nodes / n_trees trees.
int ensure_workspace(tl_ctx *ctx, int n_nodes, int n_trees)
{
    if (n_nodes <= ctx->cap_nodes && n_trees <= ctx->cap_trees) return TL_OK;
    TL_HIP(hipDeviceSynchronize());
    const int N = n_nodes > ctx->cap_nodes ? n_nodes : ctx->cap_nodes;
    const int B = n_trees > ctx->cap_trees ? n_trees : ctx->cap_trees;
    if (ctx->ws) { TL_HIP(hipFree(ctx->ws)); ctx->ws = nullptr; }
    if (ctx->hb) { TL_HIP(hipFree(ctx->hb)); ctx->hb = nullptr; }
    if (ctx->flow_ws) { TL_HIP(hipFree(ctx->flow_ws)); ctx->flow_ws = nullptr; }
    if (ctx->host_levels) { TL_HIP(hipHostFree(ctx->host_levels)); ctx->host_levels = nullptr; }
    ctx->cap_nodes = ctx->cap_trees = 0;
    const size_t bytes = workspace_bytes((size_t)N, (size_t)B);
    TL_HIP(hipMalloc(&ctx->ws, bytes));
    TL_HIP(hipMemset(ctx->ws, 0, bytes));   // includes the block of zeros at the end, which is never written again
    if (ctx->spw > 0 && ctx->cfg.precision == TL_BF16_IN) {
        const size_t hb_bytes = (size_t)N * ctx->hs * sizeof(unsigned short);
        TL_HIP(hipMalloc(&ctx->hb, hb_bytes));
        TL_HIP(hipMemset(ctx->hb, 0, hb_bytes));   // the padding at the end of each row stays zero for good
    }
    if (ctx->spw > 0 && ctx->cfg.scheduler == TL_SCHED_DATAFLOW)
        TL_HIP(hipMalloc(&ctx->flow_ws, flow_bytes(ctx->n_cg, (size_t)N)));
    TL_HIP(hipHostMalloc(&ctx->host_levels, (size_t)(N + 2) * 4, hipHostMallocDefault));
    ctx->ws_bytes = bytes;
    ctx->cap_nodes = N;
    ctx->cap_trees = B;
    return TL_OK;
}

// Cuts a workspace of workspace_bytes(cap_nodes, cap_trees) bytes at `base` into the arrays of a forward.
void carve_workspace(unsigned char *base, int cap_nodes, int cap_trees, Fwd *f)
{
    const size_t n4 = align256((size_t)(cap_nodes + 2) * 4);
    unsigned char *p = base;
    auto take = [&](size_t b) { unsigned char *r = p; p += b; return r; };
    f->parent = (int32_t *)take(n4);
    f->pending = (int32_t *)take(n4);
    f->leaf_list = (int32_t *)take(n4);
    f->height = (int32_t *)take(n4);
    f->arrive = (int32_t *)take(n4);
    f->level_cnt = (int32_t *)take(n4);
    f->level_off = (int32_t *)take(n4);
    f->level_fill = (int32_t *)take(n4);
    f->level_nodes = (int32_t *)take(n4);
    f->q_rec = (QRec *)take(2 * n4);       // n_int <= N / 2 records of 16 bytes
    f->depth_root = (int32_t *)take(n4);
    f->root_ws = (int32_t *)take(align256((size_t)cap_trees * 4));
    f->ctl = (Ctl *)take(align256(sizeof(Ctl)));
    f->gangs = (GangBox *)take(align256(sizeof(GangBox) * MAX_GANGS));
    f->zeros = (const float *)take(4096);
}

void free_all(tl_ctx *ctx)
{
    (void)hipFree(ctx->emb);
    (void)hipFree(ctx->wp_leaf);
    (void)hipFree(ctx->wp_inner);
    (void)hipFree(ctx->bp_leaf);
    (void)hipFree(ctx->bp_inner);
    (void)hipFree(ctx->ws);
    (void)hipFree(ctx->hb);
    (void)hipFree(ctx->flow_ws);
    (void)hipFree(ctx->embb);
    (void)hipFree(ctx->wp_bwd_inner);
    (void)hipFree(ctx->wp_bwd_inner1);
    (void)hipFree(ctx->bp_bwd_inner1);
    (void)hipFree(ctx->wp_bwd_leaf);
    (void)hipFree(ctx->bp_bwd_inner);
    (void)hipFree(ctx->bp_bwd_leaf);
    (void)hipFree(ctx->bw);
    (void)hipFree(ctx->gates);
    (void)hipFree(ctx->m_u);
    (void)hipFree(ctx->m_b);
    (void)hipFree(ctx->m_w_leaf);
    (void)hipFree(ctx->m_b_leaf);
    (void)hipFree(ctx->t_scratch);
    (void)hipFree(ctx->zero_bias);
    (void)hipFree(ctx->m_v);
    (void)hipFree(ctx->rntn_acc);
    (void)hipFree(ctx->rntn_part);
    (void)hipFree(ctx->rntn_done);
    if (ctx->host_levels) (void)hipHostFree(ctx->host_levels);
    if (ctx->host_ctl) (void)hipHostFree(ctx->host_ctl);
    for (auto &set : ctx->ev)
        for (auto &e : set)
            if (e) (void)hipEventDestroy(e);
    if (ctx->ev_ctl) (void)hipEventDestroy(ctx->ev_ctl);
    delete ctx;
}

// The persistent backward kernel with the weight-stationary operand gradient, and the LDS it takes: TreeLSTM with
// 5 H / 128 = spw2 (H = 128, 256, 384, 512), TreeRNN with H / 128 = spw2 (the same sizes).
typedef void (*bwh_ws_kernel)(Fwd, BwdHeights);
bwh_ws_kernel backward_ws_kernel(bool lstm, int spw2, size_t *lds)
{
    if (lstm) {
        switch (spw2) {
        case 5:  *lds = sizeof(OperandWsSmem<5>);  return bwh_ws_kernel(k_backward_heights_ws<5, true>);
        case 10: *lds = sizeof(OperandWsSmem<10>); return bwh_ws_kernel(k_backward_heights_ws<10, true>);
        case 15: *lds = sizeof(OperandWsSmem<15>); return bwh_ws_kernel(k_backward_heights_ws<15, true>);
        case 20: *lds = sizeof(OperandWsSmem<20>); return bwh_ws_kernel(k_backward_heights_ws<20, true>);
        default: break;
        }
    } else {
        switch (spw2) {
        case 1: *lds = sizeof(OperandWsSmem<1>); return bwh_ws_kernel(k_backward_heights_ws<1, false>);
        case 2: *lds = sizeof(OperandWsSmem<2>); return bwh_ws_kernel(k_backward_heights_ws<2, false>);
        case 3: *lds = sizeof(OperandWsSmem<3>); return bwh_ws_kernel(k_backward_heights_ws<3, false>);
        case 4: *lds = sizeof(OperandWsSmem<4>); return bwh_ws_kernel(k_backward_heights_ws<4, false>);
        default: break;
        }
    }
    *lds = 0;
    return nullptr;
}

int create_impl(const tl_config *cfg, tl_ctx *ctx)
{
    ctx->cfg = *cfg;
    TL_HIP(hipGetDevice(&ctx->device));
    hipDeviceProp_t prop;
    TL_HIP(hipGetDeviceProperties(&prop, ctx->device));
    ctx->n_cu = prop.multiProcessorCount;
    const int H = cfg->hidden, E = cfg->embed_dim;
    ctx->n_cg = (H + HU - 1) / HU;

    const size_t emb_bytes = (size_t)cfg->vocab * E * sizeof(float);
    TL_HIP(hipMalloc(&ctx->emb, emb_bytes));
    TL_HIP(hipMemcpy(ctx->emb, cfg->emb, emb_bytes, hipMemcpyDeviceToDevice));

    // Weight-stationary cell.  fp32: needs 16-byte aligned rows (H % 4 == 0) and at most 16 k-steps of
    // 16 per wave; bf16: at most 8 k-steps of 32 per wave (its rows come from a padded bf16 copy of h).
    const bool bf16 = cfg->precision == TL_BF16_IN;
    ctx->spw = 0;
    ctx->hs = round_up(H, 8);
    if (cfg->cell != TL_RNTN) {
        if (bf16) {
            const int needed = round_up(2 * ctx->hs, 128) / 128;
            for (int sz : WSB_SIZES)
                if (sz >= needed) { ctx->spw = sz; break; }
        } else if (H % 2 == 0) {      // rows of h must be 8-byte aligned at least
            const int needed = round_up(2 * round_up(H, 4), KC) / STEP_K / 4;
            for (int sz : WS_SIZES)
                if (sz >= needed) { ctx->spw = sz; break; }
        }
    }
    const int ws_steps16 = bf16 ? 8 * ctx->spw : 4 * ctx->spw;   // K axis of the weight-stationary cell in k-steps of 16
    ctx->spw_leaf = 0;
    ctx->es = round_up(E, 8);
    const bool leaf_range = cfg->vocab < (1 << 24) && (unsigned long long)cfg->vocab * ctx->es * 4ull < (1ull << 32);
    if (cfg->cell == TL_TREELSTM && leaf_range) {
        if (bf16) {
            const int needed = round_up(ctx->es, 128) / 128;
            for (int sz : WSB_SIZES)
                if (sz >= needed) { ctx->spw_leaf = sz; break; }
        } else if (E % 4 == 0) {
            const int needed = round_up(E, KC) / STEP_K / 4;
            for (int sz : WS_SIZES)
                if (sz >= needed) { ctx->spw_leaf = sz; break; }
        }
    }
    if (bf16 && ctx->spw_leaf > 0) {
        TL_HIP(hipMalloc(&ctx->embb, (size_t)cfg->vocab * ctx->es * sizeof(unsigned short)));
        hipLaunchKernelGGL(k_pad_bf16, dim3(1024), dim3(256), 0, 0, cfg->emb, ctx->embb, (size_t)cfg->vocab, E, ctx->es);
        TL_HIP(hipGetLastError());
    }
    int rc;
    if (cfg->cell == TL_TREELSTM) {
        if (!bf16) {
            // fp32 TreeLSTM contexts keep the parameters as given (tl_backward / tl_sgd_update / tl_get_params), a
            // scratch matrix for the transposes and a zero bias for the operand-gradient contractions
            const size_t n_u = (size_t)2 * H * 5 * H, n_w = (size_t)E * 3 * H;
            TL_HIP(hipMalloc(&ctx->m_u, n_u * sizeof(float)));
            TL_HIP(hipMalloc(&ctx->m_b, (size_t)5 * H * sizeof(float)));
            TL_HIP(hipMalloc(&ctx->m_w_leaf, n_w * sizeof(float)));
            TL_HIP(hipMalloc(&ctx->m_b_leaf, (size_t)3 * H * sizeof(float)));
            TL_HIP(hipMemcpy(ctx->m_u, cfg->u, n_u * sizeof(float), hipMemcpyDeviceToDevice));
            TL_HIP(hipMemcpy(ctx->m_b, cfg->b, (size_t)5 * H * sizeof(float), hipMemcpyDeviceToDevice));
            TL_HIP(hipMemcpy(ctx->m_w_leaf, cfg->w_leaf, n_w * sizeof(float), hipMemcpyDeviceToDevice));
            TL_HIP(hipMemcpy(ctx->m_b_leaf, cfg->b_leaf, (size_t)3 * H * sizeof(float), hipMemcpyDeviceToDevice));
            TL_HIP(hipMalloc(&ctx->t_scratch, (n_u > n_w ? n_u : n_w) * sizeof(float)));
            const size_t n_zb = (size_t)(2 * H > E ? 2 * H : E) + HU;
            TL_HIP(hipMalloc(&ctx->zero_bias, n_zb * sizeof(float)));
            TL_HIP(hipMemset(ctx->zero_bias, 0, n_zb * sizeof(float)));
            // output columns in four blocks per column group where the width allows it (see EPI_BWD_INNER_OPERAND4)
            ctx->ng_bwd_inner = (2 * H) % 4 == 0 ? 4 : 1;
            ctx->ng_bwd_leaf = E % 4 == 0 ? 4 : 1;
            ctx->ws_steps16 = ws_steps16;
            rc = pack_treelstm_f32(ctx, nullptr);
            TL_HIP(hipDeviceSynchronize());
            if (rc != TL_OK) return rc;
        } else {
            rc = pack_gemm(cfg->w_leaf, cfg->b_leaf, 3, H, 1, E, ctx->n_cg, 8 * ctx->spw_leaf, true, &ctx->g_leaf, &ctx->wp_leaf, &ctx->bp_leaf);
            if (rc != TL_OK) return rc;
            rc = pack_gemm(cfg->u, cfg->b, 5, H, 2, H, ctx->n_cg, ws_steps16, true, &ctx->g_inner, &ctx->wp_inner, &ctx->bp_inner);
            if (rc != TL_OK) return rc;
        }
    } else if (cfg->cell == TL_TREERNN && !bf16) {
        const size_t n_u = (size_t)2 * H * H;
        TL_HIP(hipMalloc(&ctx->m_u, n_u * sizeof(float)));
        TL_HIP(hipMalloc(&ctx->m_b, (size_t)H * sizeof(float)));
        TL_HIP(hipMemcpy(ctx->m_u, cfg->u, n_u * sizeof(float), hipMemcpyDeviceToDevice));
        TL_HIP(hipMemcpy(ctx->m_b, cfg->b, (size_t)H * sizeof(float), hipMemcpyDeviceToDevice));
        TL_HIP(hipMalloc(&ctx->t_scratch, n_u * sizeof(float)));
        TL_HIP(hipMalloc(&ctx->zero_bias, ((size_t)2 * H + HU) * sizeof(float)));
        TL_HIP(hipMemset(ctx->zero_bias, 0, ((size_t)2 * H + HU) * sizeof(float)));
        ctx->ng_bwd_inner = (2 * H) % 4 == 0 ? 4 : 1;
        ctx->ws_steps16 = ws_steps16;
        rc = pack_treernn_f32(ctx, nullptr);
        TL_HIP(hipDeviceSynchronize());
        if (rc != TL_OK) return rc;
    } else if (cfg->cell == TL_TREERNN) {
        rc = pack_gemm(cfg->u, cfg->b, 1, H, 2, H, ctx->n_cg, ws_steps16, bf16, &ctx->g_inner, &ctx->wp_inner, &ctx->bp_inner);
        if (rc != TL_OK) return rc;
    } else {
        // RNTN (fp32 only): the parameters as given, tensor slices and W packed per column group and q (padded K is
        // 64, 128 or 256), and what the backward pass derives from them
        const size_t D2 = (size_t)2 * H, L = (size_t)H * D2 + H;
        TL_HIP(hipMalloc(&ctx->m_v, (size_t)H * D2 * D2 * sizeof(float)));
        TL_HIP(hipMalloc(&ctx->m_u, D2 * H * sizeof(float)));
        TL_HIP(hipMalloc(&ctx->m_b, (size_t)H * sizeof(float)));
        TL_HIP(hipMemcpy(ctx->m_v, cfg->v, (size_t)H * D2 * D2 * sizeof(float), hipMemcpyDeviceToDevice));
        TL_HIP(hipMemcpy(ctx->m_u, cfg->u, D2 * H * sizeof(float), hipMemcpyDeviceToDevice));
        TL_HIP(hipMemcpy(ctx->m_b, cfg->b, (size_t)H * sizeof(float), hipMemcpyDeviceToDevice));
        TL_HIP(hipMalloc(&ctx->t_scratch, L * D2 * sizeof(float)));
        TL_HIP(hipMalloc(&ctx->rntn_acc, (D2 * L + L) * sizeof(float)));
        TL_HIP(hipMalloc(&ctx->zero_bias, (D2 + HU) * sizeof(float)));
        TL_HIP(hipMemset(ctx->zero_bias, 0, (D2 + HU) * sizeof(float)));
        ctx->ng_bwd_inner = D2 % 4 == 0 ? 4 : 1;
        rc = pack_rntn_f32(ctx, nullptr);
        if (rc != TL_OK) return rc;
    }
    TL_HIP(hipDeviceSynchronize());

    // every kernel that stages tiles needs more than the default LDS limit
    for (int v = 0; v < 2; ++v) {
        if ((rc = allow_lds(ready_kernel(cfg->cell, v, 0, bf16))) != TL_OK) return rc;
        if ((rc = allow_lds(levels_kernel(cfg->cell, v, 0, bf16))) != TL_OK) return rc;
        for (int epi = 0; epi < 4; ++epi)
            if ((rc = allow_lds(static_kernel(epi, v, bf16))) != TL_OK) return rc;
        for (int epi = EPI_BWD_INNER_GATES; epi <= EPI_BWD_LEAF_OPERAND4; ++epi)
            if (epi_is_backward(epi) && (rc = allow_lds(backward_kernel(epi, v))) != TL_OK) return rc;
    }
    int occ = 0;
    TL_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, reinterpret_cast<const void *>(ready_kernel(cfg->cell, true, 0, bf16)),
                                                        WG_THREADS, TILE_SMEM_BYTES));
    int occ2 = 0;
    TL_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ2, reinterpret_cast<const void *>(levels_kernel(cfg->cell, false, 0, bf16)),
                                                        WG_THREADS, TILE_SMEM_BYTES));
    if (occ2 < occ) occ = occ2;
    if (occ < 1) return TL_EHIP;
    if (occ > 2) occ = 2;
    ctx->persistent_grid = occ * ctx->n_cu;
    ctx->bw_grid = 0;
    if (!bf16 && cfg->cell != TL_RNTN) {
        // the backward kernel that walks all heights waits on a grid barrier: all its workgroups must be resident
        typedef void (*bwh_kernel)(Fwd, BwdHeights);
        const bwh_kernel ks[4] = {k_backward_heights<true, true>, k_backward_heights<true, false>, k_backward_heights<false, true>,
                                  k_backward_heights<false, false>};
        int o_min = 2;
        for (const bwh_kernel k : ks) {
            if ((rc = allow_lds(k)) != TL_OK) return rc;
            int o = 0;
            TL_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&o, reinterpret_cast<const void *>(k), WG_THREADS, TILE_SMEM_BYTES));
            if (o < o_min) o_min = o;
        }
        ctx->bw_grid = o_min * ctx->n_cu;
        // weight-stationary operand gradient: 5 H / 128 k-steps per wave and half of its quarter of the K axis
        ctx->bw_ws_grid = 0;
        const int H_ = cfg->hidden, n_cg_b = 2 * H_ / HU;
        if ((cfg->cell == TL_TREELSTM || cfg->cell == TL_TREERNN) && H_ % 128 == 0 && H_ <= 512 && ctx->n_cu >= n_cg_b) {
            ctx->bw_spw2 = (cfg->cell == TL_TREELSTM ? 5 : 1) * H_ / 128;
            size_t lds = 0;
            const bwh_ws_kernel k = backward_ws_kernel(cfg->cell == TL_TREELSTM, ctx->bw_spw2, &lds);
            if ((rc = allow_lds(k, lds)) != TL_OK) return rc;
            int o = 0;
            TL_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&o, reinterpret_cast<const void *>(k), WG_THREADS, lds));
            if (o >= 1) ctx->bw_ws_grid = ctx->n_cu / n_cg_b * n_cg_b;
        }
    }
    if (ctx->spw > 0) {
        ctx->ws_lds = ws_lds_bytes(ctx->spw, bf16);
        for (int v = 0; v < 2; ++v) {   // fp32: rows 16-byte aligned / 8-byte aligned
            if ((rc = allow_lds(ready_kernel(cfg->cell, v != 0, ctx->spw, bf16), ctx->ws_lds)) != TL_OK) return rc;
            if ((rc = allow_lds(levels_kernel(cfg->cell, v != 0, ctx->spw, bf16), ctx->ws_lds)) != TL_OK) return rc;
        }
        int o1 = 0, o2 = 0;
        TL_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&o1, reinterpret_cast<const void *>(ready_kernel(cfg->cell, true, ctx->spw, bf16)),
                                                            WG_THREADS, ctx->ws_lds));
        TL_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&o2, reinterpret_cast<const void *>(levels_kernel(cfg->cell, true, ctx->spw, bf16)),
                                                            WG_THREADS, ctx->ws_lds));
        if (o2 < o1) o1 = o2;
        for (int v = 0; v < 2; ++v) {
            const fwd_kernel fk = flow_kernel(cfg->cell, v != 0, ctx->spw, bf16);
            if ((rc = allow_lds(fk, ctx->ws_lds)) != TL_OK) return rc;
            TL_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&o2, reinterpret_cast<const void *>(fk), WG_THREADS, ctx->ws_lds));
            if (o2 < o1) o1 = o2;
        }
        const int want = bf16 ? 2 : 1;   // fp32: the register file of a CU holds one workgroup's weights; bf16: two
        if (o1 > want) o1 = want;
        ctx->ws_grid = o1 * ctx->n_cu;
        if (o1 < 1 || ctx->ws_grid < ctx->n_cg + 1) ctx->spw = 0;
    }

    if (ctx->spw_leaf > 0) {
        const size_t lds = leaf_lds_bytes(ctx->spw_leaf, bf16);
        const fwd_kernel lk = bf16 ? leaf_ws_bf_kernel(ctx->spw_leaf) : leaf_ws_kernel(ctx->spw_leaf);
        if ((rc = allow_lds(lk, lds)) != TL_OK) return rc;
        int o = 0;
        TL_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&o, reinterpret_cast<const void *>(lk), WG_THREADS, lds));
        const int o_max = bf16 ? 4 : 2;      // fp32: bound by its instruction stream, a third workgroup brings nothing; bf16: by latency
        if (o > o_max) o = o_max;
        ctx->leaf_grid = o * ctx->n_cu / ctx->n_cg * ctx->n_cg;
        if (ctx->leaf_grid < ctx->n_cg) ctx->spw_leaf = 0;
    }

    if (cfg->cell == TL_RNTN) {
        // frontiers of so few tiles that whole tiles would give the workgroups fewer than two rounds of work are cut into
        // parts (cell_rntn.hpp): with whole tiles the last, partly filled round and the two workgroups that share a CU's matrix
        // units decide the time of such a frontier.  One unit of the scratch area per tile of such a frontier
        const int grid = ctx->persistent_grid > ctx->ws_grid ? ctx->persistent_grid : ctx->ws_grid;
        const int units = 2 * grid / ctx->n_cg;
        if (units > 0) {
            const size_t per_unit = (size_t)ctx->n_cg * RNTN_PARTS * RNTN_PART_FLOATS * sizeof(float);
            TL_HIP(hipMalloc(&ctx->rntn_part, units * per_unit));
            TL_HIP(hipMalloc(&ctx->rntn_done, (size_t)units * ctx->n_cg * sizeof(unsigned int)));
            TL_HIP(hipMemset(ctx->rntn_done, 0, (size_t)units * ctx->n_cg * sizeof(unsigned int)));
        }
        ctx->rntn_units = units;
    }
    TL_HIP(hipHostMalloc(&ctx->host_ctl, sizeof(Ctl), hipHostMallocDefault));
    if ((rc = scratch_address(ctx->device, &ctx->scratch)) != TL_OK) return rc;
    return TL_OK;
}

void td_free(tl_td_ctx *ctx)
{
    for (int sd = 0; sd < 2; ++sd) {
        (void)hipFree(ctx->wp[sd]);
        (void)hipFree(ctx->bp[sd]);
    }
    (void)hipFree(ctx->w_stop);
    (void)hipFree(ctx->zeros);
    (void)hipFree(ctx->ctl);
    if (ctx->host_ctl) (void)hipHostFree(ctx->host_ctl);
    delete ctx;
}

// levels > 0: the first `levels` offsets of the per-height lists come along in the same wait (shallow batches then need no
// second round trip for them).
int read_ctl(tl_ctx *ctx, int levels = 0)
{
    TL_HIP(hipMemcpyAsync(ctx->host_ctl, ctx->last.ctl, sizeof(Ctl), hipMemcpyDeviceToHost, ctx->last_stream));
    if (levels > 0)
        TL_HIP(hipMemcpyAsync(ctx->host_levels, ctx->last.level_off, (size_t)levels * 4, hipMemcpyDeviceToHost, ctx->last_stream));
    TL_HIP(hipStreamSynchronize(ctx->last_stream));
    // a tree without a root shows as a root count below the number of trees
    if (ctx->host_ctl->status == 0 && !ctx->last.flow_roots && ctx->host_ctl->n_roots != ctx->last.n_trees) ctx->host_ctl->status = TL_ESTRUCT;
    return TL_OK;
}

}  // namespace

extern "C" {

int tl_create(const tl_config *cfg, tl_ctx **out)
{
    if (!cfg || !out) return TL_EINVAL;
    *out = nullptr;
    if (cfg->cell != TL_TREELSTM && cfg->cell != TL_TREERNN && cfg->cell != TL_RNTN) return TL_EINVAL;
    if (cfg->cell == TL_RNTN && (!cfg->v || cfg->hidden > 128 || cfg->precision != TL_F32)) return TL_EINVAL;
    if (cfg->precision != TL_F32 && cfg->precision != TL_BF16_IN) return TL_EINVAL;
    if (cfg->scheduler < TL_SCHED_READY || cfg->scheduler > TL_SCHED_DATAFLOW) return TL_EINVAL;
    if (cfg->vocab < 1 || cfg->embed_dim < 1 || cfg->hidden < 1 || cfg->spin_limit < 0) return TL_EINVAL;
    if (cfg->hidden > (1 << 14) || cfg->embed_dim > (1 << 16)) return TL_EINVAL;
    if (!cfg->emb || !cfg->u || !cfg->b) return TL_EINVAL;
    if (cfg->cell == TL_TREELSTM && (!cfg->w_leaf || !cfg->b_leaf)) return TL_EINVAL;
    if (cfg->cell != TL_TREELSTM && cfg->embed_dim != cfg->hidden) return TL_EINVAL;
    tl_ctx *ctx = new (std::nothrow) tl_ctx();
    if (!ctx) return TL_ENOMEM;
    int rc = create_impl(cfg, ctx);
    if (rc != TL_OK) {
        free_all(ctx);
        return rc;
    }
    *out = ctx;
    return TL_OK;
}

}  // extern "C"

namespace {

// tl_forward (static_ws false: workspace owned by the context, grown on demand) and tl_forward_noalloc (static_ws
// true: the fixed per-device array; nothing is allocated, created or freed on this path).
int forward_impl(tl_ctx *ctx, bool static_ws, int n_trees, int n_nodes, const int32_t *tree_off, const int32_t *left,
                 const int32_t *right, const int32_t *word, float *h, float *c, float *h_root, float *c_root,
                 int32_t *root, void *hip_stream)
{
    if (!ctx) return TL_EINVAL;
    if (n_trees == 0 && n_nodes == 0) {     // an empty batch: nothing to evaluate, nothing is launched or written
        ctx->ran = false;
        ctx->gates_nodes = 0;
        return TL_OK;
    }
    if (!tree_off || !left || !right || !word || !h) return TL_EINVAL;
    if (n_trees < 1 || n_nodes < n_trees) return TL_EINVAL;
    const tl_config &cfg = ctx->cfg;
    if (cfg.cell == TL_TREELSTM && !c) return TL_EINVAL;
    if (((long long)n_nodes + n_trees) % 2 != 0) return TL_ESTRUCT;   // full binary trees: N = 2 leaves - trees
    hipStream_t st = (hipStream_t)hip_stream;
    int rc = TL_OK;
    if (static_ws) {
        if (cfg.scheduler == TL_SCHED_LEVEL_HOST) return TL_EINVAL;      // reads level offsets back through a pinned buffer it would have to allocate
        if (n_nodes > TL_NOALLOC_MAX_NODES) return TL_ELIMIT;
        if (cfg.precision == TL_BF16_IN && (size_t)n_nodes * ctx->hs * sizeof(unsigned short) > NOALLOC_HB_BYTES) return TL_ELIMIT;   // bf16 copy of h
        if (!ctx->scratch) return TL_EHIP;
    } else if ((rc = ensure_workspace(ctx, n_nodes, n_trees)) != TL_OK) {
        return rc;
    }

    Fwd f{};
    f.n_trees = n_trees;
    f.n_nodes = n_nodes;
    f.n_leaf = (int)(((long long)n_nodes + n_trees) / 2);
    f.n_int = n_nodes - f.n_leaf;
    f.tree_off = tree_off; f.left = left; f.right = right; f.word = word;
    f.h = h; f.c = cfg.cell == TL_TREELSTM ? c : nullptr;
    f.h_root = h_root; f.c_root = c_root; f.root_out = root;
    f.cell = cfg.cell; f.H = cfg.hidden; f.E = cfg.embed_dim; f.vocab = cfg.vocab; f.n_cg = ctx->n_cg; f.bf16 = cfg.precision == TL_BF16_IN;
    f.emb = ctx->emb; f.embb = ctx->embb; f.es = ctx->es;
    f.leaf = ctx->g_leaf; f.inner = ctx->g_inner;
    if (static_ws) carve_workspace(ctx->scratch, TL_NOALLOC_MAX_NODES, TL_NOALLOC_MAX_NODES, &f);
    else carve_workspace(ctx->ws, ctx->cap_nodes, ctx->cap_trees, &f);
    ctx->gates_nodes = 0;
    if (!static_ws && ctx->keep_gates && cfg.cell == TL_TREELSTM && cfg.precision == TL_F32) {
        if (n_nodes > ctx->gates_cap) {
            TL_HIP(hipDeviceSynchronize());
            if (ctx->gates) { TL_HIP(hipFree(ctx->gates)); ctx->gates = nullptr; }
            ctx->gates_cap = 0;
            TL_HIP(hipMalloc(&ctx->gates, (size_t)ctx->cap_nodes * 5 * cfg.hidden * sizeof(float)));
            ctx->gates_cap = ctx->cap_nodes;
        }
        f.gates = ctx->gates;
        ctx->gates_nodes = n_nodes;
        ctx->gates_h = h;
    }
    f.spin_limit = cfg.spin_limit > 0 ? cfg.spin_limit : DEFAULT_SPIN_LIMIT;
    const bool vec4_inner = (cfg.hidden % 4 == 0) && (((uintptr_t)h & 15) == 0);
    const bool bf16 = cfg.precision == TL_BF16_IN;
    // the weight-stationary cell addresses rows with 24-bit row numbers and 32-bit byte offsets
    const bool ws_range = n_nodes < (1 << 24) && (unsigned long long)n_nodes * cfg.hidden * 4ull < (1ull << 32);
    const bool pair_inner = (cfg.hidden % 2 == 0) && (((uintptr_t)h & 7) == 0);      // rows 8-byte aligned
    const int spw = ((bf16 || pair_inner) && ws_range) ? ctx->spw : 0;     // weight-stationary cell in the persistent kernels
    const bool persistent = cfg.scheduler != TL_SCHED_LEVEL_HOST;
    // the data-flow scheduler needs the weight-stationary cell and its private lists; without them (RNTN, sizes the
    // cell does not take, the fixed workspace) the level scheduler on the device stands in.
    const bool flow = cfg.scheduler == TL_SCHED_DATAFLOW && spw > 0 && !static_ws && ctx->flow_ws != nullptr;
    // A batch of few large trees: the data-flow scheduler deals whole trees to its sets of workgroups, so with fewer
    // trees than sets the others stay idle: one bushy tree of 16 384 leaves takes 3.5 ms on one set against 0.34 ms
    // level by level on all of them, while a deep chain of 2 048 leaves takes 6.4 ms data-flow and 11.8 ms level by
    // level.  The host does not know the shapes, so both kernels are launched and the device picks
    // (internal_kernel_skipped: by the width of the first frontier).  Small trees - a sentence, say - are left with
    // the data-flow kernel alone: one set holds all that is ready of such a tree.
    const int flow_sets = ctx->n_cg > 0 ? ctx->ws_grid / ctx->n_cg : 0;
    const bool flow_or_levels = flow && n_trees < flow_sets && n_nodes / (n_trees > 0 ? n_trees : 1) >= FLOW_LARGE_TREE_NODES;
    if (persistent && spw > 0 && bf16) {
        f.hb = static_ws ? reinterpret_cast<unsigned short *>(ctx->scratch + NOALLOC_WS_BYTES) : ctx->hb;
        f.hs = ctx->hs;
    }
    // The persistent kernels' workgroups wait for each other, so all of them must be resident at once: the grid is
    // cut to what the device holds of the very kernel that is launched (the figure taken at tl_create is that of one
    // variant), and a kernel of which not even one set of workgroups fits is refused here, not found out by a stall.
    const bool ready_sched = cfg.scheduler == TL_SCHED_READY || cfg.scheduler == TL_SCHED_READY_PRIORITY;
    const fwd_kernel kern = !persistent ? nullptr
                            : ready_sched ? ready_kernel(cfg.cell, vec4_inner, spw, bf16)
                            : flow ? flow_kernel(cfg.cell, vec4_inner, spw, bf16) : levels_kernel(cfg.cell, vec4_inner, spw, bf16);
    const size_t kern_lds = spw > 0 ? ctx->ws_lds : TILE_SMEM_BYTES;
    int grid_p = (persistent && spw > 0) ? ctx->ws_grid : ctx->persistent_grid;
    if (kern) {
        int per_cu = 0;
        if ((rc = resident_per_cu(ctx, kern, kern_lds, &per_cu)) != TL_OK) return rc;
        if (per_cu * ctx->n_cu < grid_p) grid_p = per_cu * ctx->n_cu;
        if (grid_p < (spw > 0 ? ctx->n_cg : 1) + (ready_sched ? 1 : 0)) return TL_EHIP;
    }
    int grid_l2 = 0;                                  // grid of the level kernel where it is launched beside the data-flow kernel
    if (flow_or_levels) {
        int per_cu = 0;
        if ((rc = resident_per_cu(ctx, levels_kernel(cfg.cell, vec4_inner, spw, bf16), kern_lds, &per_cu)) != TL_OK) return rc;
        grid_l2 = ctx->ws_grid;
        if (per_cu * ctx->n_cu < grid_l2) grid_l2 = per_cu * ctx->n_cu;
        grid_l2 = grid_l2 / ctx->n_cg * ctx->n_cg;
        if (grid_l2 < ctx->n_cg) return TL_EHIP;
    }
    f.cap_tiles = grid_p / ctx->n_cg > 0 ? grid_p / ctx->n_cg : 1;
    // RNTN: a frontier of at most rntn_units tiles is cut into RNTN_PARTS workgroups per tile and column group
    f.rntn_part = ctx->rntn_part; f.rntn_done = ctx->rntn_done;
    f.rntn_units = cfg.cell == TL_RNTN ? (2 * grid_p / ctx->n_cg < ctx->rntn_units ? 2 * grid_p / ctx->n_cg : ctx->rntn_units) : 0;
    // ready scheduler: gangs of gang_size compute workgroups plus one scheduler workgroup each
    f.gang_size = ctx->n_cg + 1 <= grid_p ? ctx->n_cg : grid_p - 1;
    f.n_gangs = grid_p / (f.gang_size + 1) < MAX_GANGS ? grid_p / (f.gang_size + 1) : MAX_GANGS;
    f.gang_parts = 1;
    // RNTN: with few column groups (d = 64: four) a gang of one workgroup per column group leaves a tile's 129 slices to
    // four workgroups; as under the level scheduler, RNTN_PARTS workgroups per column group each add up a part of the
    // slices and the last one to arrive adds the parts (one unit of the scratch area per gang and tile in flight)
    if (cfg.cell == TL_RNTN && ready_sched && ctx->rntn_part != nullptr) {
        const int gs = ctx->n_cg * RNTN_PARTS;
        int gangs = grid_p / (gs + 1);
        if (gangs > MAX_GANGS) gangs = MAX_GANGS;
        if (gangs > ctx->rntn_units / GANG_RING) gangs = ctx->rntn_units / GANG_RING;
        if (gangs >= 1) {
            f.gang_size = gs;
            f.n_gangs = gangs;
            f.gang_parts = RNTN_PARTS;
        }
    }

    // heights and per-height node lists: for the host-driven scheduler, and as the check for cycles
    const bool need_levels = cfg.scheduler == TL_SCHED_LEVEL_HOST || cfg.validate != 0;
    f.priority = cfg.scheduler == TL_SCHED_READY_PRIORITY ? 1 : 0;
    if (flow) {
        f.flow = (cfg.cell == TL_TREELSTM && ctx->spw_leaf > 0 && ws_range) ? 2 : 1;
        // (with no internal node the data-flow kernel is not launched; where the level kernel may run instead, the root passes do)
        f.flow_roots = f.n_int > 0 && !need_levels && !flow_or_levels ? 1 : 0;
        f.flow_seen = reinterpret_cast<int32_t *>(ctx->flow_ws);
        f.flow_list = reinterpret_cast<int4 *>(ctx->flow_ws + align256((size_t)ctx->n_cg * ctx->cap_nodes * sizeof(int32_t)));
    }
    const bool vec4_leaf = cfg.embed_dim % 4 == 0;
    const int inner_epi = cfg.cell == TL_TREELSTM ? EPI_LSTM_INNER : (cfg.cell == TL_TREERNN ? EPI_RNN_INNER : EPI_RNTN_INNER);
    const bool prof = ctx->profiling != 0 && !static_ws;      // (recording may have to create events)
    const int nb_nodes = (n_nodes + 1 + 255) / 256;
    const int nb_big = (n_nodes + 1 + NODE_BLOCK - 1) / NODE_BLOCK;

    ctx->last = f;
    ctx->last_stream = st;
    ctx->ran = true;
    ctx->last_grid = 0;
    ctx->last_levels = 0;
    hipEvent_t *ev = ctx->ev[ctx->n_recorded % TL_PROFILE_RING];
    if (prof) {
        for (int i = 0; i < TL_N_STAGES; ++i)
            if (!ev[i]) TL_HIP(hipEventCreate(&ev[i]));
        TL_HIP(hipEventRecord(ev[0], st));
    }
    // ---- structure pass ----------------------------------------------------------------
    if (static_ws && f.hb && ctx->hs != cfg.hidden) {
        // the padding at the end of each row of the bf16 copy of h must read as zero, and the shared array may hold
        // what a context of another hidden size left there
        ZeroList z{};
        z.p[0] = reinterpret_cast<float *>(f.hb);
        z.n[0] = (size_t)n_nodes * ctx->hs * sizeof(unsigned short) / sizeof(float);      // hs is a multiple of 8
        hipLaunchKernelGGL(k_zero_many, dim3(256), dim3(256), 0, st, z);
    }
    // (the data-flow scheduler's fill of the rows of internal nodes takes one wave per node)
    const int nb_reset = f.flow == 1 ? (n_nodes / 4 + 1 < 256 ? 256 : (n_nodes / 4 + 1 > 4096 ? 4096 : n_nodes / 4 + 1)) : 256;
    hipLaunchKernelGGL(k_reset, dim3(nb_reset), dim3(256), 0, st, f, need_levels ? 1 : 0);
    hipLaunchKernelGGL(k_scatter, dim3(nb_big), dim3(NODE_BLOCK), 0, st, f);
    if (!f.flow_roots) hipLaunchKernelGGL(k_roots, dim3(nb_big), dim3(NODE_BLOCK), 0, st, f);
    if (need_levels) {
        hipLaunchKernelGGL(k_climb, dim3((f.n_leaf + 255) / 256), dim3(256), 0, st, f);
        hipLaunchKernelGGL(k_level_hist, dim3(nb_nodes), dim3(256), 0, st, f);
        hipLaunchKernelGGL(k_scan_levels, dim3(1), dim3(1024), 0, st, f);
        hipLaunchKernelGGL(k_fill_levels, dim3(nb_nodes), dim3(256), 0, st, f);
    }
    if (f.priority && f.n_int > 0) {
        hipLaunchKernelGGL(k_depth_walk, dim3(nb_big), dim3(NODE_BLOCK), 0, st, f);
        hipLaunchKernelGGL(k_seed_place, dim3(nb_big), dim3(NODE_BLOCK), 0, st, f);
    }
    TL_HIP(hipGetLastError());
    if (prof) TL_HIP(hipEventRecord(ev[1], st));

    // ---- leaves ------------------------------------------------------------------------
    if (cfg.cell == TL_TREELSTM && ctx->spw_leaf > 0 && ws_range) {          // (its cell addresses h and c with 32-bit offsets)
        hipLaunchKernelGGL(bf16 ? leaf_ws_bf_kernel(ctx->spw_leaf) : leaf_ws_kernel(ctx->spw_leaf), dim3(ctx->leaf_grid),
                           dim3(WG_THREADS), leaf_lds_bytes(ctx->spw_leaf, bf16), st, f);
    } else if (cfg.cell == TL_TREELSTM) {
        const LevelPlan plan = plan_level(f.n_leaf, f.cap_tiles);
        hipLaunchKernelGGL(static_kernel(EPI_LSTM_LEAF, vec4_leaf, bf16), dim3(plan.n_tiles * ctx->n_cg), dim3(WG_THREADS),
                           TILE_SMEM_BYTES, st, f, (const int32_t *)f.leaf_list, f.n_leaf, plan);
    } else {
        hipLaunchKernelGGL(k_leaf_copy, dim3(f.n_leaf), dim3(128), 0, st, f);
    }
    TL_HIP(hipGetLastError());
    if (prof) TL_HIP(hipEventRecord(ev[2], st));

    // ---- internal nodes ------------------------------------------------------------------
    if (f.n_int > 0) {
        if (ready_sched) {
            const int grid_r = f.n_gangs * (f.gang_size + 1);
            hipLaunchKernelGGL(kern, dim3(grid_r), dim3(WG_THREADS), kern_lds, st, f);
            ctx->last_grid = grid_r;
        } else if (cfg.scheduler == TL_SCHED_LEVEL_DEVICE || cfg.scheduler == TL_SCHED_DATAFLOW) {
            // weight-stationary cell: every workgroup is tied to one column group, so whole sets only
            const int grid_l = spw > 0 ? grid_p / ctx->n_cg * ctx->n_cg : grid_p;
            if (flow_or_levels) {                     // both kernels; every workgroup of the one that is not picked returns at once
                Fwd g = f;
                g.pick = 1;
                hipLaunchKernelGGL(kern, dim3(grid_l), dim3(WG_THREADS), kern_lds, st, g);
                g.pick = 2;
                hipLaunchKernelGGL(levels_kernel(cfg.cell, vec4_inner, spw, bf16), dim3(grid_l2), dim3(WG_THREADS), kern_lds, st, g);
            } else {
                hipLaunchKernelGGL(kern, dim3(grid_l), dim3(WG_THREADS), kern_lds, st, f);
            }
            ctx->last_grid = grid_l;
        } else {
            // the host needs the number of heights and the offsets of their node lists
            const int levels_ahead = n_nodes + 2 < LEVELS_AHEAD ? n_nodes + 2 : LEVELS_AHEAD;
            if ((rc = read_ctl(ctx, levels_ahead)) != TL_OK) return rc;
            const int n_levels = ctx->host_ctl->status == 0 ? ctx->host_ctl->n_levels : 0;
            if (n_levels > 1) {
                if (n_levels + 1 > levels_ahead) {
                    TL_HIP(hipMemcpyAsync(ctx->host_levels, f.level_off, (size_t)(n_levels + 1) * 4, hipMemcpyDeviceToHost, st));
                    TL_HIP(hipStreamSynchronize(st));
                }
                int max_grid = 0;
                for (int lvl = 1; lvl < n_levels; ++lvl) {
                    const int lo = ctx->host_levels[lvl], rows = ctx->host_levels[lvl + 1] - lo;
                    if (rows <= 0 || lo < 0 || lo + rows > f.n_int) return TL_EHIP;
                    const LevelPlan plan = plan_level(rows, cfg.cell == TL_RNTN ? rntn_cap_tiles(f.cap_tiles, f.rntn_units) : f.cap_tiles);
                    const int parts = plan.n_tiles <= f.rntn_units ? RNTN_PARTS : 1;
                    hipLaunchKernelGGL(static_kernel(inner_epi, vec4_inner, bf16), dim3(plan.n_tiles * ctx->n_cg * parts), dim3(WG_THREADS),
                                       TILE_SMEM_BYTES, st, f, (const int32_t *)(f.level_nodes + lo), rows, plan);
                    if (plan.n_tiles * ctx->n_cg * parts > max_grid) max_grid = plan.n_tiles * ctx->n_cg * parts;
                }
                ctx->last_grid = max_grid;
            }
            ctx->last_levels = n_levels;
        }
        TL_HIP(hipGetLastError());
    }
    if (prof) TL_HIP(hipEventRecord(ev[3], st));

    // ---- roots ---------------------------------------------------------------------------
    if (!f.flow_roots) hipLaunchKernelGGL(k_root_gather, dim3(n_trees), dim3(128), 0, st, f);
    TL_HIP(hipGetLastError());
    if (prof) {
        TL_HIP(hipEventRecord(ev[4], st));
        ctx->n_recorded += 1;
    }
    return TL_OK;
}

}  // namespace

extern "C" {

int tl_forward(tl_ctx *ctx, int n_trees, int n_nodes, const int32_t *tree_off, const int32_t *left,
               const int32_t *right, const int32_t *word, float *h, float *c, float *h_root, float *c_root,
               int32_t *root, void *hip_stream)
{
    return forward_impl(ctx, false, n_trees, n_nodes, tree_off, left, right, word, h, c, h_root, c_root, root, hip_stream);
}

int tl_forward_noalloc(tl_ctx *ctx, int n_trees, int n_nodes, const int32_t *tree_off, const int32_t *left,
                       const int32_t *right, const int32_t *word, float *h, float *c, float *h_root, float *c_root,
                       int32_t *root, void *hip_stream)
{
    return forward_impl(ctx, true, n_trees, n_nodes, tree_off, left, right, word, h, c, h_root, c_root, root, hip_stream);
}

int tl_status(tl_ctx *ctx)
{
    if (!ctx) return TL_EINVAL;
    if (!ctx->ran) return TL_OK;
    int rc = read_ctl(ctx);
    if (rc != TL_OK) return rc;
    return ctx->host_ctl->status;
}

int tl_set_profiling(tl_ctx *ctx, int on)
{
    if (!ctx) return TL_EINVAL;
    ctx->profiling = on != 0;
    ctx->n_recorded = 0;
    return TL_OK;
}

int tl_stage_ms(tl_ctx *ctx, int back, float *ms)
{
    if (!ctx || !ms || back < 0) return TL_EINVAL;
    if (back >= ctx->n_recorded || back >= TL_PROFILE_RING) return TL_EINVAL;
    hipEvent_t *ev = ctx->ev[(ctx->n_recorded - 1 - back) % TL_PROFILE_RING];
    TL_HIP(hipEventSynchronize(ev[4]));
    for (int i = 0; i < 4; ++i) TL_HIP(hipEventElapsedTime(&ms[i], ev[i], ev[i + 1]));
    TL_HIP(hipEventElapsedTime(&ms[4], ev[0], ev[4]));
    return TL_OK;
}

int tl_last_stats(tl_ctx *ctx, int *n_levels, int *n_tiles, int *n_workgroups)
{
    if (!ctx) return TL_EINVAL;
    if (n_levels) *n_levels = 0;
    if (n_tiles) *n_tiles = 0;
    if (n_workgroups) *n_workgroups = 0;
    if (!ctx->ran) return TL_OK;
    int rc = read_ctl(ctx);
    if (rc != TL_OK) return rc;
    if (n_levels) *n_levels = ctx->host_ctl->n_levels;
    if (n_tiles) *n_tiles = (int)ctx->host_ctl->tiles.v;
    if (n_workgroups) *n_workgroups = ctx->last_grid;
    return TL_OK;
}

int tl_backward(tl_ctx *ctx, int n_trees, int n_nodes, const int32_t *tree_off, const int32_t *left, const int32_t *right,
                const int32_t *word, const float *h, const float *c, const float *g_h, float *d_u, float *d_b,
                float *d_w_leaf, float *d_b_leaf, float *d_x, void *hip_stream)
{
    if (!ctx || !tree_off || !left || !right || !word || !h || !g_h || !d_u || !d_b || !d_x) return TL_EINVAL;
    const tl_config &cfg = ctx->cfg;
    if (cfg.precision != TL_F32) return TL_EINVAL;
    const bool lstm = cfg.cell == TL_TREELSTM, rntn = cfg.cell == TL_RNTN;
    if (lstm && (!c || !d_w_leaf || !d_b_leaf)) return TL_EINVAL;
    if (rntn && !d_w_leaf) return TL_EINVAL;                  // dV
    if (n_trees < 1 || n_nodes < n_trees) return TL_EINVAL;
    if (((long long)n_nodes + n_trees) % 2 != 0) return TL_ESTRUCT;
    hipStream_t st = (hipStream_t)hip_stream;
    int rc = ensure_workspace(ctx, n_nodes, n_trees);
    if (rc != TL_OK) return rc;
    const int H = cfg.hidden, E = cfg.embed_dim;
    const int n_leaf = (int)(((long long)n_nodes + n_trees) / 2), n_int = n_nodes - n_leaf;
    // workspace of the backward pass: dh, dc [N x H], gate gradients [n_int x 5H] and [n_leaf x 3H]
    // (RNTN: rows of d * 2d + d values per internal node, see backward.hpp)
    const size_t rntn_row = (size_t)H * 2 * H + H;
    if (n_nodes > ctx->bw_nodes) {
        TL_HIP(hipDeviceSynchronize());
        if (ctx->bw) { TL_HIP(hipFree(ctx->bw)); ctx->bw = nullptr; }
        ctx->bw_nodes = 0;
        const size_t cap = (size_t)ctx->cap_nodes;
        size_t floats = 2 * cap * H + cap * 5 * H;                                   // n_int*5H + n_leaf*3H <= N*5H
        if (rntn) floats = 2 * cap * H + (cap / 2 + 1) * rntn_row;
        if (floats * sizeof(float) > ((size_t)64 << 30)) return TL_ENOMEM;
        TL_HIP(hipMalloc(&ctx->bw, floats * sizeof(float)));
        ctx->bw_nodes = ctx->cap_nodes;
    }
    Fwd f{};
    f.n_trees = n_trees; f.n_nodes = n_nodes; f.n_leaf = n_leaf; f.n_int = n_int;
    f.tree_off = tree_off; f.left = left; f.right = right; f.word = word;
    f.h = const_cast<float *>(h); f.c = lstm ? const_cast<float *>(c) : nullptr;
    f.cell = cfg.cell; f.H = H; f.E = E; f.vocab = cfg.vocab; f.n_cg = ctx->n_cg;
    f.emb = ctx->emb;
    f.leaf = ctx->g_leaf; f.inner = ctx->g_inner;
    carve_workspace(ctx->ws, ctx->cap_nodes, ctx->cap_trees, &f);
    f.spin_limit = DEFAULT_SPIN_LIMIT;
    f.cap_tiles = ctx->persistent_grid / ctx->n_cg > 0 ? ctx->persistent_grid / ctx->n_cg : 1;
    const size_t cap = (size_t)ctx->bw_nodes;
    f.dh = ctx->bw;
    f.dc = f.dh + cap * H;
    const int ng_cell = lstm ? 5 : 1;                         // gate blocks of an internal node
    float *dg_int = f.dc + cap * H, *dg_leaf = dg_int + (size_t)n_int * ng_cell * H;
    const int dg_cols = rntn ? (int)rntn_row : ng_cell * H;   // length of a row of dg_int
    f.d_x = d_x;
    ctx->last = f;
    ctx->last_stream = st;
    ctx->ran = true;
    const int nb_nodes = (n_nodes + 1 + 255) / 256;
    const int nb_big = (n_nodes + 1 + NODE_BLOCK - 1) / NODE_BLOCK;
    // structure pass with heights and per-height lists (as for the host-driven level scheduler)
    hipLaunchKernelGGL(k_reset, dim3(256), dim3(256), 0, st, f, 1);
    hipLaunchKernelGGL(k_scatter, dim3(nb_big), dim3(NODE_BLOCK), 0, st, f);
    hipLaunchKernelGGL(k_roots, dim3(nb_big), dim3(NODE_BLOCK), 0, st, f);
    hipLaunchKernelGGL(k_climb, dim3((n_leaf + 255) / 256), dim3(256), 0, st, f);
    hipLaunchKernelGGL(k_level_hist, dim3(nb_nodes), dim3(256), 0, st, f);
    hipLaunchKernelGGL(k_scan_levels, dim3(1), dim3(1024), 0, st, f);
    hipLaunchKernelGGL(k_fill_levels, dim3(nb_nodes), dim3(256), 0, st, f);
    // dh starts as the upstream gradient of every node, dc as zero; d_x rows of internal nodes stay zero
    {
        ZeroList z{};
        z.src = g_h; z.dst = f.dh; z.n_copy = (size_t)n_nodes * H;
        z.p[0] = f.dc;     z.n[0] = lstm ? (size_t)n_nodes * H : 0;
        z.p[1] = d_x;      z.n[1] = (size_t)n_nodes * E;
        z.p[2] = d_b;      z.n[2] = (size_t)ng_cell * H;
        z.p[3] = d_b_leaf; z.n[3] = lstm ? (size_t)3 * H : 0;
        z.p[4] = rntn ? ctx->rntn_acc : d_u;   z.n[4] = rntn ? (size_t)2 * H * rntn_row + rntn_row : (size_t)2 * H * ng_cell * H;
        z.p[5] = d_w_leaf; z.n[5] = lstm ? (size_t)E * 3 * H : 0;
        hipLaunchKernelGGL(k_zero_many, dim3(1024), dim3(256), 0, st, z);
    }
    TL_HIP(hipGetLastError());
    const bool vec4 = H % 4 == 0 && (((uintptr_t)h & 15) == 0);
    // gate activations of the forward that wrote these h rows, if it kept them: no contraction to recompute
    const bool kept = lstm && ctx->gates_nodes == n_nodes && ctx->gates_h == h && ctx->gates != nullptr;
    const bool kept_v4 = H % 4 == 0 && (((uintptr_t)h | (uintptr_t)c) & 15) == 0;
    f.gates = kept ? ctx->gates : nullptr;
    // On request (tl_set_async_backward), gate gradients that need no contraction (kept activations; TreeRNN): all heights in
    // one persistent kernel, which finds the per-height lists on the device.  Nothing is read back, the call does not wait;
    // what the structure pass finds wrong with the batch is latched for tl_status, and every kernel below leaves at once.
    const bool persistent_ok = ctx->bw_grid > 0 && !rntn && (kept || !lstm) && n_int > 0;
    // TreeLSTM with H = 128, 256, 384 or 512: the operand gradient on weight-stationary workgroups (row offsets of dG in 32 bits)
    // (TreeRNN: the same sizes, K = H)
    const bool ws = persistent_ok && (lstm ? kept_v4 : vec4) && ctx->bw_ws_grid > 0 && ctx->ng_bwd_inner == 4 &&
                    (unsigned long long)n_int * (unsigned long long)dg_cols * 4ull < (1ull << 32);
    const bool heights_on_device = ctx->async_backward > 0 && persistent_ok;
    auto launch_all_heights = [&]() {
        BwdHeights b{};
        b.bwd4 = ctx->g_bwd_inner; b.bwd1 = ctx->g_bwd_inner1; b.ng_inner = ctx->ng_bwd_inner;
        b.dg_int = dg_int;
        b.kept_v4 = lstm ? (kept_v4 ? 1 : 0) : (vec4 ? 1 : 0);
        const bool v4 = vec4 && dg_cols % 4 == 0;
        typedef void (*bwh_kernel)(Fwd, BwdHeights);
        const bwh_kernel k = lstm ? (v4 ? bwh_kernel(k_backward_heights<true, true>) : bwh_kernel(k_backward_heights<true, false>))
                                  : (v4 ? bwh_kernel(k_backward_heights<false, true>) : bwh_kernel(k_backward_heights<false, false>));
        if (ws) {
            size_t lds = 0;
            const bwh_ws_kernel kw = backward_ws_kernel(lstm, ctx->bw_spw2, &lds);
            hipLaunchKernelGGL(kw, dim3(ctx->bw_ws_grid), dim3(WG_THREADS), lds, st, f, b);
        } else {
            hipLaunchKernelGGL(k, dim3(ctx->bw_grid), dim3(WG_THREADS), TILE_SMEM_BYTES, st, f, b);
        }
    };
    int n_levels = 0;
    const int levels_ahead = n_nodes + 2 < LEVELS_AHEAD ? n_nodes + 2 : LEVELS_AHEAD;   // offsets read back together with the control block
    bool status_pending = false;
    if (heights_on_device) {
        launch_all_heights();
    } else if (ws && ctx->async_backward == 0) {
        // The weight-stationary form is the faster one whatever the number of heights, and needs nothing from the host: the
        // structure pass's status is copied out in front of it, everything is enqueued, and the call then waits for that copy
        // alone (the device works on meanwhile) to return that status as it always has.
        if (!ctx->ev_ctl) TL_HIP(hipEventCreateWithFlags(&ctx->ev_ctl, hipEventDisableTiming));
        TL_HIP(hipMemcpyAsync(ctx->host_ctl, f.ctl, sizeof(Ctl), hipMemcpyDeviceToHost, st));
        TL_HIP(hipEventRecord(ctx->ev_ctl, st));
        status_pending = true;
        launch_all_heights();
    } else {
        if ((rc = read_ctl(ctx, levels_ahead)) != TL_OK) return rc;
        if (ctx->host_ctl->status != 0) return ctx->host_ctl->status;
        n_levels = ctx->host_ctl->n_levels;
        // Deep trees: two launches per height cost more than the persistent kernel's two grid barriers (a height of a few rows
        // takes 16 us in launches, 14 in the kernel), while the wide heights of shallow trees run faster as launches of their own.
        if (persistent_ok && ctx->async_backward == 0 && n_levels > BW_PERSISTENT_MIN_LEVELS) {
            launch_all_heights();
            n_levels = 0;
        }
    }
    auto gate_grad_kept = [&](bool inner, const Fwd &g, const int32_t *list, int rows) {
        typedef void (*kept_kernel)(Fwd, const int32_t *, int, int);
        const kept_kernel k = inner ? (kept_v4 ? kept_kernel(k_gate_grad_kept<true, 4>) : kept_kernel(k_gate_grad_kept<true, 1>))
                                    : (kept_v4 ? kept_kernel(k_gate_grad_kept<false, 4>) : kept_kernel(k_gate_grad_kept<false, 1>));
        long long blocks = ((long long)rows * (kept_v4 ? H / 4 : H) + 255) / 256;
        if (blocks > 8LL * ctx->n_cu) blocks = 8LL * ctx->n_cu;
        hipLaunchKernelGGL(k, dim3((unsigned)blocks), dim3(256), 0, st, g, list, rows, g.pos0);
    };
    if (n_levels > 1) {
        if (n_levels + 1 > levels_ahead) {
            TL_HIP(hipMemcpyAsync(ctx->host_levels, f.level_off, (size_t)(n_levels + 1) * 4, hipMemcpyDeviceToHost, st));
            TL_HIP(hipStreamSynchronize(st));
        }
        for (int lvl = n_levels - 1; lvl >= 1; --lvl) {     // roots first: a parent is always higher than its children
            const int lo = ctx->host_levels[lvl], rows = ctx->host_levels[lvl + 1] - lo;
            if (rows <= 0 || lo < 0 || lo + rows > n_int) return TL_EHIP;
            const LevelPlan plan = plan_level(rows, f.cap_tiles);
            Fwd g = f;
            g.dg = dg_int;
            g.pos0 = lo;
            if (rntn) {
                long long blocks = ((long long)rows * dg_cols + 255) / 256;
                if (blocks > 16LL * ctx->n_cu) blocks = 16LL * ctx->n_cu;
                hipLaunchKernelGGL(k_rntn_rows, dim3((unsigned)blocks), dim3(256), 0, st, g, (const int32_t *)(f.level_nodes + lo), rows, lo);
            } else if (!lstm) {
                typedef void (*rnn_kernel)(Fwd, const int32_t *, int, int);
                const bool v4 = H % 4 == 0 && (((uintptr_t)h & 15) == 0);
                long long blocks = ((long long)rows * (v4 ? H / 4 : H) + 255) / 256;
                if (blocks > 8LL * ctx->n_cu) blocks = 8LL * ctx->n_cu;
                hipLaunchKernelGGL(v4 ? rnn_kernel(k_rnn_gate_grad<4>) : rnn_kernel(k_rnn_gate_grad<1>), dim3((unsigned)blocks), dim3(256),
                                   0, st, g, (const int32_t *)(f.level_nodes + lo), rows, lo);
            } else if (kept)
                gate_grad_kept(true, g, (const int32_t *)(f.level_nodes + lo), rows);
            else
                hipLaunchKernelGGL(backward_kernel(EPI_BWD_INNER_GATES, vec4), dim3(plan.n_tiles * ctx->n_cg), dim3(WG_THREADS),
                                   TILE_SMEM_BYTES, st, g, (const int32_t *)(f.level_nodes + lo), rows, plan);
            // heights of few rows: one column block per group, so that four times as many workgroups share the
            // long K axis (5H) of the few tiles; otherwise four blocks per group, which reuse each gathered row more
            const int ng = (ctx->ng_bwd_inner == 4 && rows > 64) ? 4 : 1;
            g.bwd = (ctx->ng_bwd_inner == 4 && ng == 1) ? ctx->g_bwd_inner1 : ctx->g_bwd_inner;
            g.out_cols = 2 * H;
            g.n_cg = (2 * H / ng + HU - 1) / HU;
            hipLaunchKernelGGL(backward_kernel(ng == 4 ? EPI_BWD_INNER_OPERAND4 : EPI_BWD_INNER_OPERAND, vec4 && dg_cols % 4 == 0),
                               dim3(plan.n_tiles * g.n_cg), dim3(WG_THREADS),
                               TILE_SMEM_BYTES, st, g, (const int32_t *)(f.level_nodes + lo), rows, plan);
        }
    }
    if (!lstm) {
        hipLaunchKernelGGL(k_rnn_leaf_grad, dim3(1024), dim3(256), 0, st, f);       // leaves: d_x = dh
    } else {
        const LevelPlan plan = plan_level(n_leaf, f.cap_tiles);
        Fwd g = f;
        g.dg = dg_leaf;
        g.pos0 = 0;
        if (kept)
            gate_grad_kept(false, g, (const int32_t *)f.leaf_list, n_leaf);
        else
            hipLaunchKernelGGL(backward_kernel(EPI_BWD_LEAF_GATES, E % 4 == 0), dim3(plan.n_tiles * ctx->n_cg), dim3(WG_THREADS),
                               TILE_SMEM_BYTES, st, g, (const int32_t *)f.leaf_list, n_leaf, plan);
        g.bwd = ctx->g_bwd_leaf;
        g.out_cols = E;
        g.n_cg = (E / ctx->ng_bwd_leaf + HU - 1) / HU;
        // this contraction has few column groups (E = 300: five), so a round of the device's workgroups (two per CU) takes
        // more tiles than one of the forward's: the leaves are cut for that round, else a few tiles too many cost a second one
        const LevelPlan plan_op = plan_level(n_leaf, 2 * ctx->n_cu / g.n_cg > 0 ? 2 * ctx->n_cu / g.n_cg : 1);
        hipLaunchKernelGGL(backward_kernel(ctx->ng_bwd_leaf == 4 ? EPI_BWD_LEAF_OPERAND4 : EPI_BWD_LEAF_OPERAND, H % 4 == 0),
                           dim3(plan_op.n_tiles * g.n_cg), dim3(WG_THREADS),
                           TILE_SMEM_BYTES, st, g, (const int32_t *)f.leaf_list, n_leaf, plan_op);
    }
    // weight and bias gradients: contractions over all nodes, the node axis cut into slices so that a few
    // thousand workgroups are in flight
    auto slices = [&](int tiles, int rows) {
        int z = (8 * ctx->n_cu + tiles - 1) / tiles;
        const int max_z = (rows + 4 * WG_Q - 1) / (4 * WG_Q);
        if (z > max_z) z = max_z;
        return z < 1 ? 1 : z;
    };
    if (n_int > 0) {
        const dim3 grid((2 * H + WG_TILE - 1) / WG_TILE, (dg_cols + WG_TILE - 1) / WG_TILE, 1);
        const bool v4 = H % 4 == 0 && dg_cols % 4 == 0 && (((uintptr_t)h & 15) == 0);
        const wgrad_kernel wk = v4 ? wgrad_kernel(k_weight_grad<2, true>) : wgrad_kernel(k_weight_grad<2, false>);
        float *acc = rntn ? ctx->rntn_acc : d_u, *colsum = rntn ? ctx->rntn_acc + (size_t)2 * H * rntn_row : d_b;
        hipLaunchKernelGGL(wk, dim3(grid.x, grid.y, slices(grid.x * grid.y, n_int)), dim3(256), 0, st, f,
                           (const int32_t *)f.level_nodes, n_int, (const float *)h, H, (const float *)dg_int, dg_cols, acc, colsum);
    }
    if (rntn)      // back into the layouts of V, W and b (all zero when the batch has no internal node)
        hipLaunchKernelGGL(k_rntn_unpack, dim3(1024), dim3(256), 0, st, (const float *)ctx->rntn_acc,
                           (const float *)(ctx->rntn_acc + (size_t)2 * H * rntn_row), d_w_leaf, d_u, d_b, H);
    if (lstm) {
        const dim3 grid((E + WG_TILE - 1) / WG_TILE, (3 * H + WG_TILE - 1) / WG_TILE, 1);
        const bool v4 = E % 4 == 0 && H % 4 == 0;
        const wgrad_kernel wk = v4 ? wgrad_kernel(k_weight_grad<1, true>) : wgrad_kernel(k_weight_grad<1, false>);
        hipLaunchKernelGGL(wk, dim3(grid.x, grid.y, slices(grid.x * grid.y, n_leaf)), dim3(256), 0, st, f,
                           (const int32_t *)f.leaf_list, n_leaf, (const float *)ctx->emb, E, (const float *)dg_leaf, 3 * H, d_w_leaf,
                           d_b_leaf);
    }
    TL_HIP(hipGetLastError());
    if (status_pending) {
        TL_HIP(hipEventSynchronize(ctx->ev_ctl));
        if (ctx->host_ctl->status == 0 && !f.flow_roots && ctx->host_ctl->n_roots != n_trees) ctx->host_ctl->status = TL_ESTRUCT;
        if (ctx->host_ctl->status != 0) return ctx->host_ctl->status;
    }
    return TL_OK;
}

int tl_sgd_update(tl_ctx *ctx, float lr, int n_nodes, const int32_t *left, const int32_t *word, const float *d_u,
                  const float *d_b, const float *d_w_leaf, const float *d_b_leaf, const float *d_x, void *hip_stream)
{
    if (!ctx || !d_u || !d_b) return TL_EINVAL;
    const tl_config &cfg = ctx->cfg;
    if (cfg.precision != TL_F32) return TL_EINVAL;
    const bool lstm = cfg.cell == TL_TREELSTM, rntn = cfg.cell == TL_RNTN;
    if (lstm && (!d_w_leaf || !d_b_leaf)) return TL_EINVAL;
    if (rntn && !d_w_leaf) return TL_EINVAL;
    if (d_x && (!left || !word || n_nodes < 1)) return TL_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    const int H = cfg.hidden, E = cfg.embed_dim, ng_cell = lstm ? 5 : 1;
    SgdList z{};
    z.theta[0] = ctx->m_u;      z.grad[0] = d_u;      z.n[0] = (size_t)2 * H * ng_cell * H;
    z.theta[1] = ctx->m_b;      z.grad[1] = d_b;      z.n[1] = (size_t)ng_cell * H;
    z.theta[2] = lstm ? ctx->m_w_leaf : ctx->m_v; z.grad[2] = d_w_leaf; z.n[2] = lstm ? (size_t)E * 3 * H : rntn ? (size_t)H * 4 * H * H : 0;
    z.theta[3] = ctx->m_b_leaf; z.grad[3] = d_b_leaf; z.n[3] = lstm ? (size_t)3 * H : 0;
    hipLaunchKernelGGL(k_sgd_dense, dim3(1024), dim3(256), 0, st, z, lr);
    if (d_x) hipLaunchKernelGGL(k_sgd_embedding, dim3(1024), dim3(256), 0, st, ctx->emb, d_x, left, word, n_nodes, E, cfg.vocab, lr);
    TL_HIP(hipGetLastError());
    ctx->gates_nodes = 0;             // what a forward kept belongs to the old parameters
    return rntn ? pack_rntn_f32(ctx, st) : repack_f32(ctx, st);
}

int tl_get_params(tl_ctx *ctx, float *u, float *b, float *w_leaf, float *b_leaf, float *emb, void *hip_stream)
{
    if (!ctx) return TL_EINVAL;
    const tl_config &cfg = ctx->cfg;
    if (cfg.precision != TL_F32) return TL_EINVAL;
    const bool lstm = cfg.cell == TL_TREELSTM, rntn = cfg.cell == TL_RNTN;
    if (!lstm && b_leaf) return TL_EINVAL;
    if (!lstm && !rntn && w_leaf) return TL_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    const size_t H = cfg.hidden, E = cfg.embed_dim, ng_cell = lstm ? 5 : 1;
    if (u) TL_HIP(hipMemcpyAsync(u, ctx->m_u, 2 * H * ng_cell * H * sizeof(float), hipMemcpyDeviceToDevice, st));
    if (b) TL_HIP(hipMemcpyAsync(b, ctx->m_b, ng_cell * H * sizeof(float), hipMemcpyDeviceToDevice, st));
    if (w_leaf && rntn) TL_HIP(hipMemcpyAsync(w_leaf, ctx->m_v, H * 4 * H * H * sizeof(float), hipMemcpyDeviceToDevice, st));
    if (w_leaf && lstm) TL_HIP(hipMemcpyAsync(w_leaf, ctx->m_w_leaf, E * 3 * H * sizeof(float), hipMemcpyDeviceToDevice, st));
    if (b_leaf) TL_HIP(hipMemcpyAsync(b_leaf, ctx->m_b_leaf, 3 * H * sizeof(float), hipMemcpyDeviceToDevice, st));
    if (emb) TL_HIP(hipMemcpyAsync(emb, ctx->emb, (size_t)cfg.vocab * E * sizeof(float), hipMemcpyDeviceToDevice, st));
    return TL_OK;
}

int tl_set_keep_gates(tl_ctx *ctx, int on)
{
    if (!ctx) return TL_EINVAL;
    ctx->keep_gates = on != 0;
    if (!ctx->keep_gates) ctx->gates_nodes = 0;
    return TL_OK;
}

int tl_set_async_backward(tl_ctx *ctx, int on)
{
    if (!ctx) return TL_EINVAL;
    ctx->async_backward = on > 0 ? 1 : on < 0 ? -1 : 0;
    return TL_OK;
}

int tl_classify(tl_ctx *ctx, int n_rows, const float *h, const float *w_s, const float *b_s, int n_classes, float *probs,
                void *hip_stream)
{
    if (!ctx || !h || !w_s || !b_s || !probs) return TL_EINVAL;
    if (n_rows < 0 || n_classes < 1 || n_classes > CLS_MAX_CLASSES) return TL_EINVAL;
    if (n_rows == 0) return TL_OK;
    const int H = ctx->cfg.hidden, Hp = (H + 3) & ~3;
    const size_t lds = (size_t)n_classes * Hp * sizeof(float);
    if (lds > 96 * 1024) return TL_EINVAL;
    typedef void (*cls_kernel)(const float *, const float *, const float *, float *, int, int, int);
    const cls_kernel k = n_classes <= 2 ? k_classify<2> : n_classes <= 8 ? k_classify<8> : n_classes <= 16 ? k_classify<16> : k_classify<32>;
    TL_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    long long blocks = ((long long)n_rows + 15) / 16;
    const long long cap = (long long)ctx->n_cu * 8;
    if (blocks > cap) blocks = cap;
    hipLaunchKernelGGL(k, dim3((unsigned)blocks), dim3(256), lds, (hipStream_t)hip_stream, h, w_s, b_s, probs, n_rows, H, n_classes);
    TL_HIP(hipGetLastError());
    return TL_OK;
}

int tl_classify_backward(tl_ctx *ctx, int n_rows, const float *h, const float *w_s, const float *b_s, int n_classes,
                         const int32_t *label, float *d_logits, float *g_h, float *d_w_s, float *d_b_s, float *loss,
                         void *hip_stream)
{
    if (!ctx || !h || !w_s || !b_s || !label || !d_logits || !g_h || !d_w_s || !d_b_s || !loss) return TL_EINVAL;
    if (n_rows < 0 || n_classes < 1 || n_classes > CLS_MAX_CLASSES) return TL_EINVAL;
    const int H = ctx->cfg.hidden, Hp = (H + 3) & ~3, C = n_classes;
    const size_t lds = (size_t)C * Hp * sizeof(float);
    if (lds > 96 * 1024) return TL_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    hipLaunchKernelGGL(k_head_zero, dim3(16), dim3(256), 0, st, d_w_s, H * C, d_b_s, C, loss);
    TL_HIP(hipGetLastError());
    if (n_rows == 0) return TL_OK;
    typedef void (*bwd_kernel)(const float *, const float *, const float *, const int32_t *, float *, float *, float *, int, int, int);
    typedef void (*wg_kernel)(const float *, const float *, float *, float *, int, int, int);
    const bwd_kernel kb = C <= 2 ? k_classify_backward<2> : C <= 8 ? k_classify_backward<8> : C <= 16 ? k_classify_backward<16>
                                                                                                     : k_classify_backward<32>;
    const wg_kernel kw = C <= 2 ? k_head_weight_grad<2> : C <= 8 ? k_head_weight_grad<8> : C <= 16 ? k_head_weight_grad<16>
                                                                                                  : k_head_weight_grad<32>;
    TL_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kb), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    long long blocks = ((long long)n_rows + 15) / 16;
    const long long cap = (long long)ctx->n_cu * 4;
    if (blocks > cap) blocks = cap;
    hipLaunchKernelGGL(kb, dim3((unsigned)blocks), dim3(256), lds, st, h, w_s, b_s, label, d_logits, g_h, loss, n_rows, H, C);
    const int col_blocks = (H + 63) / 64;
    long long slices = ((long long)n_rows + 4 * HW_ROWS - 1) / (4 * HW_ROWS);
    const long long slice_cap = (2LL * ctx->n_cu + col_blocks - 1) / col_blocks;
    if (slices > slice_cap) slices = slice_cap;
    hipLaunchKernelGGL(kw, dim3((unsigned)col_blocks, (unsigned)slices), dim3(256), 0, st, h, d_logits, d_w_s, d_b_s, n_rows, H, C);
    TL_HIP(hipGetLastError());
    return TL_OK;
}

namespace {
typedef void (*td_kernel)(tl::TopDown);
td_kernel td_ws_kernel(int spw)
{
    switch (spw) {
    case 1: return tl::k_td_generate<true, 1>;
    case 2: return tl::k_td_generate<true, 2>;
    case 4: return tl::k_td_generate<true, 4>;
    case 5: return tl::k_td_generate<true, 5>;
    case 8: return tl::k_td_generate<true, 8>;
    default: return tl::k_td_generate<true, 16>;
    }
}
td_kernel td_flow_kernel(int spw)
{
    switch (spw) {
    case 1: return tl::k_td_flow<1>;
    case 2: return tl::k_td_flow<2>;
    case 4: return tl::k_td_flow<4>;
    case 5: return tl::k_td_flow<5>;
    case 8: return tl::k_td_flow<8>;
    default: return tl::k_td_flow<16>;
    }
}
// Data-flow form of the generator: workgroups that decide beside the sets that expand; rows of h and c that the reset
// kernel marks per call (16 MiB of the two arrays together, at least 1 024 rows; rows beyond are marked when reserved).
// It is the faster form while the trees in flight keep the sets of workgroups less than busy, i.e. for small batches
// (measured at H = 512: 1.3x at 1 to 4 roots, level at 32, 0.9x at 64): batches of more roots take the form with frontiers.
constexpr int TD_MIN_DECIDERS = 8, TD_MAX_DECIDERS = 64;
constexpr long long TD_MARK_BYTES = 16ll << 20;
constexpr int TD_FLOW_MAX_TREES = 32;
}  // namespace

int tl_td_create(int hidden, const float *u_td, const float *b_td, const float *w_stop, float b_stop, int spin_limit,
                 tl_td_ctx **out)
{
    if (!out) return TL_EINVAL;
    *out = nullptr;
    if (!u_td || !b_td || !w_stop || hidden < 1 || hidden > (1 << 14) || spin_limit < 0) return TL_EINVAL;
    tl_td_ctx *ctx = new (std::nothrow) tl_td_ctx();
    if (!ctx) return TL_ENOMEM;
    const int H = hidden;
    int rc = [&]() -> int {
        TL_HIP(hipGetDevice(&ctx->device));
        hipDeviceProp_t prop;
        TL_HIP(hipGetDeviceProperties(&prop, ctx->device));
        ctx->n_cu = prop.multiProcessorCount;
        ctx->H = H;
        ctx->n_cg = (H + HU - 1) / HU;
        ctx->b_stop = b_stop;
        ctx->spin_limit = spin_limit > 0 ? spin_limit : DEFAULT_SPIN_LIMIT;
        // weight-stationary expansion step: H a multiple of 4, the K axis (H) within 16 k-steps of 16 per wave, and a grid
        // that holds every (side, column group) pair at least once
        ctx->spw = 0;
        if (H % 4 == 0 && ctx->n_cu >= 2 * ctx->n_cg) {
            const int needed = round_up(H, KC) / STEP_K / 4;
            for (int sz : WS_SIZES)
                if (sz >= needed) { ctx->spw = sz; break; }
        }
        // one side's [H x 4H] block of u_td, made contiguous for the packer
        float *block = nullptr;
        TL_HIP(hipMalloc(&block, (size_t)H * 4 * H * sizeof(float)));
        for (int sd = 0; sd < 2; ++sd) {
            const hipError_t e = hipMemcpy2D(block, (size_t)4 * H * sizeof(float), u_td + (size_t)sd * 4 * H, (size_t)8 * H * sizeof(float),
                                             (size_t)4 * H * sizeof(float), (size_t)H, hipMemcpyDeviceToDevice);
            if (e != hipSuccess) { (void)hipFree(block); return TL_EHIP; }
            const int prc = pack_gemm(block, b_td + (size_t)sd * 4 * H, 4, H, 1, H, ctx->n_cg, 4 * ctx->spw, false, &ctx->side[sd], &ctx->wp[sd], &ctx->bp[sd]);
            if (prc != TL_OK) { (void)hipFree(block); return prc; }
            if (hipDeviceSynchronize() != hipSuccess) { (void)hipFree(block); return TL_EHIP; }
        }
        TL_HIP(hipFree(block));
        TL_HIP(hipMalloc(&ctx->w_stop, (size_t)round_up(H, 4) * sizeof(float)));
        TL_HIP(hipMemset(ctx->w_stop, 0, (size_t)round_up(H, 4) * sizeof(float)));
        TL_HIP(hipMemcpy(ctx->w_stop, w_stop, (size_t)H * sizeof(float), hipMemcpyDeviceToDevice));
        TL_HIP(hipMalloc(&ctx->zeros, 4096));
        TL_HIP(hipMemset(ctx->zeros, 0, 4096));
        TL_HIP(hipMalloc(&ctx->ctl, sizeof(Ctl)));
        TL_HIP(hipMemset(ctx->ctl, 0, sizeof(Ctl)));
        TL_HIP(hipHostMalloc(&ctx->host_ctl, sizeof(Ctl), hipHostMallocDefault));
        TL_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(k_td_generate<true>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (int)TILE_SMEM_BYTES));
        TL_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(k_td_generate<false>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (int)TILE_SMEM_BYTES));
        if (ctx->spw > 0) {
            TL_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(td_ws_kernel(ctx->spw)), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)ws_lds_bytes(ctx->spw, false)));
            TL_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(td_flow_kernel(ctx->spw)), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)ws_lds_bytes(ctx->spw, false)));
            // every workgroup of the data-flow form waits for others: all of them must be resident together
            int occ = 0;
            TL_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, reinterpret_cast<const void *>(td_flow_kernel(ctx->spw)), WG_THREADS,
                                                                ws_lds_bytes(ctx->spw, false)));
            // one workgroup per CU where that holds a set and the deciders (measured: a second one per CU, for more sets, is no
            // faster), two where it takes them
            const int needed = 2 * ctx->n_cg + TD_MIN_DECIDERS;
            ctx->flow_grid = occ >= 1 && ctx->n_cu >= needed ? ctx->n_cu : occ >= 2 && 2 * ctx->n_cu >= needed ? 2 * ctx->n_cu : 0;
        }
        TL_HIP(hipDeviceSynchronize());
        return TL_OK;
    }();
    if (rc != TL_OK) {
        td_free(ctx);
        return rc;
    }
    *out = ctx;
    return TL_OK;
}

int tl_td_generate(tl_td_ctx *ctx, int n_trees, int max_nodes, int max_depth, float *h, float *c, int32_t *parent,
                   int32_t *left, int32_t *right, int32_t *depth, float *score, int32_t *counts, void *hip_stream)
{
    if (!ctx || !h || !c || !parent || !left || !right || !depth || !score || !counts) return TL_EINVAL;
    if (n_trees < 1 || max_nodes < n_trees || max_depth < 0) return TL_EINVAL;
    if ((unsigned long long)max_nodes * (unsigned long long)ctx->H >= (1ull << 40)) return TL_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    TopDown a{};
    a.f.h = h; a.f.c = c; a.f.H = ctx->H; a.f.n_cg = ctx->n_cg;
    a.f.zeros = ctx->zeros; a.f.ctl = ctx->ctl; a.f.spin_limit = ctx->spin_limit;
    a.f.n_trees = n_trees; a.f.n_nodes = max_nodes;
    a.side[0] = ctx->side[0]; a.side[1] = ctx->side[1];
    a.w_stop = ctx->w_stop; a.b_stop = ctx->b_stop;
    a.n_trees = n_trees; a.max_depth = max_depth; a.max_nodes = max_nodes;
    a.parent = parent; a.left = left; a.right = right; a.depth = depth; a.score = score; a.counts = counts;
    // the grid barrier in its one-level form: at most FLAT_BARRIER_MAX workgroups, all resident (one per CU)
    int grid = ctx->n_cu < (int)FLAT_BARRIER_MAX ? ctx->n_cu : (int)FLAT_BARRIER_MAX;
    if (grid < 1) grid = 1;
    const bool vec4 = ctx->H % 4 == 0 && (((uintptr_t)h | (uintptr_t)c) & 15) == 0;
    // the weight-stationary cell addresses rows with 24-bit row numbers and 32-bit byte offsets
    const bool ws_range = max_nodes < (1 << 24) && (unsigned long long)max_nodes * ctx->H * 4ull < (1ull << 32);
    const bool flow = vec4 && ctx->spw > 0 && ws_range && ctx->flow_grid > 0 && n_trees <= TD_FLOW_MAX_TREES;
    if (flow) {
        const int combos = 2 * ctx->n_cg;
        a.n_slots = (ctx->flow_grid - TD_MIN_DECIDERS) / combos;
        a.n_dec = ctx->flow_grid - a.n_slots * combos < TD_MAX_DECIDERS ? ctx->flow_grid - a.n_slots * combos : TD_MAX_DECIDERS;
        long long marked = TD_MARK_BYTES / (8ll * ctx->H);
        if (marked < n_trees + 1024) marked = n_trees + 1024;
        a.marked_rows = marked < max_nodes ? (int)marked : max_nodes;
    }
    hipLaunchKernelGGL(k_td_reset, dim3(flow ? 2 * ctx->n_cu : 4), dim3(256), 0, st, a);
    if (flow)
        hipLaunchKernelGGL(td_flow_kernel(ctx->spw), dim3(a.n_slots * 2 * ctx->n_cg + a.n_dec), dim3(WG_THREADS), ws_lds_bytes(ctx->spw, false),
                           st, a);
    else if (vec4 && ctx->spw > 0 && ws_range && grid >= 2 * ctx->n_cg)
        hipLaunchKernelGGL(td_ws_kernel(ctx->spw), dim3(grid), dim3(WG_THREADS), ws_lds_bytes(ctx->spw, false), st, a);
    else if (vec4)
        hipLaunchKernelGGL(k_td_generate<true>, dim3(grid), dim3(WG_THREADS), TILE_SMEM_BYTES, st, a);
    else
        hipLaunchKernelGGL(k_td_generate<false>, dim3(grid), dim3(WG_THREADS), TILE_SMEM_BYTES, st, a);
    TL_HIP(hipGetLastError());
    ctx->last_stream = st;
    ctx->ran = true;
    return TL_OK;
}

int tl_td_status(tl_td_ctx *ctx)
{
    if (!ctx) return TL_EINVAL;
    if (!ctx->ran) return TL_OK;
    TL_HIP(hipMemcpyAsync(ctx->host_ctl, ctx->ctl, sizeof(Ctl), hipMemcpyDeviceToHost, ctx->last_stream));
    TL_HIP(hipStreamSynchronize(ctx->last_stream));
    return ctx->host_ctl->status;
}

int tl_td_destroy(tl_td_ctx *ctx)
{
    if (!ctx) return TL_EINVAL;
    (void)hipDeviceSynchronize();
    td_free(ctx);
    return TL_OK;
}

const char *tl_strerror(int code)
{
    switch (code) {
    case TL_OK: return "ok";
    case TL_EINVAL: return "invalid argument";
    case TL_ENOMEM: return "out of memory";
    case TL_EHIP: return "HIP runtime error";
    case TL_ESTRUCT: return "malformed tree batch";
    case TL_ESTALL: return "scheduler made no progress (unreachable nodes)";
    case TL_ELIMIT: return "batch larger than the fixed workspace of tl_forward_noalloc";
    default: return "unknown error";
    }
}

int tl_destroy(tl_ctx *ctx)
{
    if (!ctx) return TL_EINVAL;
    (void)hipDeviceSynchronize();
    free_all(ctx);
    return TL_OK;
}

}  // extern "C"
