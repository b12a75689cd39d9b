// The fused cell: gather -> MFMA contraction -> gate epilogue -> h/c rows.
//
// One call evaluates up to TILE_ROWS nodes for one column group of HU hidden units:
//   leaf tile      A row = embedding row of the leaf's word            (Figure 2, base case)
//   internal tile  A row = [h(left child) ; h(right child)]            (Figure 2, recursive case)
// G = A * W (+ bias) is accumulated in fp32 on 16x16 MFMA tiles; the packed weights put all
// gates of a hidden unit into the same lane, so sigmoid/tanh, the c update and the h output
// are computed on the accumulators and written straight to the node-major h/c arrays.
//
// Two data paths feed the MFMAs:
//   staged  (33..64 rows) A and B chunks go through LDS, shared by the four waves, each wave
//           owning one block of 16 rows;
//   direct  (1..32 rows)  few rows mean the K axis is split between the waves instead, so no
//           two waves need the same weights: every wave loads its operands from global memory
//           straight into registers, several k-steps ahead, and the partial sums meet in LDS.
//           With so few rows the tile is latency-bound, and this path has no barrier in its loop.
// Template parameter COH selects device-scope loads/stores for h and c (see common.hpp); it is
// set inside persistent kernels, where producers and consumers of a row run concurrently.
#pragma once

#include "common.hpp"

namespace tl {

enum Epi {
    EPI_LSTM_LEAF = 0, EPI_LSTM_INNER = 1, EPI_RNN_INNER = 2, EPI_RNTN_INNER = 3,
    // backward pass (backward.hpp): gate gradients of internal nodes / leaves (the forward contraction is
    // recomputed), and the gradient sent to the operand rows (gate gradients times transposed weights)
    EPI_BWD_INNER_GATES = 4, EPI_BWD_INNER_OPERAND = 5, EPI_BWD_LEAF_GATES = 6, EPI_BWD_LEAF_OPERAND = 7,
    // top-down generation (topdown.hpp): the child on one side of a node from the node's own state
    EPI_TD_CHILD = 8,
    // the two operand-gradient contractions with four blocks of output columns per column group instead of
    // one (output widths that are multiples of 4): every gathered row is reused four times as often
    EPI_BWD_INNER_OPERAND4 = 9, EPI_BWD_LEAF_OPERAND4 = 10
};
constexpr bool epi_is_backward(int epi)
{
    return (epi >= EPI_BWD_INNER_GATES && epi <= EPI_BWD_LEAF_OPERAND) || epi == EPI_BWD_INNER_OPERAND4 || epi == EPI_BWD_LEAF_OPERAND4;
}
constexpr bool epi_is_operand_gradient(int epi)
{
    return epi == EPI_BWD_INNER_OPERAND || epi == EPI_BWD_LEAF_OPERAND || epi == EPI_BWD_INNER_OPERAND4 || epi == EPI_BWD_LEAF_OPERAND4;
}

template <int EPI> struct EpiTraits;
template <> struct EpiTraits<EPI_LSTM_LEAF>  { static constexpr int NG = 3, SEG = 1; };
template <> struct EpiTraits<EPI_LSTM_INNER> { static constexpr int NG = 5, SEG = 2; };
template <> struct EpiTraits<EPI_RNN_INNER>  { static constexpr int NG = 1, SEG = 2; };
template <> struct EpiTraits<EPI_RNTN_INNER> { static constexpr int NG = 1, SEG = 2; };
template <> struct EpiTraits<EPI_BWD_INNER_GATES>   { static constexpr int NG = 5, SEG = 2; };
template <> struct EpiTraits<EPI_BWD_INNER_OPERAND> { static constexpr int NG = 1, SEG = 1; };
template <> struct EpiTraits<EPI_BWD_LEAF_GATES>    { static constexpr int NG = 3, SEG = 1; };
template <> struct EpiTraits<EPI_BWD_LEAF_OPERAND>  { static constexpr int NG = 1, SEG = 1; };
template <> struct EpiTraits<EPI_TD_CHILD>          { static constexpr int NG = 4, SEG = 1; };
template <> struct EpiTraits<EPI_BWD_INNER_OPERAND4> { static constexpr int NG = 4, SEG = 1; };
template <> struct EpiTraits<EPI_BWD_LEAF_OPERAND4>  { static constexpr int NG = 4, SEG = 1; };

// LDS carve-up (dynamic shared memory, 16-byte aligned).
struct TileSmem {
    float a[2][TILE_ROWS * A_LD];                   // A chunks, double buffered
    floatx4 b[2][(KC / STEP_K) * MAX_GATES * 64];    // B chunks, double buffered
    int node[TILE_ROWS];                             // node index per row (-1: unused row)
    int src0[TILE_ROWS];                             // first source row (word id / left child), -1: none
    int src1[TILE_ROWS];                             // second source row (right child)
    int cmd[8];                                      // scheduler broadcast slots
};
constexpr size_t TILE_SMEM_BYTES = sizeof(TileSmem);

// v_rcp_f32 (1 ulp) rather than a correctly rounded division, which costs ten instructions
__device__ inline float sigmoid_f(float x) { return __builtin_amdgcn_rcpf(1.f + __expf(-x)); }
__device__ inline float tanh_f(float x)
{
    // 1 - 2/(1+e^{2x}); the clamp keeps e^{2x} finite, beyond it tanh is 1 to fp32 precision
    float t = __expf(2.f * fminf(fmaxf(x, -15.f), 15.f));
    return __builtin_fmaf(-2.f, __builtin_amdgcn_rcpf(1.f + t), 1.f);
}

// Gate functions of the three cells on finished pre-activations (bias included).  Every data path
// calls these same functions, and the multiply-adds are spelled out as fused operations (left to
// the compiler, the choice of which product to fuse differs between call sites), so that a
// node's h and c do not depend on the path that made them.
// `keep`, when not null, receives the gate activations for the backward pass (Section 4.2.2:
// forward values are kept per call instance): i, o, u of a leaf at keep[0], keep[H], keep[2H];
// i, f_l, f_r, o, u of an internal node at keep[0] .. keep[4H].
__device__ inline void lstm_leaf_out(float gi, float go, float gu, float *c, float *h, float *keep = nullptr, int H = 0)
{
    const float i = sigmoid_f(gi), og = sigmoid_f(go), u = tanh_f(gu);
    const float cc = i * u;
    *c = cc;
    *h = og * tanh_f(cc);
    if (keep) {
        keep[0] = i;
        keep[H] = og;
        keep[2 * H] = u;
    }
}
__device__ inline void lstm_inner_out(float gi, float gfl, float gfr, float go, float gu, float cl, float cr, float *c,
                                      float *h, float *keep = nullptr, int H = 0)
{
    const float i = sigmoid_f(gi), fl = sigmoid_f(gfl), fr = sigmoid_f(gfr), og = sigmoid_f(go), u = tanh_f(gu);
    const float cc = __builtin_fmaf(fr, cr, __builtin_fmaf(fl, cl, i * u));
    *c = cc;
    *h = og * tanh_f(cc);
    if (keep) {
        keep[0] = i;
        keep[H] = fl;
        keep[2 * H] = fr;
        keep[3 * H] = og;
        keep[4 * H] = u;
    }
}
// Where a node's kept gate activations start for hidden unit hu; null when they are not kept.
__device__ inline float *kept_gates(const Fwd &f, int node, int hu)
{
    return f.gates ? f.gates + (size_t)node * (5 * f.H) + hu : nullptr;
}

// Fills node/src0/src1 of one row.  Rows without a node are marked unused.  Caller synchronises.
// `pos` is the row's position in the list the tile was cut from: the backward kernels that
// gather rows of gate gradients find them by that position.
template <int EPI, typename Smem>
__device__ inline void tile_set_rows(Smem &sm, const Fwd &f, int row, int node, int pos = 0)
{
    if (row >= TILE_ROWS) return;
    int s0 = -1, s1 = -1;
    if (node >= 0) {
        if (EPI == EPI_LSTM_LEAF || EPI == EPI_BWD_LEAF_GATES) {
            s0 = f.word[node];
        } else if (epi_is_operand_gradient(EPI)) {
            s0 = pos;
        } else {
            s0 = f.left[node];
            s1 = f.right[node];
        }
    }
    sm.node[row] = node;
    sm.src0[row] = s0;
    sm.src1[row] = s1;
}

// Loads one 4-float granule of a gathered A row: K position k of the padded axis.  Branch-free
// and select-free: whatever lies outside the row is read from a block of zeros in device
// memory, so that nothing has to wait for the load until the MFMA (or the LDS store) that uses
// it, and the loads of several k-steps can be in flight together.
template <int SEG, bool VEC4, bool COH>
__device__ inline floatx4 load_a_granule(const float *__restrict__ table, const float *__restrict__ zeros, int L, int Lp,
                                         int s0, int s1, int k)
{
    const int seg = (SEG == 2 && k >= Lp) ? 1 : 0;
    const int off = k - seg * Lp;
    const int src = seg ? s1 : s0;
    const bool ok = src >= 0 && off < L;
    const float *p = ok ? table + ((size_t)src * L + off) : zeros;
    floatx4 v;
    if (VEC4) {
        v = ld_f4<COH>(p);
    } else {
        // rows need not be 16-byte aligned here; element i is real iff off + i < L
        const int n = ok ? L - off : 4;
        v.x = ld_f<COH>(p);
        v.y = ld_f<COH>(n > 1 ? p + 1 : zeros);
        v.z = ld_f<COH>(n > 2 ? p + 2 : zeros);
        v.w = ld_f<COH>(n > 3 ? p + 3 : zeros);
    }
    return v;
}

template <int EPI, int NG, bool COH>
__device__ inline void bwd_epilogue(const TileSmem &sm, const Fwd &f, const Gemm &gm, const floatx4 (&acc)[NG], int rb,
                                    int count, int cg, int lane);   // backward.hpp

// Gate functions and h/c stores for the 4 accumulator rows a lane holds.
template <int EPI, bool COH, int NG>
__device__ inline void tile_epilogue(const TileSmem &sm, const Fwd &f, const Gemm &gm, const floatx4 (&acc)[NG],
                                     int rb, int count, int cg, int lane)
{
    if constexpr (epi_is_backward(EPI)) {
        bwd_epilogue<EPI, NG, COH>(sm, f, gm, acc, rb, count, cg, lane);
        return;
    }
    const int hu = cg * HU + (lane & 15);
    const int H = f.H;
    if (hu >= H) return;
    if constexpr (EPI == EPI_TD_CHILD) {
        // rows: node = the child to write, src0 = its parent; gates i, f, o, u of an LSTM step along the edge
        float bias[NG];
#pragma unroll
        for (int g = 0; g < NG; ++g) bias[g] = gm.bp[(cg * NG + g) * HU + (lane & 15)];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int row = rb * 16 + (lane >> 4) * 4 + v;
            if (row >= count) continue;
            const int node = sm.node[row];
            if (node < 0) continue;
            const float cp = ld_f<COH>(f.c + (size_t)sm.src0[row] * H + hu);
            const float i = sigmoid_f(acc[0][v] + bias[0]), fg = sigmoid_f(acc[1][v] + bias[1]);
            const float og = sigmoid_f(acc[2][v] + bias[2]), u = tanh_f(acc[3][v] + bias[3]);
            const float cc = __builtin_fmaf(fg, cp, i * u);
            st_f<COH>(f.c + (size_t)node * H + hu, cc);
            st_f<COH>(f.h + (size_t)node * H + hu, og * tanh_f(cc));
        }
        return;
    }
    float bias[NG];
#pragma unroll
    for (int g = 0; g < NG; ++g) bias[g] = gm.bp[(cg * NG + g) * HU + (lane & 15)];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int row = rb * 16 + (lane >> 4) * 4 + v;
        if (row >= count) continue;
        const int node = sm.node[row];
        if (node < 0) continue;
        const size_t o = (size_t)node * H + hu;
        if (EPI == EPI_LSTM_LEAF) {
            float cc, hh;
            lstm_leaf_out(acc[0][v] + bias[0], acc[1][v] + bias[1], acc[2][v] + bias[2], &cc, &hh, kept_gates(f, node, hu), H);
            st_f<COH>(f.c + o, cc);
            st_f<COH>(f.h + o, hh);
            if (f.hb) st_h<COH>(f.hb + (size_t)node * f.hs + hu, bf16_bits(hh));
        } else if (EPI == EPI_LSTM_INNER) {
            const float cl = ld_f<COH>(f.c + (size_t)sm.src0[row] * H + hu);
            const float cr = ld_f<COH>(f.c + (size_t)sm.src1[row] * H + hu);
            float cc, hh;
            lstm_inner_out(acc[0][v] + bias[0], acc[1][v] + bias[1], acc[2][v] + bias[2], acc[3][v] + bias[3],
                           acc[4][v] + bias[4], cl, cr, &cc, &hh, kept_gates(f, node, hu), H);
            st_f<COH>(f.c + o, cc);
            st_f<COH>(f.h + o, hh);
            if (f.hb) st_h<COH>(f.hb + (size_t)node * f.hs + hu, bf16_bits(hh));
        } else {
            const float hh = tanh_f(acc[0][v] + bias[0]);
            st_f<COH>(f.h + o, hh);
            if (f.hb) st_h<COH>(f.hb + (size_t)node * f.hs + hu, bf16_bits(hh));
        }
    }
}

// Summation order of the fp32 contraction, the same on every data path: the padded K axis is cut
// into four equal quarters of k-steps; within a quarter the k-steps are accumulated in increasing
// order on one MFMA accumulator chain, and the four quarter sums P0..P3 are added as
// ((P0 + P1) + P2) + P3 before the bias.  Whether a wave owns one quarter, two, or all four
// depends on how many rows a tile has, but the bits of a node's result do not.
//
// The waves that hold later quarters hand them through LDS (the B buffers, which nobody reads
// any more) to the wave that holds P0 of the same row block.  KS waves share a row block; with
// KS == 2 a wave holds two quarters: `first` and `acc`.
template <int NG>
__device__ inline void ksplit_reduce(TileSmem &sm, floatx4 (&acc)[NG], const floatx4 (&first)[NG], int KS, int ks, int rb,
                                     int lane)
{
    float *red = reinterpret_cast<float *>(&sm.b[0][0]);    // [rb 0..1][quarter][g*4+v][lane]: 2*4*20*64 floats = sizeof(b)
    auto at = [&](int q, int g, int v) { return ((rb * 4 + q) * NG * 4 + g * 4 + v) * 64 + lane; };
    if (ks > 0) {
#pragma unroll
        for (int g = 0; g < NG; ++g)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                if (KS == 4) {
                    red[at(ks, g, v)] = acc[g][v];
                } else {
                    red[at(2, g, v)] = first[g][v];
                    red[at(3, g, v)] = acc[g][v];
                }
            }
    }
    __syncthreads();
    if (ks == 0) {
        if (KS == 2) {
#pragma unroll
            for (int g = 0; g < NG; ++g) acc[g] = first[g] + acc[g];
        }
        for (int q = KS == 4 ? 1 : 2; q < 4; ++q) {
#pragma unroll
            for (int g = 0; g < NG; ++g)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[g][v] += red[at(q, g, v)];
        }
    }
}

// ---- direct path: 1..32 rows ------------------------------------------------------------
template <int EPI, bool VEC4, bool COH>
__device__ inline void cell_tile_direct(TileSmem &sm, const Fwd &f, const Gemm &gm, const float *__restrict__ table,
                                        int count, int cg)
{
    constexpr int NG = EpiTraits<EPI>::NG;
    constexpr int SEG = EpiTraits<EPI>::SEG;
    constexpr int U = NG >= 5 ? (COH ? 2 : 4) : 4;   // k-steps per register group (two groups are in flight)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nrb = (count + 15) >> 4;          // 1 or 2
    const int KS = nrb == 1 ? 4 : 2;            // waves per row block; a wave owns 4 / KS quarters of K
    const int rb = KS == 4 ? 0 : (wave & 1);
    const int ks = KS == 4 ? wave : (wave >> 1);
    const int L = gm.L, Lp = gm.Lp;
    const int n_steps = gm.n_chunks * (KC / STEP_K);
    const int quarter = n_steps >> 2;           // n_steps is a multiple of 4
    const floatx4 *wp = reinterpret_cast<const floatx4 *>(gm.wp) + (size_t)cg * n_steps * NG * 64 + lane;
    const int row = rb * 16 + (lane & 15);
    const int s0 = sm.src0[row], s1 = sm.src1[row];   // -1 beyond count
    const int kl = (lane >> 4) * 4;

    floatx4 acc[NG], first[NG];
#pragma unroll
    for (int g = 0; g < NG; ++g) acc[g] = first[g] = floatx4{0.f, 0.f, 0.f, 0.f};

    floatx4 a0[U], b0[U][NG], a1[U], b1[U][NG];
    int s_lo = 0, s_hi = 0;                           // k-steps of the quarter being accumulated
    auto load_group = [&](int grp, floatx4 (&a)[U], floatx4 (&b)[U][NG]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            // a k-step past the end re-reads the last one with a zeroed A operand
            const int s_raw = s_lo + grp * U + u;
            const bool real = s_raw < s_hi;
            const int s = real ? s_raw : s_hi - 1;
            a[u] = load_a_granule<SEG, VEC4, COH>(table, f.zeros, L, Lp, real ? s0 : -1, real ? s1 : -1, s * STEP_K + kl);
#pragma unroll
            for (int g = 0; g < NG; ++g) b[u][g] = wp[(size_t)(s * NG + g) * 64];
        }
    };
    auto mma_group = [&](const floatx4 (&a)[U], const floatx4 (&b)[U][NG]) {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int g = 0; g < NG; ++g)
                    acc[g] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[u][i], b[u][g][i], acc[g], 0, 0, 0);
    };
    // Two register groups alternate: the loads of one group are issued, then the MFMAs of the
    // other run.  The scheduling barriers keep the compiler from sinking the loads below the
    // MFMAs (which would expose the full memory latency once per group).  Nothing in the loop is
    // conditional: a branch around loads would make the wait counters at its join pessimistic.
    // Groups past the end multiply a zero A operand.
    const int n_q = 4 / KS;
    const int n_groups = (quarter + U - 1) / U;
    for (int qi = 0; qi < n_q; ++qi) {
        s_lo = (ks * n_q + qi) * quarter;
        s_hi = s_lo + quarter;
        load_group(0, a0, b0);
        for (int grp = 0; grp < n_groups; grp += 2) {
            load_group(grp + 1, a1, b1);
            __builtin_amdgcn_sched_barrier(0);
            mma_group(a0, b0);
            __builtin_amdgcn_sched_barrier(0);
            load_group(grp + 2, a0, b0);
            __builtin_amdgcn_sched_barrier(0);
            mma_group(a1, b1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (qi + 1 < n_q) {                           // the quarter sum is complete: start the next on a fresh chain
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                first[g] = acc[g];
                acc[g] = floatx4{0.f, 0.f, 0.f, 0.f};
            }
        }
    }
    ksplit_reduce<NG>(sm, acc, first, KS, ks, rb, lane);
    if (ks == 0) tile_epilogue<EPI, COH, NG>(sm, f, gm, acc, rb, count, cg, lane);
}

// ---- staged path: 33..64 rows -----------------------------------------------------------
template <int EPI, bool VEC4, bool COH>
__device__ inline void cell_tile_staged(TileSmem &sm, const Fwd &f, const Gemm &gm, const float *__restrict__ table,
                                        int count, int cg)
{
    constexpr int NG = EpiTraits<EPI>::NG;
    constexpr int SEG = EpiTraits<EPI>::SEG;
    constexpr int STEPS = KC / STEP_K;          // 4 k-steps per chunk
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nrb = (count + 15) >> 4;          // 3 or 4 row blocks, one per wave
    const int rb = wave;
    const bool active = rb < nrb;
    const int L = gm.L, Lp = gm.Lp;
    const int n_steps = gm.n_chunks * STEPS;
    const floatx4 *wp = reinterpret_cast<const floatx4 *>(gm.wp) + (size_t)cg * n_steps * NG * 64;

    // a wave walks all four quarters of K here: `acc` is the chain of the current quarter, `total`
    // the sum of the finished ones (see ksplit_reduce for the order)
    floatx4 acc[NG], total[NG];
#pragma unroll
    for (int g = 0; g < NG; ++g) acc[g] = total[g] = floatx4{0.f, 0.f, 0.f, 0.f};
    const int quarter = n_steps >> 2;
    int to_boundary = quarter;

    // staging registers: A granules (rows tid/16 + 16 j, granule tid%16), B float4s
    floatx4 ra[4], rbuf[NG];
    const int a_row0 = tid >> 4, a_k4 = tid & 15;
    int s0[4], s1[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        int row = a_row0 + 16 * j;
        s0[j] = row < nrb * 16 ? sm.src0[row] : -1;
        s1[j] = row < nrb * 16 ? sm.src1[row] : -1;
    }
    auto load_chunk = [&](int chunk) {
        const int k = chunk * KC + a_k4 * 4;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (j < nrb) ra[j] = load_a_granule<SEG, VEC4, COH>(table, f.zeros, L, Lp, s0[j], s1[j], k);
        const floatx4 *src = wp + (size_t)chunk * STEPS * NG * 64;
#pragma unroll
        for (int j = 0; j < NG; ++j) rbuf[j] = src[tid + WG_THREADS * j];
    };
    auto store_chunk = [&](int buf) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (j < nrb)
                *reinterpret_cast<floatx4 *>(&sm.a[buf][(a_row0 + 16 * j) * A_LD + a_k4 * 4]) = ra[j];
#pragma unroll
        for (int j = 0; j < NG; ++j) sm.b[buf][tid + WG_THREADS * j] = rbuf[j];
    };

    load_chunk(0);
    store_chunk(0);
    __syncthreads();
    for (int chunk = 0; chunk < gm.n_chunks; ++chunk) {
        const int buf = chunk & 1;
        const bool more = chunk + 1 < gm.n_chunks;
        if (more) load_chunk(chunk + 1);
        __builtin_amdgcn_sched_barrier(0);   // keep the global loads ahead of the MFMAs that hide them
        if (active) {
            const float *arow = &sm.a[buf][(rb * 16 + (lane & 15)) * A_LD + (lane >> 4) * 4];
            // the operands of a k-step are read from LDS one k-step ahead, so that the read runs under MFMAs
            floatx4 av_next = *reinterpret_cast<const floatx4 *>(arow);
            floatx4 bv_next[NG];
#pragma unroll
            for (int g = 0; g < NG; ++g) bv_next[g] = sm.b[buf][g * 64 + lane];
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
                if (to_boundary == 0) {                 // uniform: a quarter of K is complete
#pragma unroll
                    for (int g = 0; g < NG; ++g) {
                        total[g] += acc[g];
                        acc[g] = floatx4{0.f, 0.f, 0.f, 0.f};
                    }
                    to_boundary = quarter;
                }
                --to_boundary;
                const floatx4 av = av_next;
                floatx4 bv[NG];
#pragma unroll
                for (int g = 0; g < NG; ++g) bv[g] = bv_next[g];
                if (s + 1 < STEPS) {
                    av_next = *reinterpret_cast<const floatx4 *>(arow + (s + 1) * STEP_K);
#pragma unroll
                    for (int g = 0; g < NG; ++g) bv_next[g] = sm.b[buf][((s + 1) * NG + g) * 64 + lane];
                }
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int g = 0; g < NG; ++g)
                        acc[g] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[i], bv[g][i], acc[g], 0, 0, 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        if (more) store_chunk(buf ^ 1);
        __syncthreads();
    }
    if (active) {
#pragma unroll
        for (int g = 0; g < NG; ++g) total[g] += acc[g];
        tile_epilogue<EPI, COH, NG>(sm, f, gm, total, rb, count, cg, lane);
    }
}

// ---- staged path with bfloat16 operands ---------------------------------------------------
// Same data flow as above for 1..64 rows, but the MFMA operands are bfloat16: the gathered rows
// are rounded to nearest-even when they are stored to LDS (v_cvt_pk_bf16_f32), the weights were
// rounded when they were packed, and one v_mfma_f32_16x16x32_bf16 per gate consumes 32 k at a
// time.  Accumulators, gate functions, c and the stored h stay fp32.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
constexpr int A_LD_BF = KC + 8;      // LDS row stride of the bf16 A chunk, in elements (144 bytes)

template <int EPI, bool VEC4, bool COH>
__device__ inline void cell_tile_staged_bf16(TileSmem &sm, const Fwd &f, const Gemm &gm, const float *__restrict__ table,
                                             int count, int cg)
{
    constexpr int NG = EpiTraits<EPI>::NG;
    constexpr int SEG = EpiTraits<EPI>::SEG;
    constexpr int STEPS = KC / 32;              // 2 k-steps of 32 per chunk
    constexpr int B_UNITS = STEPS * NG * 64;    // 16-byte units of one B chunk
    constexpr int B_PER_THREAD = (B_UNITS + WG_THREADS - 1) / WG_THREADS;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nrb = (count + 15) >> 4;
    const int rb = wave;
    const bool active = rb < nrb;
    const int L = gm.L, Lp = gm.Lp;
    const int n_steps = gm.n_chunks * STEPS;
    const floatx4 *wp = reinterpret_cast<const floatx4 *>(gm.wp) + (size_t)cg * n_steps * NG * 64;
    __bf16 *a_lds[2] = {reinterpret_cast<__bf16 *>(&sm.a[0][0]), reinterpret_cast<__bf16 *>(&sm.a[1][0])};
    floatx4 *b_lds[2] = {&sm.b[0][0], &sm.b[1][0]};

    // same order of summation as the fp32 paths, in k-steps of 32: four quarters of K, each one
    // accumulator chain, added in quarter order (the packed K axis has a multiple of 4 such steps)
    floatx4 acc[NG], total[NG];
#pragma unroll
    for (int g = 0; g < NG; ++g) acc[g] = total[g] = floatx4{0.f, 0.f, 0.f, 0.f};
    const int quarter = n_steps >> 2;
    int to_boundary = quarter;

    floatx4 ra[4], rbuf[B_PER_THREAD];
    const int a_row0 = tid >> 4, a_k4 = tid & 15;
    int s0[4], s1[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        int row = a_row0 + 16 * j;
        s0[j] = row < nrb * 16 ? sm.src0[row] : -1;
        s1[j] = row < nrb * 16 ? sm.src1[row] : -1;
    }
    auto load_chunk = [&](int chunk) {
        const int k = chunk * KC + a_k4 * 4;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (j < nrb) ra[j] = load_a_granule<SEG, VEC4, COH>(table, f.zeros, L, Lp, s0[j], s1[j], k);
        const floatx4 *src = wp + (size_t)chunk * B_UNITS;
#pragma unroll
        for (int j = 0; j < B_PER_THREAD; ++j) {
            const int u = tid + WG_THREADS * j;
            rbuf[j] = src[u < B_UNITS ? u : 0];
        }
    };
    auto store_chunk = [&](int buf) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (j < nrb)
                *reinterpret_cast<bf16x4 *>(&a_lds[buf][(a_row0 + 16 * j) * A_LD_BF + a_k4 * 4]) =
                    __builtin_convertvector(ra[j], bf16x4);
#pragma unroll
        for (int j = 0; j < B_PER_THREAD; ++j) {
            const int u = tid + WG_THREADS * j;
            if (u < B_UNITS) b_lds[buf][u] = rbuf[j];
        }
    };

    load_chunk(0);
    store_chunk(0);
    __syncthreads();
    for (int chunk = 0; chunk < gm.n_chunks; ++chunk) {
        const int buf = chunk & 1;
        const bool more = chunk + 1 < gm.n_chunks;
        if (more) load_chunk(chunk + 1);
        __builtin_amdgcn_sched_barrier(0);
        if (active) {
            const __bf16 *arow = &a_lds[buf][(rb * 16 + (lane & 15)) * A_LD_BF + (lane >> 4) * 8];
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
                if (to_boundary == 0) {
#pragma unroll
                    for (int g = 0; g < NG; ++g) {
                        total[g] += acc[g];
                        acc[g] = floatx4{0.f, 0.f, 0.f, 0.f};
                    }
                    to_boundary = quarter;
                }
                --to_boundary;
                const bf16x8 av = *reinterpret_cast<const bf16x8 *>(arow + s * 32);
#pragma unroll
                for (int g = 0; g < NG; ++g) {
                    const bf16x8 bv = *reinterpret_cast<const bf16x8 *>(&b_lds[buf][(s * NG + g) * 64 + lane]);
                    acc[g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bv, acc[g], 0, 0, 0);
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        if (more) store_chunk(buf ^ 1);
        __syncthreads();
    }
    if (active) {
#pragma unroll
        for (int g = 0; g < NG; ++g) total[g] += acc[g];
        tile_epilogue<EPI, COH, NG>(sm, f, gm, total, rb, count, cg, lane);
    }
}

// The tile.  All WG_THREADS threads of the workgroup call it together; sm.node/src0/src1 hold
// the rows (see tile_set_rows) and a __syncthreads() has been passed since they were written.
//   table : source rows of the gather (embedding table, or h)
//   count : rows in use (1..TILE_ROWS);  cg : column group
template <bool VEC4, bool COH>
__device__ inline void rntn_tile_any(TileSmem &sm, const Fwd &f, const Gemm &gm, int count, int cg);   // cell_rntn.hpp

template <int EPI, bool VEC4, bool COH, bool BF16 = false>
__device__ inline void cell_tile(TileSmem &sm, const Fwd &f, const Gemm &gm, const float *__restrict__ table,
                                 int count, int cg)
{
    if constexpr (EPI == EPI_RNTN_INNER) rntn_tile_any<VEC4, COH>(sm, f, gm, count, cg);
    else if constexpr (BF16) cell_tile_staged_bf16<EPI, VEC4, COH>(sm, f, gm, table, count, cg);
    else if (count <= 32) cell_tile_direct<EPI, VEC4, COH>(sm, f, gm, table, count, cg);
    else cell_tile_staged<EPI, VEC4, COH>(sm, f, gm, table, count, cg);
    __syncthreads();   // the row tables and the LDS buffers may be rewritten after this call
}

}  // namespace tl
