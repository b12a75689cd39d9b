// Weight-stationary form of the fused cell, for persistent kernels.
//
// Every internal node of every tree multiplies the same matrix U (Figure 2: one LSTM cell
// re-used at every recursive call).  A persistent workgroup therefore owns one column group of
// HU hidden units for the whole forward and keeps its slice of U in registers: the K axis is
// split between the four waves, and each wave holds SPW k-steps x NG gates of MFMA B operands
// (up to 16 x 5 x 4 = 320 VGPRs of the 512 a wave may use when one wave per SIMD is resident).
// Per block of 16 rows a wave then loads only its part of the gathered A rows, runs SPW x NG x 4
// MFMAs on register operands, and the four partial sums meet in LDS, from where each wave
// finishes four of the sixteen rows (gate functions, c update, h/c stores).  The weights are
// read from memory once per forward instead of once per tile, which removes the L2 -> CU traffic
// that bounds small tiles, and a 16-row block costs SPW x NG x 4 MFMAs of latency however few
// rows are ready.
//
// The summation order of a node is fixed (each wave walks its K range in order, the four partial
// sums are added in wave order), so a node's result does not depend on which rows happened to
// share its tile: results are bit-identical from run to run and between the two persistent
// schedulers.
#pragma once

#include <cstddef>

#include "cell_tile.hpp"

namespace tl {

constexpr int WS_RED_FLOATS = 4 * MAX_GATES * 4 * 64;
static_assert(2 * WS_RED_FLOATS * sizeof(float) <= sizeof(TileSmem::a) + sizeof(TileSmem::b), "reduction buffers must fit the staging area");
static_assert(offsetof(TileSmem, b) == sizeof(TileSmem::a), "staging area must be contiguous");

template <int NG, int SPW> struct WsWeights {
    floatx4 b[SPW][NG];
    float bias[NG];
};
template <int NG> struct WsWeights<NG, 0> {};   // streaming kernels keep nothing

// Loads this wave's slice of the packed weights: k-steps [wave*SPW, (wave+1)*SPW) of column
// group cg.  The packed matrix has exactly 4*SPW k-steps (the host pads it).
template <int NG, int SPW>
__device__ inline void ws_load(WsWeights<NG, SPW> &w, const Gemm &gm, int cg, int wave, int lane)
{
    const floatx4 *wp = reinterpret_cast<const floatx4 *>(gm.wp) + ((size_t)cg * 4 * SPW + (size_t)wave * SPW) * NG * 64 + lane;
#pragma unroll
    for (int s = 0; s < SPW; ++s)
#pragma unroll
        for (int g = 0; g < NG; ++g) w.b[s][g] = wp[(size_t)(s * NG + g) * 64];
#pragma unroll
    for (int g = 0; g < NG; ++g) w.bias[g] = gm.bp[(cg * NG + g) * HU + (lane & 15)];
}

// Evaluates the `count` rows in sm.node/src0/src1 for column group cg.  All four waves call it
// together; a __syncthreads() has been passed since the row tables were written.
template <int EPI, bool COH, int SPW>
__device__ inline void ws_tile(TileSmem &sm, const Fwd &f, const Gemm &gm, const float *__restrict__ table, int count,
                               int cg, const WsWeights<EpiTraits<EPI>::NG, SPW> &w)
{
    constexpr int NG = EpiTraits<EPI>::NG;
    constexpr int SEG = EpiTraits<EPI>::SEG;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nrb = (count + 15) >> 4;
    const int L = gm.L, Lp = gm.Lp, H = f.H;
    const int hu = cg * HU + (lane & 15);
    const bool hu_ok = hu < H;
    const int k0 = STEP_K * wave * SPW + (lane >> 4) * 4;
    // A operands of block rb+1 are requested while block rb is being multiplied: as soon as the
    // MFMAs of a k-step have consumed a[s], the same registers are re-loaded for the next block
    // (the register file has no room for a second copy next to the weights).
    floatx4 a[SPW];
    {
        const int row = lane & 15;
        const int s0 = sm.src0[row], s1 = sm.src1[row];     // -1 beyond count
#pragma unroll
        for (int s = 0; s < SPW; ++s)
            a[s] = load_a_granule<SEG, true, COH>(table, f.zeros, L, Lp, s0, s1, k0 + s * STEP_K);
    }
    for (int rb = 0; rb < nrb; ++rb) {
        // [wave][g][v][lane], 20 KB, alternating between two buffers laid over the (unused) A/B staging area
        float *red = reinterpret_cast<float *>(&sm) + (rb & 1) * WS_RED_FLOATS;
        // rows of the next block (none: gather zeros)
        const int nrow = (rb + 1) * 16 + (lane & 15);
        const bool has_next = rb + 1 < nrb;
        const int ns0 = has_next ? sm.src0[nrow & (TILE_ROWS - 1)] : -1;
        const int ns1 = has_next ? sm.src1[nrow & (TILE_ROWS - 1)] : -1;
        // the row this lane finishes after the reduction, and its c operands (requested early)
        const int erow = rb * 16 + (lane >> 4) * 4 + wave;
        const int enode = erow < count ? sm.node[erow] : -1;
        const bool ev = enode >= 0 && hu_ok;
        float cl = 0.f, cr = 0.f;
        if (EPI == EPI_LSTM_INNER) {
            cl = ld_f<COH>(ev ? f.c + (size_t)sm.src0[erow] * H + hu : f.zeros);
            cr = ld_f<COH>(ev ? f.c + (size_t)sm.src1[erow] * H + hu : f.zeros);
        }
        floatx4 acc[NG];
#pragma unroll
        for (int g = 0; g < NG; ++g) acc[g] = floatx4{0.f, 0.f, 0.f, 0.f};
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s = 0; s < SPW; ++s) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int g = 0; g < NG; ++g)
                    acc[g] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[s][i], w.b[s][g][i], acc[g], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            a[s] = load_a_granule<SEG, true, COH>(table, f.zeros, L, Lp, ns0, ns1, k0 + s * STEP_K);
            __builtin_amdgcn_sched_barrier(0);
        }
        // the four K-range partial sums meet in LDS; wave w finishes accumulator row w
#pragma unroll
        for (int g = 0; g < NG; ++g)
#pragma unroll
            for (int v = 0; v < 4; ++v) red[((wave * NG + g) * 4 + v) * 64 + lane] = acc[g][v];
        __syncthreads();
        float gate[NG];
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            float sum = red[((0 * NG + g) * 4 + wave) * 64 + lane];
            sum += red[((1 * NG + g) * 4 + wave) * 64 + lane];
            sum += red[((2 * NG + g) * 4 + wave) * 64 + lane];
            sum += red[((3 * NG + g) * 4 + wave) * 64 + lane];
            gate[g] = sum + w.bias[g];
        }
        if (ev) {
            const size_t o = (size_t)enode * H + hu;
            if constexpr (EPI == EPI_LSTM_INNER) {
                const float i = sigmoid_f(gate[0]);
                const float fl = sigmoid_f(gate[1]);
                const float fr = sigmoid_f(gate[2]);
                const float og = sigmoid_f(gate[3]);
                const float u = tanh_f(gate[NG - 1]);
                const float cc = i * u + fl * cl + fr * cr;
                st_f<COH>(f.c + o, cc);
                st_f<COH>(f.h + o, og * tanh_f(cc));
            } else if constexpr (EPI == EPI_LSTM_LEAF) {
                const float i = sigmoid_f(gate[0]);
                const float og = sigmoid_f(gate[1]);
                const float u = tanh_f(gate[NG - 1]);
                const float cc = i * u;
                st_f<COH>(f.c + o, cc);
                st_f<COH>(f.h + o, og * tanh_f(cc));
            } else {
                st_f<COH>(f.h + o, tanh_f(gate[0]));
            }
        }
        // no second barrier: the next block writes the other half of the reduction buffer, and the
        // block after that passes the next block's barrier before it writes this half again
    }
    __syncthreads();                                        // row tables and LDS may be rewritten after this call
}

}  // namespace tl
