// RNTN cell (Section 6.1 names the model; the form used is h_k = tanh(a^T V_k a + (a W)_k + b_k)
// with a = [h_left ; h_right], V of shape d x 2d x 2d).
//
// The bilinear term is evaluated as a sequence of ordinary contractions on the MFMA units:
//     a^T V_k a = sum_q a_q * T_q[k],    T_q[k] = sum_p a_p V[k][p][q]
// so for every q the tile's rows are multiplied with the [2d x 16] slice B_q[p][k] = V[k][p][q]
// of one column group (16 outputs k), and the 16x16 result is scaled per row by a_q and added
// up in registers.  The linear term is one more such slice (B = W, scale 1).  The four waves of a
// workgroup take q = wave, wave + 4, ... for all row blocks of the tile; their partial sums meet
// in LDS and wave w finishes row block w (bias, tanh, h rows).
#pragma once

#include "cell_tile.hpp"

namespace tl {

// Packed V (+ W) of one column group: [q in 0..Kp][k-step s][lane][4] with
//   p = 16 s + 4 (lane / 16) + i on the padded K axis, k = 16 cg + lane % 16,
// q = Kp holding W[p][k].  Padded p or q positions hold zeros.
__global__ void k_pack_rntn(const float *__restrict__ v, const float *__restrict__ w, float *__restrict__ vp, int d, int Lp,
                            int Kp, int n_cg)
{
    const int n_steps = Kp / STEP_K;
    const size_t total = (size_t)n_cg * (Kp + 1) * n_steps * 256;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (size_t)gridDim.x * blockDim.x) {
        const int i = (int)(e & 3), lane = (int)((e >> 2) & 63);
        size_t r = e >> 8;
        const int s = (int)(r % n_steps);
        r /= n_steps;
        const int q = (int)(r % (Kp + 1));
        const int cg = (int)(r / (Kp + 1));
        const int p = 16 * s + 4 * (lane >> 4) + i;
        const int k = cg * HU + (lane & 15);
        const int pseg = p / Lp, poff = p - pseg * Lp;
        float val = 0.f;
        if (k < d && pseg < 2 && poff < d) {
            const int pl = pseg * d + poff;                 // logical index into a = [h_l ; h_r]
            if (q == Kp) {
                val = w[(size_t)pl * d + k];
            } else {
                const int qseg = q / Lp, qoff = q - qseg * Lp;
                if (qseg < 2 && qoff < d) val = v[((size_t)k * 2 * d + pl) * 2 * d + (qseg * d + qoff)];
            }
        }
        vp[e] = val;
    }
}

// Order of summation over q, the same however the work is spread: the slices fall into 16 classes by
// q mod 16; a class is added up in ascending q on one accumulator; part p (p = 0..3) is the sum of the classes
// p, p + 4, p + 8, p + 12 in that order; the result is ((part 0 + part 1) + part 2) + part 3, then the bias.
// A workgroup evaluates one part of a tile and column group (sm.cmd[5] = p; its four waves take one class each),
// or all four parts one after the other (sm.cmd[5] = -1).  With one part per workgroup, four workgroups share a
// tile and column group: each leaves its part in a scratch area (unit sm.cmd[6] of it), counts itself done, and
// the one that completes the count adds the parts up and writes h.  A height of a few rows thus spreads over
// four times as many workgroups, each with a quarter of the slices: with d = 64 there are only four column
// groups, and a block of 16 rows costs 129 slices x 32 MFMAs whatever the number of rows.
constexpr int RNTN_PARTS = 4;
constexpr int RNTN_PART_FLOATS = TILE_ROWS * HU;            // one part of one tile and column group in the scratch area
// Tiles that the grid works on at once when a tile and column group is shared by RNTN_PARTS workgroups: a frontier is cut
// (plan_level) so that its tiles fill one round of the grid where they can - a second round of small tiles costs a whole
// item's latency more (records, child rows, first slice, exchange, scratch area), taller tiles only their matrix instructions.
__host__ __device__ inline int rntn_cap_tiles(int cap_tiles, int rntn_units)
{
    return rntn_units > 0 && cap_tiles >= RNTN_PARTS ? cap_tiles / RNTN_PARTS : cap_tiles;
}

template <int NS, bool VEC4, bool COH>
__device__ inline void rntn_tile(TileSmem &sm, const Fwd &f, const Gemm &gm, int count, int cg)
{
    constexpr int Kp = NS * STEP_K;
    constexpr int LD = Kp + 4;                              // LDS row stride of the A tile, floats
    constexpr int RED_FLOATS = 4 * 2 * 4 * 64;              // [wave][2 row blocks x 4 values][lane]
    static_assert((TILE_ROWS * LD + RED_FLOATS) * sizeof(float) <= sizeof(TileSmem::a) + sizeof(TileSmem::b),
                  "A tile and the exchange area must fit the staging area");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nrb = (count + 15) >> 4;
    const int part = sm.cmd[5], unit = sm.cmd[6];           // written by the caller before its barrier
    float *a_lds = reinterpret_cast<float *>(&sm);
    float *red = a_lds + TILE_ROWS * LD;
    // ---- the tile's gathered rows, once, into LDS ----------------------------------------
    for (int g = tid; g < nrb * 16 * (Kp / 4); g += WG_THREADS) {
        const int row = g / (Kp / 4), k4 = g - row * (Kp / 4);
        const floatx4 v = load_a_granule<2, VEC4, COH>(f.h, f.zeros, gm.L, gm.Lp, sm.src0[row], sm.src1[row], k4 * 4);
        *reinterpret_cast<floatx4 *>(&a_lds[row * LD + k4 * 4]) = v;
    }
    __syncthreads();

    const floatx4 *vp = reinterpret_cast<const floatx4 *>(gm.wp) + (size_t)cg * (Kp + 1) * NS * 64 + lane;
    floatx4 out[4];
    floatx4 b0[NS], b1[NS];
    auto load_slice = [&](int q, floatx4 (&b)[NS]) {
        const int qq = q <= Kp ? q : Kp;                    // past the end: re-read the last slice, never used
#pragma unroll
        for (int s = 0; s < NS; ++s) b[s] = vp[(size_t)(qq * NS + s) * 64];
    };
    auto use_slice = [&](int q, const floatx4 (&b)[NS]) {
        if (q > Kp) return;
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) {
            if (rb >= nrb) continue;
            const float *arow = &a_lds[(rb * 16 + (lane & 15)) * LD + (lane >> 4) * 4];
            floatx4 t = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                const floatx4 av = *reinterpret_cast<const floatx4 *>(arow + s * STEP_K);
#pragma unroll
                for (int i = 0; i < 4; ++i) t = __builtin_amdgcn_mfma_f32_16x16x4f32(av[i], b[s][i], t, 0, 0, 0);
            }
            // scale accumulator row (4 (lane/16) + v) by that row's a_q; the linear slice is not scaled
            const float *mrow = &a_lds[(rb * 16 + (lane >> 4) * 4) * LD + (q < Kp ? q : 0)];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float m = q < Kp ? mrow[v * LD] : 1.f;
                out[rb][v] += m * t[v];
            }
        }
    };
    float mine[4] = {0.f, 0.f, 0.f, 0.f};                   // wave w: row block w, parts added up so far
    const int p_lo = part < 0 ? 0 : part, p_hi = part < 0 ? RNTN_PARTS - 1 : part;
    for (int pp = p_lo; pp <= p_hi; ++pp) {
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) out[rb] = floatx4{0.f, 0.f, 0.f, 0.f};
        const int cls = pp + RNTN_PARTS * wave;             // this wave's class of the part
        load_slice(cls, b0);
        for (int q = cls; q <= Kp; q += 32) {
            load_slice(q + 16, b1);
            __builtin_amdgcn_sched_barrier(0);
            use_slice(q, b0);
            __builtin_amdgcn_sched_barrier(0);
            load_slice(q + 32, b0);
            __builtin_amdgcn_sched_barrier(0);
            use_slice(q + 16, b1);
            __builtin_amdgcn_sched_barrier(0);
        }
        // the part: the four waves' class sums in wave order; wave w takes row block w, two row blocks per round
        float ppart[4] = {0.f, 0.f, 0.f, 0.f};
        for (int r0 = 0; r0 < nrb; r0 += 2) {
            __syncthreads();                                // the exchange area is free again
#pragma unroll
            for (int rbi = 0; rbi < 2; ++rbi)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    float x = 0.f;
#pragma unroll
                    for (int rb = 0; rb < 4; ++rb) if (rb == r0 + rbi) x = out[rb][v];
                    red[(wave * 8 + rbi * 4 + v) * 64 + lane] = x;
                }
            __syncthreads();
            if (wave >= r0 && wave < r0 + 2) {
                const int rbi = wave - r0;
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    ppart[v] = ((red[(0 * 8 + rbi * 4 + v) * 64 + lane] + red[(1 * 8 + rbi * 4 + v) * 64 + lane]) +
                                red[(2 * 8 + rbi * 4 + v) * 64 + lane]) + red[(3 * 8 + rbi * 4 + v) * 64 + lane];
            }
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) mine[v] = pp == p_lo ? ppart[v] : mine[v] + ppart[v];
    }
    const int rb = wave;
    const int hu = cg * HU + (lane & 15);
    const float bias = gm.bp[cg * HU + (lane & 15)];
    if (part < 0) {
        if (rb < nrb && hu < f.H) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = rb * 16 + (lane >> 4) * 4 + v;
                const int node = row < count ? sm.node[row] : -1;
                if (node >= 0) st_f<COH>(f.h + (size_t)node * f.H + hu, tanh_f(mine[v] + bias));
            }
        }
        return;
    }
    // ---- one part per workgroup: parts meet in the scratch area, the last one to arrive finishes ----
    float *sc = f.rntn_part + (size_t)(unit * f.n_cg + cg) * RNTN_PARTS * RNTN_PART_FLOATS;
    unsigned int *done = f.rntn_done + (size_t)unit * f.n_cg + cg;
    if (rb < nrb) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int row = rb * 16 + (lane >> 4) * 4 + v;
            st_dev(sc + part * RNTN_PART_FLOATS + row * HU + (lane & 15), mine[v]);
        }
    }
    wait_mem();
    __syncthreads();
    if (tid == 0) sm.cmd[7] = (int)add_dev(done, 1u);
    __syncthreads();
    if (sm.cmd[7] != RNTN_PARTS - 1) return;                // uniform: not the last part of this tile and column group
    if (tid == 0) st_dev(done, 0u);                         // the counter is ready for its next use
    if (rb < nrb && hu < f.H) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int row = rb * 16 + (lane >> 4) * 4 + v;
            const int node = row < count ? sm.node[row] : -1;
            const float *e = sc + row * HU + (lane & 15);
            const float sum = ((ld_dev(e) + ld_dev(e + RNTN_PART_FLOATS)) + ld_dev(e + 2 * RNTN_PART_FLOATS)) +
                              ld_dev(e + 3 * RNTN_PART_FLOATS);
            if (node >= 0) st_f<COH>(f.h + (size_t)node * f.H + hu, tanh_f(sum + bias));
        }
    }
}

// Dispatch on the padded K length (k-steps of 16): d <= 32, 64, 128.
template <bool VEC4, bool COH>
__device__ inline void rntn_tile_any(TileSmem &sm, const Fwd &f, const Gemm &gm, int count, int cg)
{
    const int ns = gm.n_chunks * (KC / STEP_K);
    if (ns == 4) rntn_tile<4, VEC4, COH>(sm, f, gm, count, cg);
    else if (ns == 8) rntn_tile<8, VEC4, COH>(sm, f, gm, count, cg);
    else rntn_tile<16, VEC4, COH>(sm, f, gm, count, cg);
}

}  // namespace tl
