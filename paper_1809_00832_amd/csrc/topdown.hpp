// Top-down generation of trees whose shape depends on computed values (Section 6.3, "Dynamically
// Structured Models"): whether a node gets children is decided from the node's own state, so
// nothing about the trees beyond their roots is known before the evaluation, and there is no
// structure pass.  One persistent kernel grows all trees of a batch breadth first:
//
//   frontier 0 = the roots (rows 0 .. n_trees-1 of h / c, given by the caller)
//   decide     every node of the frontier: score = w_stop . h + b_stop; a node with score > 0
//              below the depth limit reserves two new rows (one atomic per workgroup and 16
//              nodes) and records the links parent <-> children
//   (grid barrier, which also carries the number of rows reserved so far)
//   expand     the new rows are the next frontier; they come in (left, right) pairs, and the
//              state of a child is an LSTM step from its parent's state with the weights of its
//              side: tiles of up to 64 pairs x one side x 16 hidden units on the streaming cell
//              (gather of the parents' h rows, MFMA contraction, gates, c / h rows)
//   (grid barrier: the children's rows are complete before anybody scores them)
//
// A node's row number is its position in that breadth-first queue, so the row arrays are the
// queue and nothing is moved.  Which rows two siblings get depends on the order in which
// workgroups reach the atomic; the trees themselves do not: every contraction is summed in the
// fixed order of the streaming cell and every score in a fixed order, so each node's state and
// decision are the same bits in every run.
// The loop ends when a frontier reserves nothing (at the latest at the depth limit); every wait
// is the bounded grid barrier of schedulers.hpp.
#pragma once

#include "schedulers.hpp"

namespace tl {

struct TopDown {
    Fwd f;                        // h, c, H, n_cg, zeros, ctl, spin_limit are used
    Gemm side[2];                 // packed [H x 4H] weights and bias of the left / right edge
    const float *w_stop;
    float b_stop;
    int n_trees, max_depth, max_nodes;
    int32_t *parent, *left, *right, *depth;
    float *score;
    int32_t *counts;              // [4]: nodes, truncated, frontiers, 0
};

constexpr int TD_DECIDE = 16;     // nodes per workgroup and decision step (4 per wave)

__global__ void k_td_reset(TopDown a)
{
    const int stride = gridDim.x * blockDim.x;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < (int)(sizeof(Ctl) / 4); i += stride) ((unsigned int *)a.f.ctl)[i] = 0;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < a.n_trees; i += stride) {
        a.parent[i] = -1;
        a.depth[i] = 0;
    }
}

// SPW > 0: the expansion step runs on the weight-stationary cell (cell_ws.hpp): every workgroup is tied to one side
// and one column group for the whole call and keeps that slice of the step's matrix in registers (SPW k-steps per
// wave), instead of streaming 4 H^2 weights per side and frontier through LDS.  Needs H % 4 == 0, 16-byte aligned
// rows, at least 2 n_cg workgroups, fewer than 2^24 rows and less than 4 GiB of h (the host checks).
template <bool VEC4, int SPW = 0>
__global__ __launch_bounds__(WG_THREADS, 1) void k_td_generate(TopDown a)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    using Smem = std::conditional_t<(SPW > 0), WsSmemT<(SPW > 0 ? SPW : 1)>, TileSmem>;
    Smem &sm = *reinterpret_cast<Smem *>(smem_raw);
    const Fwd &f = a.f;
    Ctl *ctl = f.ctl;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int H = f.H, B = a.n_trees;
    const int last_row = B + 2 * ((a.max_nodes - B) / 2);       // rows that whole pairs can fill
    // weight-stationary form: this workgroup's side, column group and share of the rows
    const int combos = 2 * f.n_cg;
    const int my_sd = ((int)blockIdx.x % combos) / f.n_cg, my_cg = ((int)blockIdx.x % combos) % f.n_cg;
    const int slot = (int)blockIdx.x / combos, n_slots = (int)gridDim.x / combos;
    WsWeights<EpiTraits<EPI_TD_CHILD>::NG, SPW> w;
    if constexpr (SPW > 0) {
        if (slot < n_slots) ws_load(w, a.side[my_sd], my_cg, wave, lane);
    }
    unsigned epoch = 0;
    int begin = 0, end = B, d = 0;
    for (;; ++d) {
        // ---- decide ------------------------------------------------------------------------
        unsigned appended = 0;
        const int n_front = end - begin;
        for (int chunk = blockIdx.x; chunk * TD_DECIDE < n_front; chunk += gridDim.x) {
            const int first = begin + chunk * TD_DECIDE;
            // the wave's four nodes side by side: their rows are requested together, one round trip per 256 (64) elements
            // of H instead of one per node and piece (every lane still adds up its elements of a row in ascending order)
            const float *hr[4];
            bool valid[4];
            float part[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int n = first + wave * 4 + j;
                valid[j] = n < end;
                hr[j] = f.h + (size_t)(valid[j] ? n : 0) * H;
            }
            if (VEC4) {
                for (int k = lane * 4; k < H; k += 256) {
                    floatx4 x[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) x[j] = ld_f4<true>(hr[j] + k);
                    const floatx4 wv = *reinterpret_cast<const floatx4 *>(a.w_stop + k);
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        part[j] = __builtin_fmaf(x[j].x, wv.x, part[j]);
                        part[j] = __builtin_fmaf(x[j].y, wv.y, part[j]);
                        part[j] = __builtin_fmaf(x[j].z, wv.z, part[j]);
                        part[j] = __builtin_fmaf(x[j].w, wv.w, part[j]);
                    }
                }
            } else {
                for (int k = lane; k < H; k += 64) {
                    float x[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) x[j] = ld_f<true>(hr[j] + k);
                    const float wv = a.w_stop[k];
#pragma unroll
                    for (int j = 0; j < 4; ++j) part[j] = __builtin_fmaf(x[j], wv, part[j]);
                }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int n = first + wave * 4 + j;
                float p = part[j];
#pragma unroll
                for (int o = 32; o >= 1; o >>= 1) p += __shfl_xor(p, o);
                const float score = p + a.b_stop;
                if (lane == 0) {
                    sm.src0[wave * 4 + j] = (valid[j] && score > 0.f && d < a.max_depth) ? 1 : 0;
                    if (valid[j]) a.score[n] = score;
                }
            }
            __syncthreads();
            if (tid < 64) {
                const int n = first + tid;
                const bool valid = tid < TD_DECIDE && n < end;
                const bool want = tid < TD_DECIDE && sm.src0[tid] != 0;
                const unsigned long long mask = __ballot(want);
                int base = 0;
                if (mask != 0ull) {
                    if (tid == 0) base = B + (int)add_dev(&ctl->q_tail.v, 2u * (unsigned)__popcll(mask));
                    base = __shfl(base, 0);
                }
                const int l = base + 2 * __popcll(mask & ((1ull << tid) - 1ull));
                const bool ok = want && l + 2 <= a.max_nodes;
                const unsigned long long got = __ballot(ok);
                if (valid) {
                    a.left[n] = ok ? l : -1;
                    a.right[n] = ok ? l + 1 : -1;
                }
                if (ok) {
                    st_dev(&a.parent[l], n);              // read by other workgroups after the barrier
                    st_dev(&a.parent[l + 1], n);
                    a.depth[l] = d + 1;
                    a.depth[l + 1] = d + 1;
                }
                if (tid == 0) {
                    appended += 2u * (unsigned)__popcll(got);
                    const unsigned lost = (unsigned)__popcll(mask & ~got);
                    if (lost) add_dev(&ctl->truncated.v, lost);
                }
            }
            __syncthreads();
        }
        unsigned len = 0;
        if (!grid_barrier(sm, f, epoch, appended, (unsigned)B, &len)) return;
        const int new_end = (int)len < last_row ? (int)len : last_row;
        const int pairs = (new_end - end) / 2;
        if (pairs <= 0) break;
        // ---- expand --------------------------------------------------------------------------
        if constexpr (SPW > 0) {
            if (slot < n_slots) {
                // every slot takes a contiguous share of the pairs, a multiple of 16 rows, in pieces of the row tables' size
                const int share = ((pairs + n_slots - 1) / n_slots + 15) & ~15;
                const int lo = slot * share, hi = pairs < lo + share ? pairs : lo + share;
                for (int piece = lo; piece < hi; piece += WS_TABLE_ROWS) {
                    const int count = hi - piece < WS_TABLE_ROWS ? hi - piece : WS_TABLE_ROWS;
                    {
                        int child = -1, par = 0;
                        if (tid < count) {
                            child = end + 2 * (piece + tid) + my_sd;
                            par = ld_dev(&a.parent[child]);
                        }
                        sm.node[tid] = child;
                        sm.src0[tid] = par > 0 ? par : 0;       // (rows that do not exist read row 0; nothing of them is stored)
                        sm.src1[tid] = 0;
                    }
                    __syncthreads();
                    ws_tile<EPI_TD_CHILD, true, SPW>(sm, f, a.side[my_sd], f.h, a.max_nodes, count, my_cg, w);
                }
            }
            unsigned unused_ws = 0;
            if (!grid_barrier(sm, f, epoch, 0u, (unsigned)B, &unused_ws)) return;
            begin = end;
            end = new_end;
            continue;
        }
        const int n_cg = f.n_cg;
        int conc = (int)gridDim.x / (2 * n_cg);               // tiles the grid works on at once
        if (conc < 1) conc = 1;
        int rpt = ((pairs + conc - 1) / conc + 15) & ~15;       // rows per tile: spread over the grid, in blocks of 16
        if (rpt > TILE_ROWS) rpt = TILE_ROWS;
        const int n_tiles = (pairs + rpt - 1) / rpt;
        for (int item = blockIdx.x; item < n_tiles * 2 * n_cg; item += gridDim.x) {
            const int tile = item / (2 * n_cg), rem = item - tile * 2 * n_cg;
            const int sd = rem / n_cg, cg = rem - sd * n_cg;
            const int start = tile * rpt;
            const int count = pairs - start < rpt ? pairs - start : rpt;
            if (tid < TILE_ROWS) {
                int child = -1, par = -1;
                if (tid < count) {
                    child = end + 2 * (start + tid) + sd;
                    par = ld_dev(&a.parent[child]);
                }
                sm.node[tid] = child;
                sm.src0[tid] = par;
                sm.src1[tid] = -1;
            }
            __syncthreads();
            if constexpr (SPW == 0) cell_tile<EPI_TD_CHILD, VEC4, true>(sm, f, a.side[sd], f.h, count, cg);
        }
        unsigned unused = 0;
        if (!grid_barrier(sm, f, epoch, 0u, (unsigned)B, &unused)) return;
        begin = end;
        end = new_end;
    }
    if (blockIdx.x == 0 && tid == 0) {
        a.counts[0] = end;
        a.counts[1] = (int)ld_dev(&ctl->truncated.v);
        a.counts[2] = d + 1;                                     // frontiers walked (depths 0 .. d)
        a.counts[3] = 0;
    }
}

}  // namespace tl
