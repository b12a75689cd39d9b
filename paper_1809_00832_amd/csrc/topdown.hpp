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
    // data-flow form: sets of workgroups that expand, workgroups that decide, rows of h / c that the reset kernel marks
    // as not written yet (0: the form with frontiers and grid barriers runs)
    int n_slots, n_dec, marked_rows;
};

constexpr int TD_DECIDE = 16;     // nodes per workgroup and decision step (4 per wave)

constexpr int TD_UNDECIDED = -2;  // data-flow form: left[n] of a row whose decision has not been taken, parent[n] of a row nobody has reserved

__global__ void k_td_reset(TopDown a)
{
    const int stride = gridDim.x * blockDim.x;
    const int first = blockIdx.x * blockDim.x + threadIdx.x;
    for (int i = first; i < (int)(sizeof(Ctl) / 4); i += stride) ((unsigned int *)a.f.ctl)[i] = 0;
    for (int i = first; i < a.n_trees; i += stride) {
        a.parent[i] = -1;
        a.depth[i] = 0;
    }
    if (a.marked_rows == 0) return;
    // data-flow form: no row has been decided, no row beyond the roots reserved; the rows that children will be written to
    // show the pattern that no cell stores (cell_ws.hpp), the first marked_rows of them from here, later ones from whoever
    // reserves them
    for (int i = first; i < a.max_nodes; i += stride) {
        a.left[i] = TD_UNDECIDED;
        if (i >= a.n_trees) {
            a.parent[i] = TD_UNDECIDED;
            a.depth[i] = TD_UNDECIDED;
        }
    }
    const int H4 = a.f.H / 4;                                    // (this form needs H % 4 == 0 and 16-byte aligned rows)
    const long long lo = (long long)a.n_trees * H4, hi = (long long)a.marked_rows * H4;
    const floatx4 mark = {__uint_as_float(FLOW_SENTINEL), __uint_as_float(FLOW_SENTINEL), __uint_as_float(FLOW_SENTINEL),
                          __uint_as_float(FLOW_SENTINEL)};
    for (long long i = lo + first; i < hi; i += stride) {
        reinterpret_cast<floatx4 *>(a.f.h)[i] = mark;
        reinterpret_cast<floatx4 *>(a.f.c)[i] = mark;
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

// ---- data-flow form ---------------------------------------------------------------------------
// The same trees without frontiers and without a barrier: a child is expanded as soon as its own parent has been
// decided, whatever the rest of its depth is doing, so a deep tree is not held back by the wide ones beside it and a
// depth costs a chain of memory round trips instead of two grid barriers.
//
// The row arrays are still the queue (a row is reserved by one atomic and never moves), cut into blocks of 16 rows.
//   deciders   (n_dec workgroups; block b belongs to decider b mod n_dec) wait until the rows of their next block that
//              have been reserved are complete - every element of the h row differs from the pattern that the reset
//              kernel left there, the validity carried by the data itself as in the forward pass (cell_ws.hpp) -
//              score them, reserve the rows of the children (one atomic per block and visit), and publish left[n]:
//              the row of the left child, or -1.  A block that is only partly reserved is visited again.
//   expanders  (n_slots sets of 2 n_cg workgroups, each tied to one side and one column group, with that slice of the
//              step's matrix in registers; block b belongs to set b mod n_slots) walk the rows of their blocks in order
//              and compute their 16 hidden units of the child on their side for every n that has children: tiles of
//              up to 64 decided parents on the weight-stationary cell.  When the next rows in line are reserved but
//              not decided, a workgroup does not wait for the decision: it takes up to 16 of them as a tile, waits
//              for their h rows as a decider does, and computes what their children would be while the decider
//              scores them; the decision is needed only where the results are stored (or dropped).  The step from a
//              row to its children is then one chain of row arrival, contraction and gates, with the decision beside it.
// Nothing waits on a barrier across workgroups.  A workgroup takes its rows strictly in order, and a tile that waits for
// rows holds no row in front of them, so whatever a workgroup waits for is the result of work on rows with smaller
// numbers (a child's row number is larger than its parent's) by workgroups that are themselves held up only by still
// smaller ones: the waits cannot form a cycle.  One word
// counts the rows reserved and the rows whose decision is published: when the two agree nothing is left to do and
// nothing can be reserved any more, and everybody leaves.  Every wait is bounded by the spin budget and the abort flag.
// Each node's state, score and decision are the same bits as in the other form and in every run (same cell, same
// order of summation); which rows a node's children get depends on timing.
// Rows at and after marked_rows do not show the pattern yet when they are reserved: whoever reserves them writes it
// and waits for those stores before it publishes parent[row], and a decider takes a row for complete only when it has
// seen its parent and depth entries (which the reset kernel has set to "none yet" for all rows but the roots').
template <typename Smem>
__device__ inline void td_decider(Smem &sm, const TopDown &a, int dd)
{
    const Fwd &f = a.f;
    Ctl *ctl = f.ctl;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int H = f.H, B = a.n_trees;
    const int last_row = B + 2 * ((a.max_nodes - B) / 2);       // rows that whole pairs can fill
    int b = dd, lo = 16 * dd;                                   // the block, and its first row that is not decided yet
    int spins = 0, it = 0, rows = B;
    for (;; ++it) {
        int *cmd = &sm.cmd[(it & 1) * 4];
        if (tid == 0) {
            const unsigned long long da = ld_dev(&ctl->td_rows.v);
            const unsigned ab = ld_dev(&ctl->abort.v);
            const unsigned reserved = (unsigned)da, room = (unsigned)(last_row - B);
            const int r = B + (int)(reserved < room ? reserved : room);
            cmd[0] = r;
            cmd[1] = ((int)(da >> 32) == r || ab != 0u) ? 1 : 0;
        }
        __syncthreads();
        rows = cmd[0];
        const bool over = cmd[1] != 0;
        const int hi = rows < 16 * b + 16 ? rows : 16 * b + 16;
        if (hi <= lo) {
            if (over) break;
            if (++spins > f.spin_limit) {
                if (tid == 0) flow_give_up(f);
                break;
            }
            backoff();
            continue;
        }
        spins = 0;
        // ---- the wave's four rows: wait until they are complete, score them ---------------------
        // (Rows of the block that are reserved while the wave waits join the visit: a block whose rows are reserved by
        // several others within a microsecond is then decided in one visit, not in one per reservation.)
        bool valid[4];
        const float *hr[4];
        int n4[4];
        int hi_w = hi;                                          // this wave's view of the end of the visit
        float part[4];
        int dep[4];
        bool gave_up = false;
        for (int tries = 0;; ++tries) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                n4[j] = lo + wave * 4 + j;
                valid[j] = n4[j] < hi_w;
                if (!valid[j]) n4[j] = 0;
                hr[j] = f.h + (size_t)n4[j] * H;
            }
            unsigned m[4] = {0u, 0u, 0u, 0u};
            int par[4];
            const unsigned long long da = ld_dev(&ctl->td_rows.v);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                part[j] = 0.f;
                par[j] = -1;
                dep[j] = 0;
                if (valid[j]) {                                 // (the same for all lanes of the wave)
                    par[j] = ld_dev(&a.parent[n4[j]]);
                    dep[j] = ld_dev(&a.depth[n4[j]]);
                }
            }
            for (int k = lane * 4; k < H; k += 256) {
                floatx4 x[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    x[j] = floatx4{0.f, 0.f, 0.f, 0.f};
                    if (valid[j]) x[j] = ld_f4<true>(hr[j] + k);
                }
                const floatx4 wv = *reinterpret_cast<const floatx4 *>(a.w_stop + k);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    m[j] = flow_fold<float>(m[j], x[j]);
                    part[j] = __builtin_fmaf(x[j].x, wv.x, part[j]);
                    part[j] = __builtin_fmaf(x[j].y, wv.y, part[j]);
                    part[j] = __builtin_fmaf(x[j].z, wv.z, part[j]);
                    part[j] = __builtin_fmaf(x[j].w, wv.w, part[j]);
                }
            }
            bool waiting = false;                               // (the roots are the caller's and complete)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                waiting = waiting || (valid[j] && n4[j] >= B && (m[j] == FLOW_SENTINEL || par[j] == TD_UNDECIDED || dep[j] == TD_UNDECIDED));
            if (__ballot(waiting) == 0ull) break;
            if (tries > f.spin_limit || ((tries & 63) == 63 && ld_dev(&ctl->abort.v) != 0u)) {
                gave_up = true;
                break;
            }
            {
                const unsigned reserved = (unsigned)da, room = (unsigned)(last_row - B);
                const int r = B + (int)(reserved < room ? reserved : room);
                const int h2 = r < 16 * b + 16 ? r : 16 * b + 16;
                if (h2 > hi_w) hi_w = h2;
            }
            backoff();
        }
        if (gave_up && lane == 0) {
            flow_give_up(f);
            sm.cmd[7] = 1;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float p = part[j];
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) p += __shfl_xor(p, o);
            const float score = p + a.b_stop;
            if (lane == 0) {
                sm.src0[wave * 4 + j] = (valid[j] && score > 0.f && dep[j] < a.max_depth) ? 1 : 0;
                sm.src1[wave * 4 + j] = dep[j];
                sm.node[wave * 4 + j] = valid[j] ? 1 : 0;
                if (valid[j] && !gave_up) a.score[n4[j]] = score;
            }
        }
        __syncthreads();
        if (sm.cmd[7] != 0) break;                              // a wait was abandoned: everybody leaves
        // the visit: the rows from lo on that every wave concerned has waited for
        const unsigned long long seen = __ballot(lane < 16 && sm.node[lane & 15] != 0);
        const int hi_v = lo + (seen == 0xFFFFull ? 16 : __builtin_ctzll(~seen));
        // ---- rows for the children, links, publication -------------------------------------------
        if (tid < 64) {
            const int n = lo + tid;
            const bool in_block = tid < 16 && n < hi_v;
            const bool want = in_block && sm.src0[tid & 15] != 0;
            const int d = sm.src1[tid & 15];
            const unsigned long long mask = __ballot(want);
            const int k = __popcll(mask);
            int base = 0;
            if (k > 0) {
                if (tid == 0) base = B + (int)(unsigned)add_dev(&ctl->td_rows.v, (unsigned long long)(2 * k));
                base = __shfl(base, 0);
            }
            const int l = base + 2 * __popcll(mask & ((1ull << tid) - 1ull));
            const bool ok = want && l + 2 <= a.max_nodes;
            const unsigned long long got = __ballot(ok);
            // reserved rows that the reset kernel has not marked: mark them now, and wait until that has happened
            const int m_lo = base > a.marked_rows ? base : a.marked_rows;
            const int m_hi = base + 2 * k < last_row ? base + 2 * k : last_row;
            if (k > 0 && m_lo < m_hi) {
                const int H2 = H / 2;
                for (long long i = (long long)m_lo * H2 + tid; i < (long long)m_hi * H2; i += 64) {
                    st_dev(reinterpret_cast<unsigned long long *>(f.h) + i, ~0ull);
                    st_dev(reinterpret_cast<unsigned long long *>(f.c) + i, ~0ull);
                }
                wait_mem();
            }
            if (ok) {
                st_dev(&a.depth[l], d + 1);
                st_dev(&a.depth[l + 1], d + 1);
                st_dev(&a.parent[l], n);
                st_dev(&a.parent[l + 1], n);
            }
            if (in_block) {
                a.right[n] = ok ? l + 1 : -1;
                st_dev(&a.left[n], ok ? l : -1);                // what the expanders wait for
            }
            if (got != 0ull) {
                int dmax = ok ? d + 1 : 0;
#pragma unroll
                for (int o = 8; o >= 1; o >>= 1) dmax = max(dmax, __shfl_xor(dmax, o));
                if (tid == 0) __hip_atomic_fetch_max(&ctl->td_depth.v, (unsigned)dmax, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            if (tid == 0) {
                const unsigned lost = (unsigned)__popcll(mask & ~got);
                if (lost) add_dev(&ctl->truncated.v, lost);
            }
            // the decisions count as published once everything above has been acknowledged
            wait_mem();
            if (tid == 0) add_dev(&ctl->td_rows.v, (unsigned long long)(hi_v - lo) << 32);
        }
        lo = hi_v;
        if (lo == 16 * b + 16) {
            b += a.n_dec;
            lo = 16 * b;
        }
    }
    if (dd == 0 && tid == 0) {
        a.counts[0] = rows;
        a.counts[1] = (int)ld_dev(&ctl->truncated.v);
        a.counts[2] = (int)ld_dev(&ctl->td_depth.v) + 1;        // depths 0 .. deepest
        a.counts[3] = 0;
    }
}

// What the cell asks while it evaluates rows whose decision is not known yet (cell_ws.hpp, WS_ROW_PENDING): left[parent]
// is requested when a block's rows have arrived and looked at when the block's rows are finished, one block later.
struct TdPendingHook {
    const int32_t *left;
    const int *src0;              // the tile's parents (LDS)
    int side, lane, wave;
    int ahead[2];
    __device__ inline void operator()(int rb)
    {
        if (rb < 0) return;
        const int erow = rb * 16 + (lane >> 4) * 4 + wave;      // the row this lane finishes
        const int l = ld_dev(&left[src0[erow & (WS_TABLE_ROWS - 1)]]);
        if (rb & 1) ahead[1] = l; else ahead[0] = l;
    }
    static constexpr int undecided = TD_UNDECIDED;
    __device__ inline int ahead_of(int erow) const { return ((erow >> 4) & 1) ? ahead[1] : ahead[0]; }
    __device__ inline int ask(int parent) const { return ld_dev(&left[parent]); }
};

constexpr int TD_AHEAD_ROWS = 16;     // places of the window that a tile of undecided rows may span

template <int SPW>
__global__ __launch_bounds__(WG_THREADS, SPW <= 8 ? 2 : 1) void k_td_flow(TopDown a)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    using Smem = WsSmemT<SPW>;
    Smem &sm = *reinterpret_cast<Smem *>(smem_raw);
    const Fwd &f = a.f;
    Ctl *ctl = f.ctl;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int B = a.n_trees;
    const int last_row = B + 2 * ((a.max_nodes - B) / 2);
    const int combos = 2 * f.n_cg;
    if (tid < 8) sm.cmd[tid] = 0;
    __syncthreads();
    if ((int)blockIdx.x >= a.n_slots * combos) {
        td_decider(sm, a, (int)blockIdx.x - a.n_slots * combos);
        return;
    }
    const int my_sd = ((int)blockIdx.x % combos) / f.n_cg, my_cg = ((int)blockIdx.x % combos) % f.n_cg;
    const int slot = (int)blockIdx.x / combos;
    WsWeights<EpiTraits<EPI_TD_CHILD>::NG, SPW> w;
    ws_load(w, a.side[my_sd], my_cg, wave, lane);
    sm.node[tid] = -1;                                          // (WS_TABLE_ROWS == WG_THREADS)
    sm.src0[tid] = 0;
    sm.src1[tid] = 0;
    // This set's sequence of rows: place j is row j % 16 of the set's block j / 16.  A window of 64 places starts at
    // `cursor`; `done` marks the places in it that need nothing more from this workgroup.
    int cursor = 0;
    unsigned long long done = 0ull;
    int spins = 0;
    bool seen_over = false;
    for (int it = 0;; ++it) {
        int *cmd = &sm.roots[(it & 1) * 8];
        __syncthreads();                                        // the row tables are free; the other half of cmd has been read
        if (tid < 64) {
            const int j = cursor + tid;
            const long long row = ((long long)(j >> 4) * a.n_slots + slot) * 16 + (j & 15);
            const bool open = ((done >> tid) & 1ull) == 0ull;
            int v = TD_UNDECIDED, dp = TD_UNDECIDED, par = TD_UNDECIDED;
            if (open && row < last_row) {
                v = ld_dev(&a.left[row]);
                dp = ld_dev(&a.depth[row]);
                par = ld_dev(&a.parent[row]);
            }
            // Decided rows first, wherever they are in the window (they are complete: such a tile waits for nothing).  Only
            // when there are none: the first row that is still open, if it is reserved (its depth and parent are there) and
            // sure to show the pattern until it is written, and the rows like it behind it, undecided - except at the
            // depth limit, where no row has children whatever its score.  A tile of undecided rows waits for its rows, so
            // everything in front of it must have been dealt with: it starts at the first open place.
            // (These reads are not one snapshot: a row may read as undecided and its child, a moment later, as reserved.  A
            // tile that held both would wait for what it has to produce itself, so no row follows its parent into one.)
            const bool decided = open && v != TD_UNDECIDED;
            const unsigned long long m_decided = __ballot(decided);
            unsigned long long keep = __ballot(decided && v >= 0), dealt = m_decided;
            if (keep == 0ull) {
                const unsigned long long still = ~(done | m_decided);
                const int p0 = still == 0ull ? 0 : __builtin_ctzll(still);
                const int row0 = __shfl((int)(row < last_row ? row : last_row), p0);
                const bool ahead = open && !decided && dp != TD_UNDECIDED && par != TD_UNDECIDED && par < row0 &&
                                   row < a.marked_rows;
                const unsigned long long stop = __ballot(open && !decided && !ahead);
                const int lim = stop == 0ull ? 64 : __builtin_ctzll(stop);
                const bool taken = ahead && tid < lim && tid < p0 + TD_AHEAD_ROWS;
                keep = __ballot(taken && dp < a.max_depth);
                dealt |= __ballot(taken);
            }
            const int n_keep = __popcll(keep);
            if ((keep >> tid) & 1ull) {
                const int idx = __popcll(keep & ((1ull << tid) - 1ull));
                sm.src0[idx] = (int)row;
                sm.node[idx] = v >= 0 ? v + my_sd : WS_ROW_PENDING;
            }
            // the rest of the last block of 16 asks for the first row again (whatever row a table entry names is requested)
            if (n_keep > 0) {
                const int first = __shfl((int)row, __builtin_ctzll(keep));
                if (tid >= n_keep && tid < ((n_keep + 15) & ~15)) sm.src0[tid] = first;
            }
            if (tid == 0) {
                const unsigned long long now = done | dealt;
                const int shift = now == ~0ull ? 64 : __builtin_ctzll(~now);
                const unsigned long long next = shift == 64 ? 0ull : now >> shift;
                cmd[0] = dealt != 0ull ? 1 : 0;
                cmd[1] = n_keep;
                cmd[3] = shift;
                cmd[4] = (int)(unsigned)next;
                cmd[5] = (int)(unsigned)(next >> 32);
                if (dealt == 0ull) {
                    const unsigned long long da = ld_dev(&ctl->td_rows.v);
                    const unsigned ab = ld_dev(&ctl->abort.v);
                    const unsigned reserved = (unsigned)da, room = (unsigned)(last_row - B);
                    const int r = B + (int)(reserved < room ? reserved : room);
                    cmd[2] = ((int)(da >> 32) == r || ab != 0u) ? 1 : 0;
                }
            }
        }
        __syncthreads();
        const int count = cmd[1];
        if (cmd[0] == 0) {
            // nothing new.  When every reserved row has been decided and published, one more look at the rows (which is then
            // certain to see every decision) ends the walk.
            if (seen_over) break;
            seen_over = cmd[2] != 0;
            if (!seen_over) {
                if (++spins > f.spin_limit) {
                    if (tid == 0) flow_give_up(f);
                    break;
                }
                backoff();
            }
            continue;
        }
        spins = 0;
        seen_over = false;
        cursor += cmd[3];
        done = (unsigned long long)(unsigned)cmd[4] | (unsigned long long)(unsigned)cmd[5] << 32;
        if (count > 0) {
            TdPendingHook hook{a.left, sm.src0, my_sd, lane, wave, {TD_UNDECIDED, TD_UNDECIDED}};
            ws_tile<EPI_TD_CHILD, true, SPW, false, true>(sm, f, a.side[my_sd], f.h, a.max_nodes, count, my_cg, w, hook);
            if (sm.cmd[7] != 0) break;                          // a wait was abandoned: everybody leaves
        }
    }
}

}  // namespace tl
