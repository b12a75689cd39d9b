// The three ways internal nodes reach the fused cell (enum tl_scheduler), plus the leaf kernel.
#pragma once

#include "cell_tile.hpp"

namespace tl {

// ---------------------------------------------------------------------------------------
// Static tiles: `total` nodes from `list`, cut into tiles by plan_level(); block b works on
// tile b / n_cg, column group b % n_cg.  Used for the leaves (all ready at once: Section 6.2
// notes that the (N+1)/2 leaves of a tree are mutually independent) and by the host-driven
// level scheduler, one launch per height.  Kernel boundaries order producers and consumers,
// so plain cached loads and stores are used.
template <int EPI, bool VEC4>
__global__ __launch_bounds__(WG_THREADS, 2) void k_tiles_static(Fwd f, const int32_t *__restrict__ list, int total,
                                                                LevelPlan plan)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    TileSmem &sm = *reinterpret_cast<TileSmem *>(smem_raw);
    if (f.ctl->status != 0) return;
    const int tile = blockIdx.x / f.n_cg, cg = blockIdx.x % f.n_cg;
    int start, count;
    plan_tile(plan, total, tile, &start, &count);
    if (count <= 0) return;
    const int tid = threadIdx.x;
    tile_set_rows<EPI>(sm, f, tid, tid < count ? list[start + tid] : -1);
    __syncthreads();
    const Gemm &gm = EPI == EPI_LSTM_LEAF ? f.leaf : f.inner;
    const float *table = EPI == EPI_LSTM_LEAF ? f.emb : f.h;
    cell_tile<EPI, VEC4, false>(sm, f, gm, table, count, cg);
}

// Leaves of TreeRNN / RNTN: h = embedding row.
__global__ void k_leaf_copy(Fwd f)
{
    if (f.ctl->status != 0) return;
    const int i = blockIdx.x;
    if (i >= f.n_leaf) return;
    const int n = f.leaf_list[i];
    const int w = f.word[n];
    for (int j = threadIdx.x; j < f.H; j += blockDim.x) f.h[(size_t)n * f.H + j] = f.emb[(size_t)w * f.E + j];
}

// ---------------------------------------------------------------------------------------
// Grid-wide barrier for a grid whose workgroups are all resident and whose size is a multiple
// of N_XCD.  Two levels, so that no single word takes hundreds of back-to-back atomics: the
// workgroups of one L2 domain count on their own line, the last of each domain counts on a
// shared line, and the very last one raises a flag line per domain, which the others poll.
// Data visibility does not come from the barrier: callers write shared data with device-scope
// stores and call wait_mem() first.  Returns false if the wait was abandoned (spin budget
// exhausted somewhere); every workgroup then leaves the kernel.
__device__ inline bool grid_barrier(TileSmem &sm, const Fwd &f, unsigned &epoch)
{
    Ctl *ctl = f.ctl;
    wait_mem();
    __syncthreads();
    epoch += 1;
    if (threadIdx.x == 0) {
        const int x = blockIdx.x % N_XCD;
        const unsigned per = gridDim.x / N_XCD;
        if (add_dev(&ctl->bar_xcd[x].v, 1u) == per * epoch - 1u) {
            if (add_dev(&ctl->bar_all.v, 1u) == (unsigned)N_XCD * epoch - 1u)
                for (int i = 0; i < N_XCD; ++i) st_dev(&ctl->bar_flag[i].v, epoch);
        }
        int ok = 1;
        int spins = 0;
        while (ld_dev(&ctl->bar_flag[x].v) < epoch) {
            if (++spins > f.spin_limit || ((spins & 63) == 0 && ld_dev(&ctl->abort.v))) {
                st_dev(&ctl->abort.v, 1u);
                latch_error(ctl, TL_ESTALL);
                ok = 0;
                break;
            }
            backoff();
        }
        sm.cmd[0] = ok;
    }
    __syncthreads();
    const int ok = sm.cmd[0];
    __syncthreads();
    return ok != 0;
}

// Level frontiers on the device: heights 1, 2, ... with a grid barrier between them (the
// depth-wise batching of Section 6.3, without a launch or a host round trip per depth).
template <int EPI, bool VEC4>
__global__ __launch_bounds__(WG_THREADS, 2) void k_levels_persistent(Fwd f)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    TileSmem &sm = *reinterpret_cast<TileSmem *>(smem_raw);
    if (f.ctl->status != 0) return;
    const int n_levels = f.ctl->n_levels;
    const int tid = threadIdx.x;
    unsigned epoch = 0;
    for (int lvl = 1; lvl < n_levels; ++lvl) {
        const int lo = f.level_off[lvl], rows = f.level_off[lvl + 1] - lo;
        const LevelPlan plan = plan_level(rows, f.cap_tiles);
        const int items = plan.n_tiles * f.n_cg;
        for (int item = blockIdx.x; item < items; item += gridDim.x) {
            const int tile = item / f.n_cg, cg = gang_cg(item % f.n_cg, f.n_cg, f.n_cg);
            int start, count;
            plan_tile(plan, rows, tile, &start, &count);
            tile_set_rows<EPI>(sm, f, tid, tid < count ? f.level_nodes[lo + start + tid] : -1);
            __syncthreads();
            cell_tile<EPI, VEC4, true>(sm, f, f.inner, f.h, count, cg);
        }
        if (lvl + 1 < n_levels && !grid_barrier(sm, f, epoch)) return;
    }
}

// ---------------------------------------------------------------------------------------
// Ready-counter scheduler (Section 4.1): the device form of "enqueue an operation once all of
// its inputs are resolved".  State, all in device memory:
//   pending[n]   internal children of n that have not finished
//   q_nodes[]    append-only ready queue; q_tail = entries reserved, q_head = entries consumed
//   gangs[g]     mailbox of gang g
// The grid is n_gangs gangs of gang_size workgroups; member j of a gang owns column group(s)
// gang_cg(j, ..), so a gang covers all hidden units of a tile.  The leader (member 0) cuts a
// tile of ready nodes off the queue and posts it in the gang's mailbox; every member evaluates
// its columns of the tile and counts itself done; the leader then decrements the counter of each
// row's parent and pushes parents that reach zero.  Gangs run independently of each other: no
// barrier spans the grid, and a tile starts as soon as its nodes are ready and a gang is free.
// Every wait is bounded by spin_limit and by the abort flag, so the grid always drains.
template <int EPI, bool VEC4>
__global__ __launch_bounds__(WG_THREADS, 2) void k_ready_persistent(Fwd f)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    TileSmem &sm = *reinterpret_cast<TileSmem *>(smem_raw);
    Ctl *ctl = f.ctl;
    if (ctl->status != 0) return;
    const int tid = threadIdx.x;
    const int gang = blockIdx.x / f.gang_size, member = blockIdx.x % f.gang_size;
    GangBox *box = &f.gangs[gang];
    const bool leader = member == 0;
    const unsigned n_int = (unsigned)f.n_int;
    unsigned seq = 0;                      // tiles this gang has been given so far

    for (;;) {
        seq += 1;
        // ---- the leader cuts the next tile off the ready queue and posts it -------------
        if (tid == 0) {
            unsigned start = 0, rows = GANG_EXIT_ROWS;
            int spins = 0;
            if (leader) {
                unsigned last_tail = ~0u;
                for (;;) {
                    unsigned head = ld_dev(&ctl->q_head.v);
                    if (head >= n_int) break;                            // every node has been handed out
                    unsigned tail = ld_dev(&ctl->q_tail.v);
                    if (tail > n_int) tail = n_int;
                    if (tail > head) {
                        const unsigned m = (unsigned)tile_rows_for(tail - head, (unsigned)f.n_gangs);
                        if (cas_dev(&ctl->q_head.v, &head, head + m)) { start = head; rows = m; break; }
                        continue;
                    }
                    if (tail != last_tail) { last_tail = tail; spins = 0; }
                    if (++spins > f.spin_limit || ((spins & 15) == 0 && ld_dev(&ctl->abort.v))) {
                        st_dev(&ctl->abort.v, 1u);
                        latch_error(ctl, TL_ESTALL);
                        break;
                    }
                    backoff();
                }
                st_dev(&box->desc.v, ((unsigned long long)seq << 40) | ((unsigned long long)rows << 32) | start);
                if (rows != GANG_EXIT_ROWS) add_dev(&ctl->tiles.v, 1u);
            } else {
                // the leader always posts, at the latest when its own wait gives up: the larger
                // budget here is only a safety net
                unsigned long long d;
                long long polls = 0;
                while (((d = ld_dev(&box->desc.v)) >> 40) < seq) {
                    if (++polls > 64ll * f.spin_limit) { d = GANG_EXIT_ROWS << 32; break; }
                    backoff();
                }
                start = (unsigned)d;
                rows = (unsigned)(d >> 32) & 0xffu;
            }
            sm.cmd[0] = (int)rows;
            sm.cmd[1] = (int)start;
            sm.cmd[2] = 1;
        }
        __syncthreads();
        const int count = sm.cmd[0], start = sm.cmd[1];
        if (count == (int)GANG_EXIT_ROWS) return;

        // ---- rows of the tile: queue entries (a reserved slot may not be written yet) ----
        {
            int node = -1;
            if (tid < count) {
                unsigned v;
                int spins = 0;
                while ((v = ld_dev(&f.q_nodes[start + tid])) == 0u) {
                    if (++spins > f.spin_limit) { sm.cmd[2] = 0; break; }
                    backoff();
                }
                node = (int)v - 1;
            }
            tile_set_rows<EPI>(sm, f, tid, node);
        }
        __syncthreads();
        const bool rows_ok = sm.cmd[2] != 0;

        if (rows_ok)
            for (int j = member; j < f.n_cg; j += f.gang_size)
                cell_tile<EPI, VEC4, true>(sm, f, f.inner, f.h, count, gang_cg(j, f.gang_size, f.n_cg));

        // ---- completion -------------------------------------------------------------------
        wait_mem();            // this wave's h/c stores have reached memory
        __syncthreads();
        if (tid == 0) add_dev(&box->done.v, 1u);
        if (!leader) continue;

        if (tid == 0) {
            const unsigned target = seq * (unsigned)f.gang_size;
            int spins = 0, ok = rows_ok ? 1 : 0;
            while (ld_dev(&box->done.v) < target) {
                if (++spins > f.spin_limit) { ok = 0; break; }
                backoff();
            }
            if (!ok) { st_dev(&ctl->abort.v, 1u); latch_error(ctl, TL_ESTALL); }
            sm.cmd[3] = ok;
        }
        __syncthreads();
        if (sm.cmd[3] && tid < 64) {
            // first wave: one lane per row; parents that become ready are pushed with one
            // reservation on q_tail for the whole tile
            int p = -1;
            if (tid < count) {
                p = f.parent[sm.node[tid]];
                if (p >= 0 && add_dev(&f.pending[p], -1) != 1) p = -1;
            }
            const unsigned long long ready = __ballot(p >= 0);
            const int n_ready = __popcll(ready);
            unsigned base = 0;
            if (tid == 0 && n_ready > 0) base = add_dev(&ctl->q_tail.v, (unsigned)n_ready);
            base = __shfl(base, 0);
            if (p >= 0) {
                const unsigned slot = base + (unsigned)__popcll(ready & ((1ull << tid) - 1ull));
                if (slot < n_int) st_dev(&f.q_nodes[slot], (unsigned)p + 1u);
            }
        }
        __syncthreads();
    }
}

}  // namespace tl
