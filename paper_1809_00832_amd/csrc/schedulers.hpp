// The three ways internal nodes reach the fused cell (enum tl_scheduler), plus the leaf kernel.
#pragma once

#include "cell_tile.hpp"

namespace tl {

__device__ inline void backoff() { __builtin_amdgcn_s_sleep(4); }

// ---------------------------------------------------------------------------------------
// Static tiles: `total` nodes from `list`, cut into tiles of `rows_per_tile`; block b works on
// tile b / n_cg, column group b % n_cg.  Used for the leaves (all ready at once: Section 6.2
// notes that the (N+1)/2 leaves of a tree are mutually independent) and by the host-driven
// level scheduler, one launch per height.
template <int EPI, bool VEC4>
__global__ __launch_bounds__(WG_THREADS) void k_tiles_static(Fwd f, const int32_t *__restrict__ list, int total,
                                                             int rows_per_tile)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    TileSmem &sm = *reinterpret_cast<TileSmem *>(smem_raw);
    if (f.ctl->status != 0) return;
    const int tile = blockIdx.x / f.n_cg, cg = blockIdx.x % f.n_cg;
    const int start = tile * rows_per_tile;
    const int count = min(rows_per_tile, total - start);
    if (count <= 0) return;
    const int tid = threadIdx.x;
    tile_set_rows<EPI>(sm, f, tid, tid < count ? list[start + tid] : -1);
    __syncthreads();
    const Gemm &gm = EPI == EPI_LSTM_LEAF ? f.leaf : f.inner;
    const float *table = EPI == EPI_LSTM_LEAF ? f.emb : f.h;
    cell_tile<EPI, VEC4>(sm, f, gm, table, count, cg);
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
// Grid-wide barrier for a grid whose workgroups are all resident.  Returns false if the wait
// was abandoned (spin budget exhausted somewhere); every workgroup then leaves the kernel.
__device__ inline bool grid_barrier(TileSmem &sm, const Fwd &f, unsigned &epoch)
{
    Ctl *ctl = f.ctl;
    __threadfence();
    __syncthreads();
    epoch += 1;
    if (threadIdx.x == 0) {
        const unsigned target = epoch * gridDim.x;
        add_acq_rel(&ctl->bar_count, 1u);
        int ok = 1;
        int spins = 0;
        while (ld_relaxed(&ctl->bar_count) < target) {
            if (ld_relaxed(&ctl->abort)) { ok = 0; break; }
            if (++spins > f.spin_limit) {
                st_relaxed(&ctl->abort, 1);
                latch_error(ctl, TL_ESTALL);
                ok = 0;
                break;
            }
            backoff();
        }
        fence_acquire();
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
__global__ __launch_bounds__(WG_THREADS) void k_levels_persistent(Fwd f)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    TileSmem &sm = *reinterpret_cast<TileSmem *>(smem_raw);
    if (f.ctl->status != 0) return;
    const int n_levels = f.ctl->n_levels;
    const int tid = threadIdx.x;
    unsigned epoch = 0;
    for (int lvl = 1; lvl < n_levels; ++lvl) {
        const int lo = f.level_off[lvl], rows = f.level_off[lvl + 1] - lo;
        const int m = tile_rows_for((unsigned)rows, (unsigned)f.cap_tiles);
        const int n_tiles = (rows + m - 1) / m;
        const int items = n_tiles * f.n_cg;
        for (int item = blockIdx.x; item < items; item += gridDim.x) {
            const int tile = item / f.n_cg, cg = item % f.n_cg;
            const int start = tile * m;
            const int count = min(m, rows - start);
            tile_set_rows<EPI>(sm, f, tid, tid < count ? f.level_nodes[lo + start + tid] : -1);
            __syncthreads();
            cell_tile<EPI, VEC4>(sm, f, f.inner, f.h, count, cg);
        }
        if (lvl + 1 < n_levels && !grid_barrier(sm, f, epoch)) return;
    }
}

// ---------------------------------------------------------------------------------------
// Ready-counter scheduler (Section 4.1): the device form of "enqueue an operation once all of
// its inputs are resolved".  State, all in device memory:
//   pending[n]   internal children of n that have not finished
//   q_nodes[]    append-only ready queue (q_tail = reserved entries)
//   formed       (entries consumed, tiles formed) packed in 64 bits, advanced by one CAS
//   tile_desc[t] where tile t sits in the queue and how many rows it has
//   part_next[p] next (tile, column group) item of column-group partition p
//   tile_done[t] column groups of tile t that have finished
// A workgroup repeatedly (1) claims an item of a formed tile, preferring the column-group
// partition of its own L2 domain, else (2) forms a new tile from unconsumed queue entries, else
// (3) leaves if every entry has been consumed and every item claimed, else waits.  Every wait is
// bounded by spin_limit and by the abort flag, so the grid always drains.
template <int EPI, bool VEC4>
__global__ __launch_bounds__(WG_THREADS) void k_ready_persistent(Fwd f)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    TileSmem &sm = *reinterpret_cast<TileSmem *>(smem_raw);
    Ctl *ctl = f.ctl;
    if (ctl->status != 0) return;
    const int tid = threadIdx.x;
    const int n_cg = f.n_cg;
    const int n_parts = n_cg < N_XCD ? n_cg : N_XCD;
    const int my_part = (blockIdx.x % N_XCD) % n_parts;
    const unsigned n_int = (unsigned)f.n_int;

    for (;;) {
        // ---- scheduling step, thread 0 ------------------------------------------------
        if (tid == 0) {
            int tile = -1, cg = 0;
            int spins = 0;
            unsigned long long last_w = ~0ull;
            unsigned last_done = ~0u;
            for (;;) {
                unsigned long long w = ld_relaxed(&ctl->formed);
                const unsigned head = (unsigned)w, n_tiles = (unsigned)(w >> 32);
                bool got = false;
                for (int pp = 0; pp < n_parts && !got; ++pp) {
                    const int p = (my_part + pp) % n_parts;
                    const int c0 = part_start(p, n_cg, n_parts);
                    const unsigned cgs = (unsigned)(part_start(p + 1, n_cg, n_parts) - c0);
                    unsigned i = ld_relaxed(&ctl->part_next[p]);
                    while (i / cgs < n_tiles) {
                        if (cas_acq_rel(&ctl->part_next[p], &i, i + 1u)) {
                            tile = (int)(i / cgs);
                            cg = c0 + (int)(i % cgs);
                            got = true;
                            break;
                        }
                    }
                }
                if (got) break;
                const unsigned tail = min(ld_relaxed(&ctl->q_tail), n_int);
                const unsigned done = ld_relaxed(&ctl->tiles_done);
                if (tail > head) {
                    const unsigned in_flight = n_tiles - min(done, n_tiles);
                    const unsigned room = (unsigned)f.cap_tiles > in_flight ? (unsigned)f.cap_tiles - in_flight : 0u;
                    const int m = tile_rows_for(tail - head, room);
                    if (m > 0) {
                        const unsigned long long nw = ((unsigned long long)(n_tiles + 1u) << 32) | (head + (unsigned)m);
                        if (cas_acq_rel(&ctl->formed, &w, nw))
                            st_release(&f.tile_desc[n_tiles],
                                       (1ull << 63) | ((unsigned long long)m << 32) | (unsigned long long)head);
                        spins = 0;
                        continue;
                    }
                } else if (head >= n_int) {
                    break;   // every ready entry consumed, every item claimed: done
                }
                if (ld_relaxed(&ctl->abort)) break;
                if (w != last_w || done != last_done) { last_w = w; last_done = done; spins = 0; }
                if (++spins > f.spin_limit) {
                    st_relaxed(&ctl->abort, 1);
                    latch_error(ctl, TL_ESTALL);
                    break;
                }
                backoff();
            }
            unsigned long long desc = 0;
            if (tile >= 0) {   // the former publishes the descriptor right after its CAS
                int spins2 = 0;
                while (((desc = ld_relaxed(&f.tile_desc[tile])) >> 63) == 0) {
                    if (++spins2 > f.spin_limit) { st_relaxed(&ctl->abort, 1); latch_error(ctl, TL_ESTALL); tile = -1; break; }
                    backoff();
                }
            }
            sm.cmd[0] = tile;
            sm.cmd[1] = cg;
            sm.cmd[2] = (int)(unsigned)desc;                 // start in the queue
            sm.cmd[3] = (int)((desc >> 32) & 0x7fffffffu);   // rows
            sm.cmd[4] = 1;                                   // rows all present
        }
        __syncthreads();
        const int tile = sm.cmd[0], cg = sm.cmd[1], start = sm.cmd[2], count = sm.cmd[3];
        if (tile < 0) return;

        // ---- rows of the tile: queue entries (wait for reserved slots to be written) ----
        {
            int node = -1;
            if (tid < count) {
                unsigned v;
                int spins = 0;
                while ((v = ld_relaxed(&f.q_nodes[start + tid])) == 0u) {
                    if (++spins > f.spin_limit) { sm.cmd[4] = 0; break; }
                    backoff();
                }
                node = (int)v - 1;
            }
            fence_acquire();   // children's h/c rows were released before the entry was pushed
            tile_set_rows<EPI>(sm, f, tid, node);
        }
        __syncthreads();
        if (sm.cmd[4] == 0) {
            if (tid == 0) { st_relaxed(&ctl->abort, 1); latch_error(ctl, TL_ESTALL); }
            return;
        }

        cell_tile<EPI, VEC4>(sm, f, f.inner, f.h, count, cg);

        // ---- completion: last column group of the tile resolves the parents' counters ----
        __threadfence();   // release this thread's h/c stores
        __syncthreads();
        if (tid == 0) sm.cmd[5] = (add_acq_rel(&f.tile_done[tile], 1u) == (unsigned)n_cg - 1u);
        __syncthreads();
        if (sm.cmd[5]) {
            if (tid < count) {
                const int p = f.parent[sm.node[tid]];
                if (p >= 0 && add_acq_rel(&f.pending[p], -1) == 1) {
                    const unsigned slot = add_relaxed(&ctl->q_tail, 1u);
                    if (slot < n_int) st_release(&f.q_nodes[slot], (unsigned)p + 1u);
                }
            }
            __syncthreads();
            if (tid == 0) add_relaxed(&ctl->tiles_done, 1u);
        }
        __syncthreads();
    }
}

}  // namespace tl
