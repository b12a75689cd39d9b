// The three ways internal nodes reach the fused cell (enum tl_scheduler), plus the leaf kernel.
#pragma once

#include <type_traits>

#include "structure.hpp"
#include "cell_ws.hpp"
#include "cell_rntn.hpp"

namespace tl {

// ---------------------------------------------------------------------------------------
// Static tiles: `total` nodes from `list`, cut into tiles by plan_level(); block b works on
// tile b / n_cg, column group b % n_cg.  Used for the leaves (all ready at once: Section 6.2
// notes that the (N+1)/2 leaves of a tree are mutually independent) and by the host-driven
// level scheduler, one launch per height.  Kernel boundaries order producers and consumers,
// so plain cached loads and stores are used.
template <int EPI, bool VEC4, bool BF16>
__global__ __launch_bounds__(WG_THREADS, 2) void k_tiles_static(Fwd f, const int32_t *__restrict__ list, int total,
                                                                LevelPlan plan)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    TileSmem &sm = *reinterpret_cast<TileSmem *>(smem_raw);
    if (batch_rejected(f)) return;
    // RNTN cell, frontier of few tiles: RNTN_PARTS workgroups per tile and column group, one part of the sums each
    const int parts = (EPI == EPI_RNTN_INNER && plan.n_tiles <= f.rntn_units) ? RNTN_PARTS : 1;
    const int tile = blockIdx.x / (f.n_cg * parts), rem = blockIdx.x % (f.n_cg * parts);
    const int cg = rem % f.n_cg, part = rem / f.n_cg;
    int start, count;
    plan_tile(plan, total, tile, &start, &count);
    if (count <= 0) return;
    const int tid = threadIdx.x;
    tile_set_rows<EPI>(sm, f, tid, tid < count ? list[start + tid] : -1, f.pos0 + start + tid);
    if (tid == 0) {
        sm.cmd[3] = f.pos0 + start;                         // list position of row 0 (backward kernels)
        sm.cmd[5] = parts > 1 ? part : -1;
        sm.cmd[6] = tile;                                   // unit of the scratch area
    }
    __syncthreads();
    constexpr bool LEAF_ROWS = EPI == EPI_LSTM_LEAF || EPI == EPI_BWD_LEAF_GATES;
    constexpr bool GRAD_ROWS = epi_is_operand_gradient(EPI);
    const Gemm &gm = LEAF_ROWS ? f.leaf : (GRAD_ROWS ? f.bwd : f.inner);
    const float *table = LEAF_ROWS ? f.emb : (GRAD_ROWS ? f.dg : f.h);
    cell_tile<EPI, VEC4, false, BF16>(sm, f, gm, table, count, cg);
}

// Leaves with the weight-stationary cell (fp32): the leaf matrix is small (E x 3H), so a column
// group's slice takes few registers, two workgroups fit on a CU, and every workgroup keeps its
// slice while it walks a contiguous share of the leaf list in pieces of up to WS_TABLE_ROWS rows.
template <int SPW>
__global__ __launch_bounds__(WG_THREADS, 2) void k_leaf_ws(Fwd f)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    WsSmemT<SPW> &sm = *reinterpret_cast<WsSmemT<SPW> *>(smem_raw);
    if (batch_rejected(f)) return;
    const int tid = threadIdx.x;
    // (data-flow scheduler: the stores that mark the internal nodes' rows go out first and complete beside the cells)
    if (f.flow == 2) flow_fill(f, (size_t)blockIdx.x * 4 + (tid >> 6), (size_t)gridDim.x * 4);
    const int cg = gang_cg(blockIdx.x % f.n_cg, f.n_cg, f.n_cg);
    const int slot = blockIdx.x / f.n_cg, n_slots = gridDim.x / f.n_cg;
    WsWeights<EpiTraits<EPI_LSTM_LEAF>::NG, SPW> w;
    ws_load(w, f.leaf, cg, tid >> 6, tid & 63);
    const int share = ((f.n_leaf + n_slots - 1) / n_slots + 15) & ~15;
    const int lo = slot * share, hi = min(f.n_leaf, lo + share);
    for (int piece = lo; piece < hi; piece += WS_TABLE_ROWS) {
        const int count = min(hi - piece, WS_TABLE_ROWS);
        const int node = tid < count ? f.leaf_list[piece + tid] : -1;
        sm.node[tid] = node;
        sm.src0[tid] = node >= 0 ? f.word[node] : 0;
        sm.src1[tid] = 0;
        __syncthreads();
        ws_tile<EPI_LSTM_LEAF, false, SPW>(sm, f, f.leaf, f.emb, f.vocab, count, cg, w);
    }
}

// The same with bf16 operands: rows come from a bf16 copy of the embedding table (rows padded with
// zeros to a multiple of 8 elements).
// (Four workgroups per CU: the matrix instructions of a block of leaves take 0.1 us, the block's phases - rows, park,
// barrier, gates - 1.2 us.)
template <int S> using LeafSmemBf = WsSmemBfT<S, EpiTraits<EPI_LSTM_LEAF>::NG, false>;
template <int S>
__global__ __launch_bounds__(WG_THREADS, 4) void k_leaf_ws_bf(Fwd f)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    LeafSmemBf<S> &sm = *reinterpret_cast<LeafSmemBf<S> *>(smem_raw);
    if (batch_rejected(f)) return;
    const int tid = threadIdx.x;
    if (f.flow == 2) flow_fill(f, (size_t)blockIdx.x * 4 + (tid >> 6), (size_t)gridDim.x * 4);
    const int cg = gang_cg(blockIdx.x % f.n_cg, f.n_cg, f.n_cg);
    const int slot = blockIdx.x / f.n_cg, n_slots = gridDim.x / f.n_cg;
    WsWeightsBf<EpiTraits<EPI_LSTM_LEAF>::NG, S> w;
    ws_load(w, sm, f.leaf, cg, tid >> 6, tid & 63);
    const int share = ((f.n_leaf + n_slots - 1) / n_slots + 15) & ~15;
    const int lo = slot * share, hi = min(f.n_leaf, lo + share);
    for (int piece = lo; piece < hi; piece += WS_TABLE_ROWS) {
        const int count = min(hi - piece, WS_TABLE_ROWS);
        const int node = tid < count ? f.leaf_list[piece + tid] : -1;
        sm.node[tid] = node;
        sm.src0[tid] = node >= 0 ? f.word[node] : 0;
        __syncthreads();
        ws_tile<EPI_LSTM_LEAF, false, S>(sm, f, f.leaf, f.embb, f.vocab, f.es, count, cg, w);
    }
}

// Leaves of TreeRNN / RNTN: h = embedding row.
__global__ void k_leaf_copy(Fwd f)
{
    if (batch_rejected(f)) return;
    const int i = blockIdx.x;
    if (i >= f.n_leaf) return;
    const int n = f.leaf_list[i];
    const int w = f.word[n];
    for (int j = threadIdx.x; j < f.H; j += blockDim.x) {
        const float x = f.emb[(size_t)w * f.E + j];
        f.h[(size_t)n * f.H + j] = x;
        if (f.hb) f.hb[(size_t)n * f.hs + j] = bf16_bits(x);
    }
}

// ---------------------------------------------------------------------------------------
// Grid-wide barrier for a grid whose workgroups are all resident; it also tells every workgroup
// how long the ready queue has become (`queue_len`), the same figure for all.
//
// Up to FLAT_BARRIER_MAX workgroups: every workgroup adds itself to the word of its L2 domain (no
// single word takes hundreds of back-to-back atomics, and nobody waits for the result of its own
// arrival), then one lane per domain polls the domains' words until all of them show the arrivals
// of this barrier.  The same atomic carries the number of ready-queue records the workgroup has
// appended since the last barrier, in the high half of the word, so that the poll which sees
// everybody arrived also sees the length of the queue, without another round trip.
//
// Larger grids (two workgroups per CU): that many pollers on the words the arrivals are counted
// on delay the arrivals themselves (accesses to one address are served one after the other), so
// a second level is used: the last arrival of a domain counts the domain on a shared word, the
// very last one reads the queue length and raises one flag per domain, and a workgroup polls only
// the flag of its own domain.
//
// Data visibility does not come from the barrier: callers write shared data with device-scope
// stores, and wait_mem() here lets them complete first.  Returns false if the wait was abandoned
// (spin budget exhausted somewhere); every workgroup then leaves the kernel.
constexpr unsigned FLAT_BARRIER_MAX = 256;

template <typename Smem>
__device__ inline bool grid_barrier(Smem &sm, const Fwd &f, unsigned &epoch, unsigned appended, unsigned n_seed,
                                    unsigned *queue_len)
{
    Ctl *ctl = f.ctl;
    wait_mem();
    __syncthreads();
    epoch += 1;
    if (threadIdx.x < 64) {
        const unsigned lane = threadIdx.x;
        const unsigned n_dom = gridDim.x < (unsigned)N_XCD ? gridDim.x : (unsigned)N_XCD;   // domains that hold workgroups
        const unsigned x = blockIdx.x % N_XCD;
        int ok = 1, spins = 0;
        unsigned len = 0;
        auto give_up = [&]() {
            st_dev(&ctl->abort.v, 1u);
            latch_error(ctl, TL_ESTALL);
            ok = 0;
        };
        auto aborted = [&]() { return __ballot(lane == 0 && ld_dev(&ctl->abort.v) != 0u) != 0ull; };
        if (gridDim.x <= FLAT_BARRIER_MAX) {
            if (lane == 0) add_dev(&ctl->bar_xcd[x].v, 1ull | (unsigned long long)appended << 32);
            const unsigned per = (gridDim.x - lane + N_XCD - 1u) / N_XCD;                     // workgroups of domain `lane`
            const unsigned long long all_domains = (1ull << n_dom) - 1ull;
            unsigned long long v = 0;
            for (;;) {
                if (lane < n_dom) v = ld_dev(&ctl->bar_xcd[lane].v);      // one lane per domain, nobody else loads
                if (__ballot(lane < n_dom && (unsigned)v >= per * epoch) == all_domains) break;
                if (++spins > f.spin_limit || ((spins & 63) == 0 && aborted())) { give_up(); break; }
                backoff();
            }
            len = lane < n_dom ? (unsigned)(v >> 32) : 0u;
            for (int o = N_XCD / 2; o >= 1; o >>= 1) len += __shfl_xor(len, o);
            len += n_seed;
        } else {
            unsigned long long flag = 0;
            if (lane == 0) {
                const unsigned per = (gridDim.x - x + N_XCD - 1u) / N_XCD;                    // workgroups of this domain
                if ((unsigned)add_dev(&ctl->bar_xcd[x].v, 1ull) == per * epoch - 1u) {
                    if (add_dev(&ctl->bar_all.v, 1u) == n_dom * epoch - 1u) {
                        // everybody has arrived, so every append made before the barrier is counted
                        const unsigned long long v = pack2(epoch, ld_dev(&ctl->q_tail.v));
                        for (unsigned i = 0; i < n_dom; ++i) st_dev(&ctl->bar_flag[i].v, v);
                    }
                }
            }
            for (;;) {
                if (lane == 0) flag = ld_dev(&ctl->bar_flag[x].v);
                if (__ballot(lane == 0 && (unsigned)flag >= epoch) != 0ull) break;
                if (++spins > f.spin_limit || ((spins & 63) == 0 && aborted())) { give_up(); break; }
                backoff();
            }
            len = (unsigned)(flag >> 32);
        }
        if (lane == 0) {
            sm.cmd[0] = ok;
            sm.cmd[1] = (int)len;
        }
    }
    __syncthreads();
    const int ok = sm.cmd[0];
    *queue_len = (unsigned)sm.cmd[1];
    __syncthreads();
    return ok != 0;
}

// Level frontiers on the device: the depth-wise batching of Section 6.3 without a launch, a host
// round trip or a separate pass over the trees per depth.  The frontiers are built as the
// evaluation goes, with the ready counters of Section 4.1: frontier 1 is the set of internal nodes
// over two leaves (the structure pass left them at the head of the ready queue); while frontier k
// is evaluated, one wave per tile decrements the counter of each row's parent and appends the
// parents that reach zero to the queue; after a grid barrier those appended entries are frontier
// k + 1.  A parent's counter may reach zero before its children's rows are stored: nobody reads
// the appended entries before the barrier, which every workgroup passes only after its stores
// have completed.  The loop ends when a frontier is empty; if nodes are left then (a cycle), the
// batch is reported as malformed.
// SPW > 0 selects the weight-stationary cell (cell_ws.hpp, SPW k-steps per wave in registers,
// every workgroup tied to one column group; one workgroup per CU in fp32, two with bf16
// operands); SPW == 0 the streaming cell.
template <int SPW, bool BF16>
using PersistentSmem = std::conditional_t<(SPW > 0), std::conditional_t<BF16, WsSmemBfT<(SPW > 0 ? SPW : 1)>, WsSmemT<(SPW > 0 ? SPW : 1)>>, TileSmem>;
template <int NG, int SPW, bool BF16>
using PersistentWeights = std::conditional_t<(SPW > 0 && BF16), WsWeightsBf<NG, SPW>, WsWeights<NG, SPW>>;

// Parents of 64 rows of the row table (from row0 on), first half: wave 0, one lane per row,
// sends the decrements.  The returned values are needed only in frontier_push(), after the rows
// have been computed.
struct ParentTicket {
    int p, old, left, right;      // parent of this lane's row (-1: none), its counter before the decrement, its children
};
template <typename Smem> __device__ inline ParentTicket frontier_decrement(const Smem &sm, const Fwd &f, int count, int row0)
{
    ParentTicket t{-1, 0, -1, -1};
    const int lane = row0 + (int)threadIdx.x;
    if (lane < count) {
        const int node = sm.node[lane];
        if (node >= 0) t.p = f.parent[node];
    }
    if (t.p >= 0) {
        t.old = add_dev(&f.pending[t.p], -1);
        t.left = f.left[t.p];
        t.right = f.right[t.p];
    }
    return t;
}
// Second half: parents whose counter reached zero are appended with one reservation per tile.
__device__ inline unsigned frontier_push(const Fwd &f, const ParentTicket &t)
{
    const int lane = threadIdx.x;
    const bool ready = t.p >= 0 && t.old == 1;
    const unsigned long long mask = __ballot(ready);
    const int n_ready = __popcll(mask);
    if (n_ready == 0) return 0u;
    unsigned base = 0;
    if (lane == 0) base = add_dev(&f.ctl->q_tail.v, (unsigned)n_ready);
    base = __shfl(base, 0);
    if (ready) {
        const unsigned slot = base + (unsigned)__popcll(mask & ((1ull << lane) - 1ull));
        if (slot < (unsigned)f.n_int) qrec_store<true>(&f.q_rec[slot], t.p, t.left, t.right);
    }
    return (unsigned)n_ready;
}

template <int EPI, bool VEC4, int SPW, bool BF16 = false>
__global__ __launch_bounds__(WG_THREADS, (SPW > 0 && !BF16) ? 1 : 2) void k_levels_persistent(Fwd f)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    using Smem = PersistentSmem<SPW, BF16>;
    Smem &sm = *reinterpret_cast<Smem *>(smem_raw);
    Ctl *ctl = f.ctl;
    if (batch_rejected(f) || internal_kernel_skipped(f)) return;
    const int tid = threadIdx.x;
    // A slot is a set of workgroups that covers all column groups; the workgroups of a slot gather the same child rows.
    // (Putting every slot on one L2 domain, so that its rows cross the fabric once instead of once per domain that
    // holds some of its column groups, was measured and is not done: no faster on the H=512 batch, whose fabric
    // reads are far from any limit, and up to 7 % slower on narrow batches.)
    const int n_slots = gridDim.x / f.n_cg;
    const int member = blockIdx.x % f.n_cg, slot = blockIdx.x / f.n_cg;
    const int my_cg = gang_cg(member, f.n_cg, f.n_cg);
    PersistentWeights<EpiTraits<EPI>::NG, SPW, BF16> w;
    if constexpr (SPW > 0 && BF16) ws_load(w, sm, f.inner, my_cg, tid >> 6, tid & 63);
    else if constexpr (SPW > 0) ws_load(w, f.inner, my_cg, tid >> 6, tid & 63);
    unsigned epoch = 0;
    const unsigned n_seed = (unsigned)ctl->n_seed;
    unsigned begin = 0, end = n_seed;
    unsigned appended = 0;                        // records this workgroup has appended since the last barrier (wave 0 counts)
    const unsigned n_int = (unsigned)f.n_int;
    if (end > n_int) end = n_int;
    int frontiers = 0;
    while (end > begin) {
        int rows = (int)(end - begin);
        if constexpr (SPW > 0) {
            // The slots advance together, 16 rows each per step, so a frontier costs ceil(rows / (16 n_slots)) steps of
            // the whole machine, and a few rows beyond a multiple cost a whole step.  Such a remainder of a large
            // frontier (at most 32 rows beyond one or more full steps) is left in the queue: it becomes the head of
            // the next frontier, whose last step usually has room (on the H=512 evaluation batch: 57 steps
            // instead of 60).  Every row of the queue is still taken exactly once.  Only where a step is long (fp32,
            // 16 k-steps per wave: about 6 us): a node left behind may cost its tree one more frontier, which is
            // worth a step there and not where steps are short.
            constexpr bool LEAVE_REMAINDER = !BF16 && SPW >= 16;
            const int step_rows = 16 * n_slots, rem = rows % step_rows;
            if (LEAVE_REMAINDER && rows > step_rows && rem > 0 && rem <= 32) rows -= rem;
            // Every slot (a set of workgroups that covers all column groups) takes one contiguous share of
            // the frontier, a multiple of 16 rows, and walks it in pieces of up to WS_TABLE_ROWS rows: one
            // fill of the row tables and one start of the row-request pipeline per piece.  The parents of
            // rows [64 j, 64 j + 64) of a piece are looked after by wave 0 of member (frontier + slot + j) %
            // n_cg, so that this duty rotates; the decrements are sent while the piece's first rows are on their
            // way and their results are used after the piece.
            const int share = ((rows + n_slots - 1) / n_slots + 15) & ~15;
            const int lo = slot * share, hi = min(rows, lo + share);
            for (int piece = lo; piece < hi; piece += WS_TABLE_ROWS) {
                const int count = min(hi - piece, WS_TABLE_ROWS);
                {
                    int node = -1, s0 = -1, s1 = -1;
                    if (tid < count && !qrec_load(&f.q_rec[begin + piece + tid], &node, &s0, &s1)) {
                        node = s0 = s1 = -1;
                        latch_error(ctl, TL_ESTALL);          // a record inside the frontier that is not there: never skipped silently
                    }
                    sm.node[tid] = node;
                    sm.src0[tid] = max(s0, 0);
                    sm.src1[tid] = max(s1, 0);
                }
                __syncthreads();
                // this wave's 64-row group of parents, if any.  The decrements of the last one are sent from inside the
                // cell, once its first row requests are out: looking up the parents is a memory round trip of its own,
                // which then runs beside that of the rows instead of in front of it.  (Earlier groups - fewer column
                // groups than 64-row groups - are dealt with at once.)
                int j_mine = -1;
                if (tid < 64) {
                    for (int j = 0; j * 64 < count; ++j) {
                        if ((frontiers + slot + j) % f.n_cg != member) continue;
                        if (j_mine >= 0) appended += frontier_push(f, frontier_decrement(sm, f, count, j_mine * 64));
                        j_mine = j;
                    }
                }
                ParentTicket ticket{-1, 0, -1, -1};
                auto hook = [&](int where) {            // -1: the first row requests are out
                    if (where == -1 && j_mine >= 0) ticket = frontier_decrement(sm, f, count, j_mine * 64);
                };
                if constexpr (BF16) ws_tile<EPI, true, SPW>(sm, f, f.inner, f.hb, f.n_nodes, f.hs, count, my_cg, w, hook);
                else ws_tile<EPI, true, SPW, !VEC4>(sm, f, f.inner, f.h, f.n_nodes, count, my_cg, w, hook);
                if (j_mine >= 0) appended += frontier_push(f, ticket);
            }
        } else {
            const LevelPlan plan = plan_level(rows, EPI == EPI_RNTN_INNER ? rntn_cap_tiles(f.cap_tiles, f.rntn_units) : f.cap_tiles);
            // tile T of a frontier: its rows' parents are looked after by the workgroup that computes
            // column group T % n_cg of it
            const int parts = (EPI == EPI_RNTN_INNER && plan.n_tiles <= f.rntn_units) ? RNTN_PARTS : 1;
            const int items = plan.n_tiles * f.n_cg * parts;
            for (int item = blockIdx.x; item < items; item += gridDim.x) {
                const int tile = item / (f.n_cg * parts), rem = item % (f.n_cg * parts);
                const int cg_index = rem % f.n_cg, part = rem / f.n_cg;
                int start, count;
                plan_tile(plan, rows, tile, &start, &count);
                if (tid == 0) {
                    sm.cmd[5] = parts > 1 ? part : -1;
                    sm.cmd[6] = tile;                       // unit of the scratch area
                }
                if (tid < TILE_ROWS) {
                    int node = -1, s0 = -1, s1 = -1;
                    if (tid < count && !qrec_load(&f.q_rec[begin + start + tid], &node, &s0, &s1)) {
                        node = s0 = s1 = -1;
                        latch_error(ctl, TL_ESTALL);
                    }
                    sm.node[tid] = node;
                    sm.src0[tid] = s0;
                    sm.src1[tid] = s1;
                }
                __syncthreads();
                const bool keeper = cg_index == tile % f.n_cg && part == 0 && tid < 64;
                ParentTicket ticket{-1, 0, -1, -1};
                if (keeper) ticket = frontier_decrement(sm, f, count, 0);
                cell_tile<EPI, VEC4, true, BF16>(sm, f, f.inner, f.h, count, gang_cg(cg_index, f.n_cg, f.n_cg));
                if (keeper) appended += frontier_push(f, ticket);
            }
        }
        frontiers += 1;
        begin += (unsigned)rows;
        if (begin >= n_int) break;                // every internal node has been handed out
        unsigned queue_len = 0;
        if (!grid_barrier(sm, f, epoch, appended, n_seed, &queue_len)) return;
        appended = 0;
        end = queue_len < n_int ? queue_len : n_int;
    }
    if (blockIdx.x == 0 && tid == 0) {
        ctl->n_levels = frontiers + 1;            // the leaves and the frontiers (= the heights, unless rows were left over)
        if (end < n_int) latch_error(ctl, TL_ESTRUCT);   // nodes that never became ready: not a forest
    }
}

// ---------------------------------------------------------------------------------------
// Data-flow scheduler: the ready counters of Section 4.1 with nothing shared between the workers.
//
// The trees of the batch are dealt to the slots in contiguous ranges of about equal node count (a
// slot is a set of workgroups that covers all column groups, see above), and every workgroup of a
// slot evaluates, for its own column group, all internal nodes of the slot's trees.  It keeps the
// whole scheduling state to itself: a counter of handed-out children per node and an append-only
// list of the nodes that have become ready (both in a part of the workspace that no other
// workgroup touches).  It starts with the nodes over two leaves, found by scanning the slot's node
// range; handing out a node counts it at its parent, and a parent whose internal children have all
// been handed out goes to the end of the list, so the list is filled ahead of the evaluation and a
// node always comes after its children.  Nothing is exchanged about the schedule: no shared
// queue, no records, no grid barrier, no mailbox.
//
// What a node does need from the other workgroups of its slot are the children's rows, of which
// every workgroup produces 16 hidden units.  Their completion is read off the rows themselves
// (cell_ws.hpp, "validity carried by the data"): the rows of all internal nodes are filled with a
// pattern no cell produces before the kernel starts, a consumer requests a child row as early as
// it likes and repeats the request while a piece of it still shows the pattern.  A dependent step
// then costs the producer's store, its way through the memory system and the consumer's load -
// about one round trip - where the level scheduler pays the stores' acknowledgement, a grid
// barrier of two round trips, the records of the next frontier and then the rows.  Slots do not
// wait for each other at all.
//
// All workgroups of a slot build the same list and take it in the same pieces, and a piece depends on
// earlier pieces only, so the workgroup that is furthest behind never waits for anything unfinished:
// the waits always end (and each is bounded by the spin budget and the abort flag).
// Nodes that never become ready (a cycle) are never listed; the workgroup then finishes with fewer
// nodes than its slot has and reports the batch as malformed.
// The state of root n goes to the per-tree outputs: one lane copies the 16 hidden units of column group cg.  An
// internal root's units have been stored by the lane's own workgroup (and those stores have arrived), a leaf's by
// the leaf kernel, so ordinary loads see them.  The tree is one of [t_lo, t_hi).
__device__ inline void flow_copy_root(const Fwd &f, int n, int cg, int t_lo, int t_hi)
{
    int lo = t_lo, hi = t_hi - 1;                             // largest t with tree_off[t] <= n
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (f.tree_off[mid] <= n) lo = mid; else hi = mid - 1;
    }
    const int t = lo, H = f.H, u0 = cg * HU;
    const size_t src = (size_t)n * H + u0, dst = (size_t)t * H + u0;
    const bool quad = (H & 3) == 0 && u0 + HU <= H &&
                      (((uintptr_t)f.h | (uintptr_t)f.c | (uintptr_t)f.h_root | (uintptr_t)f.c_root) & 15) == 0;
    if (quad) {
        floatx4 vh[4], vc[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            vh[j] = *reinterpret_cast<const floatx4 *>(f.h + src + 4 * j);
            if (f.c) vc[j] = *reinterpret_cast<const floatx4 *>(f.c + src + 4 * j);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (f.h_root) *reinterpret_cast<floatx4 *>(f.h_root + dst + 4 * j) = vh[j];
            if (f.c_root && f.c) *reinterpret_cast<floatx4 *>(f.c_root + dst + 4 * j) = vc[j];
        }
    } else {
        for (int j = 0; j < HU && u0 + j < H; ++j) {
            if (f.h_root) f.h_root[dst + j] = f.h[src + j];
            if (f.c_root && f.c) f.c_root[dst + j] = f.c[src + j];
        }
    }
    if (cg == 0) {                                            // once per root
        if (f.root_out) f.root_out[t] = n;
        if (atomicCAS(&f.root_ws[t], -1, n) != -1) latch_error(f.ctl, TL_ESTRUCT);      // a second root of the same tree
    }
}

struct FlowTicket {
    int p, key, left, right, up;  // parent that became ready with this lane's row (-1: none), its place among the group's parents, its children and its own parent
};
// One lane per row of rows [row0, row0 + 64) of the row table: counts the row at its parent.  All workgroups of a
// slot must build the same list in the same order (they take its entries in pieces, and a piece must hold the same
// nodes everywhere), so the order in which a group's parents are listed must not depend on which of two siblings in
// the group happened to be counted second: the first child to arrive leaves its lane and the group's stamp in the
// counter word, and the parent is listed under the larger of its children's lanes when both are in the group.
// p: the parent of the lane's row (-1: none), which the row's list entry carries.
__device__ inline FlowTicket flow_count_at_parent(const Fwd &f, unsigned *seen, int p, unsigned stamp)
{
    FlowTicket t{-1, 0, -1, -1, -1};
    const int lane = (int)__lane_id();                // (recomputed: a value kept across the cell's loop would be spilled)
    if (p >= 0) {
        // counter word: children counted (2 bits) | lane of the first one (6 bits) | stamp of its group (24 bits)
        const unsigned old = __hip_atomic_fetch_add(&seen[p], 1u | (unsigned)lane << 2 | stamp << 8, __ATOMIC_RELAXED,
                                                    __HIP_MEMORY_SCOPE_WORKGROUP);
        const int need = f.pending[p];                // internal children, as the structure pass left it
        t.left = f.left[p];
        t.right = f.right[p];
        t.up = f.parent[p];
        if ((int)(old & 3u) + 1 == need) {
            t.p = p;
            const int other = (int)(old >> 2 & 63u);
            t.key = (need == 2 && old >> 8 == (stamp & 0xFFFFFFu) && other > lane) ? other : lane;
        }
    }
    return t;
}
// Parents that have become ready go to the end of this workgroup's list (its length is kept in LDS), in key order.
// `scratch`: two words of LDS that only this wave uses (the set of keys is put together there: LDS operations of one
// wave are executed in the order in which they are issued).
typedef __attribute__((address_space(3))) unsigned lds_uint;
__device__ inline void flow_append(int4 *list, int capacity, int *len, unsigned *scratch_generic, const FlowTicket &t,
                                   int (*nxt)[FLOW_NXT_ROWS], int win0)
{
    const int lane = threadIdx.x;
    const bool ready = t.p >= 0;
    const unsigned long long own = __ballot(ready && t.key == lane);
    unsigned long long keys = own;
    if (__ballot(ready && t.key != lane) != 0ull) {           // a parent listed under its other child's lane
        lds_uint *scratch = (lds_uint *)scratch_generic;      // (known to be LDS: plain ds_ instructions, no memory waits)
        if (lane == 0) {
            scratch[0] = 0u;
            scratch[1] = 0u;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        if (ready) __hip_atomic_fetch_or(&scratch[t.key >> 5], 1u << (t.key & 31), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        const unsigned lo = __hip_atomic_load(&scratch[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
        const unsigned hi = __hip_atomic_load(&scratch[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
        keys = (unsigned long long)hi << 32 | lo;
    }
    if (keys == 0ull) return;
    int base = 0;
    if (lane == 0) {
        base = *len;
        *len = base + __popcll(keys);
    }
    base = __builtin_amdgcn_readfirstlane(base);
    if (ready) {
        const int pos = base + __popcll(keys & ((1ull << t.key) - 1ull));
        if (pos < capacity) list[pos] = int4{t.p, t.left, t.right, t.up};
        const unsigned at = (unsigned)(pos - win0);
        if (at < (unsigned)FLOW_NXT_ROWS) {
            nxt[0][at] = t.p;
            nxt[1][at] = t.left;
            nxt[2][at] = t.right;
            nxt[3][at] = t.up;
        }
    }
}

template <int EPI, bool VEC4, int SPW, bool BF16 = false>
__global__ __launch_bounds__(WG_THREADS, BF16 ? 2 : 1) void k_flow_persistent(Fwd f)
{
    static_assert(SPW > 0, "the data-flow scheduler uses the weight-stationary cell");
    extern __shared__ __align__(16) unsigned char smem_raw[];
    using Smem = PersistentSmem<SPW, BF16>;
    Smem &sm = *reinterpret_cast<Smem *>(smem_raw);
    Ctl *ctl = f.ctl;
    if (batch_rejected(f) || internal_kernel_skipped(f)) return;
    const int tid = threadIdx.x;
    const int n_slots = gridDim.x / f.n_cg;
    const int member = blockIdx.x % f.n_cg, slot = blockIdx.x / f.n_cg;
    const int my_cg = member;
    PersistentWeights<EpiTraits<EPI>::NG, SPW, BF16> w;        // (loaded below, behind the first requests of the scan)

    // the slot's trees: [t_lo, t_hi), cut where the node count passes slot / n_slots of the batch.  Both cuts are
    // looked for at once, lanes 0-31 of every wave for this slot's and lanes 32-63 for the next one's, 32 candidates per
    // round trip (a bisection is one dependent load per halving).
    int t_lo, t_hi;
    {
        const int lane = tid & 63, half = lane >> 5, i = lane & 31;
        const long long bound = ((long long)(slot + half) * f.n_nodes + n_slots - 1) / n_slots;
        int lo = 0, hi = f.n_trees;                   // smallest t with tree_off[t] >= bound is in [lo, hi]; tree_off[n_trees] = n_nodes >= bound
        while (__ballot(lo < hi) != 0ull) {
            const int step = (hi - lo + 30) / 31;     // candidates lo, lo + step, ..., the last one clamped to hi
            const int cand = min(lo + i * step, hi);
            const bool ge = cand >= hi || f.tree_off[cand] >= bound;                    // (at hi it holds by the invariant)
            const unsigned long long m = __ballot(ge) >> (32 * half) & 0xFFFFFFFFull;   // never empty: the last candidate is hi
            const int k = __builtin_ctzll(m);         // first candidate at or above the cut
            if (lo < hi) {
                const int new_hi = min(lo + k * step, hi);
                lo = k == 0 ? lo : min(lo + (k - 1) * step, hi) + 1;                    // (k == 0: the cut is lo itself)
                hi = new_hi;
            }
        }
        t_lo = __builtin_amdgcn_readlane(lo, 0);      // (scalar values, like everything derived from them)
        t_hi = __builtin_amdgcn_readlane(lo, 32);
    }
    const int nb = f.tree_off[t_lo], ne = f.tree_off[t_hi];
    const int slot_internal = ((ne - nb) - (t_hi - t_lo)) / 2;      // full binary trees
    if (ne <= nb) return;
    unsigned *seen = reinterpret_cast<unsigned *>(f.flow_seen) + (size_t)member * f.n_nodes;   // this workgroup's own: [nb, ne) of it
    int4 *list = f.flow_list + (size_t)member * f.n_int + (nb - t_lo) / 2;
    int *len = &sm.cmd[4];
    if (tid == 0) {
        sm.cmd[6] = 0;                                // roots found
        sm.cmd[7] = 0;                                // a wait was abandoned
    }
    __syncthreads();
    // the list starts with the slot's nodes over two leaves, in node order.  The same pass over the slot's nodes counts
    // the roots (nodes without a parent): there must be one per tree (a second one in a tree is caught where the roots
    // are copied out, after the last piece).  A thread looks at four consecutive nodes per round, all their loads in
    // flight together: a round costs a memory round trip and two barriers however many nodes it covers.
    constexpr int SCAN_Q = 4;
    int l[SCAN_Q], r[SCAN_Q], up[SCAN_Q], pend[SCAN_Q];
    auto scan_requests = [&](int base) {
#pragma unroll
        for (int j = 0; j < SCAN_Q; ++j) {
            const int n = min(base + tid * SCAN_Q + j, ne - 1);       // (ne > nb here)
            l[j] = f.left[n];
            r[j] = f.right[n];
            up[j] = f.parent[n];
            pend[j] = f.pending[n];
        }
    };
    // The first round's requests go out in front of the weights' (a wave's loads return in order): the scan of a slot
    // of up to 1 024 nodes then runs while the weights arrive, instead of behind them.
    scan_requests(nb);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (BF16) ws_load(w, sm, f.inner, my_cg, tid >> 6, tid & 63);
    else ws_load(w, f.inner, my_cg, tid >> 6, tid & 63);
    __builtin_amdgcn_sched_barrier(0);
    for (int n = nb + tid; n < ne; n += WG_THREADS) seen[n] = 0u;
    int n_listed = 0, n_roots = 0;
    for (int base = nb; base < ne; base += WG_THREADS * SCAN_Q) {
        const int n0 = base + tid * SCAN_Q;
        if (base != nb) scan_requests(base);
        unsigned seeds = 0u;
        const unsigned long long below = (1ull << (tid & 63)) - 1ull;
        int before = 0, in_wave = 0;                  // seeds of lower lanes of this wave, and of the whole wave
#pragma unroll
        for (int j = 0; j < SCAN_Q; ++j) {
            const bool here = n0 + j < ne;
            const bool seed = here && l[j] >= 0 && pend[j] == 0;
            const unsigned long long mask = __ballot(seed);
            before += __popcll(mask & below);
            in_wave += __popcll(mask);
            seeds |= (seed ? 1u : 0u) << j;
            if (f.flow_roots) {
                const bool is_root = here && up[j] < 0;
                n_roots += __popcll(__ballot(is_root));       // (every wave counts its own; added up below)
                if (is_root) {
                    const int at = atomicAdd(&sm.cmd[6], 1);
                    if (at < FLOW_ROOTS_KEPT) sm.roots[at] = n0 + j;
                }
            }
        }
        __syncthreads();                              // (the counts of the previous round have been read)
        if ((tid & 63) == 0) sm.cmd[tid >> 6] = in_wave;
        __syncthreads();
        int at = n_listed + before;
        for (int wv = 0; wv < (tid >> 6); ++wv) at += sm.cmd[wv];
#pragma unroll
        for (int j = 0; j < SCAN_Q; ++j) {
            if (seeds >> j & 1u) {
                if (at < slot_internal) list[at] = int4{n0 + j, l[j], r[j], up[j]};
                at += 1;
            }
        }
        n_listed += sm.cmd[0] + sm.cmd[1] + sm.cmd[2] + sm.cmd[3];
    }
    __syncthreads();
    if (f.flow_roots) {
        if ((tid & 63) == 0) sm.cmd[tid >> 6] = n_roots;
        __syncthreads();
        if (tid == 0 && member == 0 && sm.cmd[0] + sm.cmd[1] + sm.cmd[2] + sm.cmd[3] != t_hi - t_lo) latch_error(ctl, TL_ESTRUCT);
    }
    const int roots_found = sm.cmd[6];
    if (tid == 0) *len = n_listed;
    wait_mem();
    __syncthreads();
    // The list is taken in pieces of whole 16-row blocks as long as it holds that many: what is left over waits for
    // the entries that the piece itself brings (a node is listed when its last child is handed out, so everything
    // listed so far depends on earlier pieces only, and the rows of a piece never wait for each other).
    // A piece that takes everything the list holds is followed by a piece of entries that it lists itself: those
    // are also kept in LDS (sm.nxt), so that in the narrow part of a tree - where every step waits for the one
    // before - the next piece's rows are known without a trip to the list in memory.
    int begin = 0, pieces = 0;
    bool from_lds = false;
    for (;;) {
        const int avail = min(*len, slot_internal) - begin;
        if (avail <= 0) break;                        // every listed node has been handed out, so nothing more will be listed
        int count = min(avail, WS_TABLE_ROWS);
        if (count > 16) count &= ~15;
        {
            // rows beyond the piece stand in with the sources of its first row: they are requested like the others
            // (a request needs no test), so they must be rows that do become valid
            const int i = tid < count ? tid : 0;
            int4 rec;
            if (from_lds) rec = int4{sm.nxt[0][i], sm.nxt[1][i], sm.nxt[2][i], sm.nxt[3][i]};
            else rec = list[begin + i];
            sm.node[tid] = tid < count ? rec.x : -1;
            sm.src0[tid] = rec.y;
            sm.src1[tid] = rec.z;
            sm.par[tid] = tid < count ? rec.w : -1;
        }
        const bool takes_all = avail == count;
        const int win0 = takes_all ? begin + count : -(1 << 30);
        __syncthreads();
        // Wave 0 counts the piece's rows at their parents, 64 rows (four blocks) at a time; the parent of a row comes with
        // its list entry.  The count (a chain of two memory round trips) is sent when the group's first block has its
        // rows - for the first group: as soon as the first row requests are out - and what it brings back is used with
        // the group's last block, or after the last matrix instructions of the piece, to list the parents that have
        // become ready.  (Using it one block after the count instead, right after that block's rows have arrived,
        // was measured: slower, the count's answers are not always there by then.)
        FlowTicket ticket{-1, 0, -1, -1, -1};
        const unsigned stamp0 = (unsigned)pieces * (WS_TABLE_ROWS / 64) + 1u;
        unsigned *scratch = reinterpret_cast<unsigned *>(&sm.cmd[5]);
        auto hook = [&](int where) {
            if (tid >= 64) return;
            if (where == -1) {
                ticket = flow_count_at_parent(f, seen, sm.par[tid], stamp0);
            } else if (where == -2) {
                flow_append(list, slot_internal, len, scratch, ticket, sm.nxt, win0);
                ticket.p = -1;
            } else if (where > 0 && (where & 3) == 0) {
                ticket = flow_count_at_parent(f, seen, where * 16 + tid < count ? sm.par[where * 16 + tid] : -1, stamp0 + (unsigned)(where >> 2));
            } else if ((where & 3) == 3) {
                flow_append(list, slot_internal, len, scratch, ticket, sm.nxt, win0);
                ticket.p = -1;
            }
        };
        if constexpr (BF16) ws_tile<EPI, true, SPW, true>(sm, f, f.inner, f.hb, f.n_nodes, f.hs, count, my_cg, w, hook);
        else ws_tile<EPI, true, SPW, !VEC4, true>(sm, f, f.inner, f.h, f.n_nodes, count, my_cg, w, hook);
        if (sm.cmd[7] != 0) return;                   // a wait was abandoned: everybody leaves
        pieces += 1;
        begin += count;
        // (wave 0 has listed the piece's last parents before the last barrier inside the cell, so *len and sm.nxt are final)
        from_lds = takes_all && *len - begin <= FLOW_NXT_ROWS;      // everything listed since is in the LDS tables
        if (!from_lds) {
            wait_mem();                               // the next piece is read from the list in memory: wave 0's entries have arrived there
            __syncthreads();
        }
    }
    if (tid == 0) {
        __hip_atomic_fetch_max(&ctl->n_levels, pieces + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (begin < slot_internal) latch_error(ctl, TL_ESTRUCT);     // nodes that never became ready: not a forest
    }
    if (f.flow_roots) {
        // the roots' states, every workgroup the hidden units it has computed itself (or, for a tree of one node,
        // that the leaf kernel has left), once its own stores have arrived
        wait_mem();
        __syncthreads();
        if (roots_found <= FLOW_ROOTS_KEPT) {
            for (int i = tid; i < roots_found; i += WG_THREADS) flow_copy_root(f, sm.roots[i], my_cg, t_lo, t_hi);
        } else {
            for (int n = nb + tid; n < ne; n += WG_THREADS)
                if (f.parent[n] < 0) flow_copy_root(f, n, my_cg, t_lo, t_hi);
        }
    }
}

// ---------------------------------------------------------------------------------------
// Ready-counter scheduler (Section 4.1): the device form of "the master enqueues an operation
// once all of its inputs are resolved; idle execution threads take operations off the ready
// queue".  State, all in device memory:
//   pending[n]   internal children of n that have not finished
//   q_nodes[]    append-only ready queue; q_tail = entries reserved, q_head = entries consumed
//   gangs[g]     mailbox of gang g
// The grid is n_gangs gangs.  A gang is one scheduler workgroup (the master's role) and
// gang_size compute workgroups (the workers); compute member j owns column group(s)
// gang_cg(j, ..), so a gang covers all hidden units of a tile.  The scheduler cuts a tile of
// ready nodes off the queue, resolves their child rows and posts the tile in the gang's mailbox -
// up to GANG_RING tiles ahead of the compute workgroups, so that they find the next tile waiting
// when they finish one.  Every compute member evaluates its columns and counts itself done; the
// scheduler then decrements the counter of each row's parent and pushes parents that reach zero.
// Gangs run independently of each other: no barrier spans the grid, and a tile starts as soon as
// its nodes are ready and a gang is free.  Every wait is bounded by spin_limit and by the abort
// flag, so the grid always drains.
__device__ inline unsigned long long slot_entry(unsigned seq, unsigned rows, int value)
{
    return ((unsigned long long)((seq << 8) | rows) << 32) | (unsigned)value;
}

// Scheduler workgroup: only its first wave works, one lane per row of a tile.
__device__ inline void ready_scheduler(const Fwd &f, GangBox *box)
{
    Ctl *ctl = f.ctl;
    const int lane = threadIdx.x;
    if (lane >= 64) return;
    const unsigned n_int = (unsigned)f.n_int;
    unsigned published = 0, completed = 0;       // tiles posted / tiles whose parents have been resolved
    // this lane's row of the tiles in flight: its parent (-1: none) and the parent's children and distance from the
    // root.  They are looked up when the tile is posted, while the compute workgroups are busy with it, so that a
    // finished tile costs one round trip (the decrement) before its parents can be handed on, not three.
    int my_p[GANG_RING], my_pl[GANG_RING], my_pr[GANG_RING], my_pd[GANG_RING];
#pragma unroll
    for (int r = 0; r < GANG_RING; ++r) { my_p[r] = -1; my_pl[r] = -1; my_pr[r] = -1; my_pd[r] = 0; }
    auto remember = [&](int r, int node) {
        int p = -1, pl = -1, pr = -1, pd = 0;
        if (node >= 0) {
            p = f.parent[node];
            if (p >= 0) {
                pl = f.left[p];
                pr = f.right[p];
                if (f.priority) pd = f.depth_root[p];
            }
        }
#pragma unroll
        for (int q = 0; q < GANG_RING; ++q)
            if (q == r) { my_p[q] = p; my_pl[q] = pl; my_pr[q] = pr; my_pd[q] = pd; }
    };
    int spins = 0;
    unsigned last_head = 0u, last_tail = 0u, last_direct = ~0u;
    bool leave = false;
    // priorities: a parent with at least crit_thr dependent steps above it is critical; while this gang holds
    // critical nodes (handed back to it tile after tile) it takes nothing else off the queue
    const int crit_thr = f.priority ? critical_threshold(f) : 0x7fffffff;
    bool holding = false;
    while (!leave) {
        bool progress = false;
        // ---- (1) a finished tile: resolve its rows' parents -------------------------------
        if (completed < published) {
            // tile number t = completed + 1 is the ceil(t / GANG_RING)-th tile of ring slot t % GANG_RING
            const unsigned t = completed + 1;
            const int r = (int)(t % GANG_RING);
            unsigned d = 0;
            if (lane == 0) d = ld_dev(&box->done[r].v);
            d = __shfl(d, 0);
            if (d >= (t + GANG_RING - 1) / GANG_RING * (unsigned)f.gang_size) {
                int p = -1, pl = -1, pr = -1, pd = 0;
#pragma unroll
                for (int q = 0; q < GANG_RING; ++q)
                    if (q == r) { p = my_p[q]; pl = my_pl[q]; pr = my_pr[q]; pd = my_pd[q]; }
                if (p >= 0 && add_dev(&f.pending[p], -1) != 1) p = -1;
                const unsigned long long ready = __ballot(p >= 0);
                // Parents that became ready.  While the queue holds less than one row per gang (the regime
                // in which the next dependent step waits for this one: chains, the top of a tree) they go
                // straight back to this gang as its next tile: no queue round trip between a node and its
                // parent.  Otherwise they are pushed on the queue with one reservation on q_tail for the
                // tile (handing them back while the queue is well filled only cuts the work into many
                // small tiles: measured).  With priorities, critical parents are handed back in any case.
                const bool scarce = last_tail - last_head < (unsigned)f.n_gangs;
                const unsigned long long critical = f.priority ? __ballot(p >= 0 && pd >= crit_thr) : 0ull;
                const unsigned long long direct_set = scarce ? ready : critical;
                const unsigned long long queue_set = ready & ~direct_set;
                const int n_direct = __popcll(direct_set), n_queue = __popcll(queue_set);
                holding = critical != 0ull;
                if (n_direct > 0) {
                    // lane j < n_direct takes the j-th chosen lane's node (position of the j-th set bit)
                    int pos = 0, rem = lane;
#pragma unroll
                    for (int b = 32; b >= 1; b >>= 1) {
                        const int cnt = __popcll(direct_set & (((1ull << b) - 1ull) << pos));
                        if (cnt <= rem) { pos += b; rem -= cnt; }
                    }
                    pos &= 63;
                    int node2 = __shfl(p, pos), s0 = __shfl(pl, pos), s1 = __shfl(pr, pos);
                    if (lane >= n_direct) node2 = s0 = s1 = -1;
                    if (lane == 0) add_dev(&ctl->direct.v, (unsigned)n_direct);
                    const unsigned seq = published + 1;
                    const int r2 = (int)(seq % GANG_RING);
                    unsigned long long *e = box->slot[r2];
                    st_dev(&e[lane], slot_entry(seq, (unsigned)n_direct, node2));
                    st_dev(&e[TILE_ROWS + lane], slot_entry(seq, (unsigned)n_direct, s0));
                    st_dev(&e[2 * TILE_ROWS + lane], slot_entry(seq, (unsigned)n_direct, s1));
                    remember(r2, node2);
                    published += 1;
                }
                if (n_queue > 0) {
                    unsigned base = 0;
                    if (lane == 0) base = add_dev(&ctl->q_tail.v, (unsigned)n_queue);
                    base = __shfl(base, 0);
                    if ((queue_set >> lane) & 1ull) {
                        const unsigned slot = base + (unsigned)__popcll(queue_set & ((1ull << lane) - 1ull));
                        if (slot < n_int) qrec_store<true>(&f.q_rec[slot], p, pl, pr);
                    }
                }
                completed += 1;
                progress = true;
            }
        }
        // ---- (2) room in the ring: cut the next tile off the ready queue --------------------
        unsigned head = 0, tail = 0, direct = 0;
        if (lane == 0) { head = ld_dev(&ctl->q_head.v); tail = ld_dev(&ctl->q_tail.v); direct = ld_dev(&ctl->direct.v); }
        head = __shfl(head, 0);
        tail = __shfl(tail, 0);
        direct = __shfl(direct, 0);
        if (tail > n_int) tail = n_int;
        if (head != last_head || tail != last_tail || direct != last_direct) {   // others progress
            last_head = head;
            last_tail = tail;
            last_direct = direct;
            spins = 0;
        }
        const unsigned in_flight = published - completed;
        if (!holding && in_flight < (unsigned)GANG_RING && tail > head) {
            const unsigned avail = tail - head;
            // an idle gang takes what there is; a busy gang looks ahead only when there is plenty for all
            if (in_flight == 0 || avail >= 16u * (unsigned)f.n_gangs) {
                const unsigned m = (unsigned)tile_rows_for(avail, (unsigned)f.n_gangs);
                int won = 0;
                if (lane == 0) { unsigned expect = head; won = cas_dev(&ctl->q_head.v, &expect, head + m) ? 1 : 0; }
                won = __shfl(won, 0);
                if (won) {
                    const unsigned seq = published + 1;
                    int node = -1, s0 = -1, s1 = -1;
                    if ((unsigned)lane < m) {
                        int wait = 0;
                        bool there;
                        while (!(there = qrec_load(&f.q_rec[head + lane], &node, &s0, &s1))) {   // reserved, not written yet
                            if (++wait > f.spin_limit) break;
                            backoff();
                        }
                        if (!there) {
                            node = s0 = s1 = -1;
                            st_dev(&ctl->abort.v, 1u);
                            latch_error(ctl, TL_ESTALL);
                        }
                    }
                    const int r = (int)(seq % GANG_RING);
                    unsigned long long *e = box->slot[r];
                    st_dev(&e[lane], slot_entry(seq, m, node));
                    st_dev(&e[TILE_ROWS + lane], slot_entry(seq, m, s0));
                    st_dev(&e[2 * TILE_ROWS + lane], slot_entry(seq, m, s1));
                    remember(r, node);
                    published += 1;
                    progress = true;
                }
            }
        }
        // ---- (3) leave when every node has been handed out and all own tiles are resolved -----
        if (published == completed) {
            unsigned ab = 0;
            if (lane == 0) ab = ld_dev(&ctl->abort.v);
            ab = __shfl(ab, 0);
            if (head + direct >= n_int || ab) leave = true;     // every node has been handed out, by the queue or directly
        }
        if (progress) {
            spins = 0;
        } else if (!leave) {
            if (++spins > f.spin_limit) {
                st_dev(&ctl->abort.v, 1u);
                latch_error(ctl, TL_ESTALL);
                leave = true;           // compute workgroups stuck in a tile give up by their own budget
            }
            backoff();
        }
    }
    // "leave" message in the next slot; statistics
    const unsigned seq = published + 1;
    unsigned long long *e = box->slot[seq % GANG_RING];
    st_dev(&e[lane], slot_entry(seq, 0, VALUE_EXIT));
    st_dev(&e[TILE_ROWS + lane], slot_entry(seq, 0, -1));
    st_dev(&e[2 * TILE_ROWS + lane], slot_entry(seq, 0, -1));
    if (lane == 0) add_dev(&ctl->tiles.v, published);
}

template <int EPI, bool VEC4, int SPW, bool BF16 = false>
__global__ __launch_bounds__(WG_THREADS, (SPW > 0 && !BF16) ? 1 : 2) void k_ready_persistent(Fwd f)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    using Smem = PersistentSmem<SPW, BF16>;
    Smem &sm = *reinterpret_cast<Smem *>(smem_raw);
    if (batch_rejected(f)) return;
    const int tid = threadIdx.x;
    const int n_compute = f.n_gangs * f.gang_size;
    if ((int)blockIdx.x >= n_compute) {           // scheduler workgroups come after all compute workgroups
        ready_scheduler(f, &f.gangs[blockIdx.x - n_compute]);
        return;
    }
    const int gang = blockIdx.x / f.gang_size, member = blockIdx.x % f.gang_size;
    GangBox *box = &f.gangs[gang];
    // weight-stationary cell (SPW > 0): gang_size == n_cg, the member's column group is fixed
    const int my_cg = gang_cg(member, f.gang_size, f.n_cg);
    PersistentWeights<EpiTraits<EPI>::NG, SPW, BF16> w;
    if constexpr (SPW > 0) {
        if constexpr (BF16) ws_load(w, sm, f.inner, my_cg, tid >> 6, tid & 63);
        else ws_load(w, f.inner, my_cg, tid >> 6, tid & 63);
        // tiles have at most TILE_ROWS rows here; the rest of the cell's row tables reads "no row"
        sm.node[tid] = -1;
        sm.src0[tid] = 0;
        sm.src1[tid] = 0;
    }

    unsigned long long entry = 0;                 // this thread's entry of the next tile, requested ahead
    if (tid < SLOT_ENTRIES) entry = ld_dev(&box->slot[1 % GANG_RING][tid]);
    for (unsigned seq = 1;; ++seq) {
        // ---- rows of tile `seq`: wait until this thread's entry carries the tile's tag ----------
        if (tid == 0) sm.cmd[2] = 1;
        __syncthreads();
        if (tid < SLOT_ENTRIES) {
            long long polls = 0;
            while ((unsigned)(entry >> 40) != seq) {
                if (++polls > 64ll * f.spin_limit) { sm.cmd[2] = 0; break; }   // the scheduler always posts; safety net
                backoff();
                entry = ld_dev(&box->slot[seq % GANG_RING][tid]);
            }
            const int value = (int)(unsigned)entry;
            if (tid < TILE_ROWS) sm.node[tid] = value;
            else if (tid < 2 * TILE_ROWS) sm.src0[tid - TILE_ROWS] = SPW > 0 ? max(value, 0) : value;
            else sm.src1[tid - 2 * TILE_ROWS] = SPW > 0 ? max(value, 0) : value;
            if (tid == 0) {
                sm.cmd[0] = (int)((entry >> 32) & 0xffu);
                // RNTN cell: this workgroup adds up all parts itself, or (gangs of several workgroups per column group)
                // its own part, in the scratch unit of this gang and ring slot
                sm.cmd[5] = f.gang_parts > 1 ? member / f.n_cg : -1;
                sm.cmd[6] = gang * GANG_RING + (int)(seq % GANG_RING);
            }
        }
        __syncthreads();
        const int count = sm.cmd[0];
        if (sm.cmd[2] == 0 || sm.node[0] == VALUE_EXIT || count == 0) return;
        // request the next tile's entry now; it arrives while this tile is computed
        if (tid < SLOT_ENTRIES) entry = ld_dev(&box->slot[(seq + 1) % GANG_RING][tid]);

        if constexpr (SPW > 0 && BF16) {
            ws_tile<EPI, true, SPW>(sm, f, f.inner, f.hb, f.n_nodes, f.hs, count, my_cg, w);
        } else if constexpr (SPW > 0) {
            ws_tile<EPI, true, SPW, !VEC4>(sm, f, f.inner, f.h, f.n_nodes, count, my_cg, w);
        } else {
            if (f.gang_parts > 1) {
                cell_tile<EPI, VEC4, true, BF16>(sm, f, f.inner, f.h, count, member % f.n_cg);
            } else {
                for (int j = member; j < f.n_cg; j += f.gang_size)
                    cell_tile<EPI, VEC4, true, BF16>(sm, f, f.inner, f.h, count, gang_cg(j, f.gang_size, f.n_cg));
            }
        }

        // ---- completion: the tile's h/c rows are in memory before the scheduler hears of it -----
        wait_mem();
        __syncthreads();
        if (tid == 0) add_dev(&box->done[seq % GANG_RING].v, 1u);
    }
}

}  // namespace tl
