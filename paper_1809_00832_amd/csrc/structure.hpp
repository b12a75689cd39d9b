// Structure pass: integer-only kernels that turn the child arrays of a batch into what the
// schedulers need.  This is the device counterpart of the master that sorts operations into a
// ready queue or a waiting list by their number of unresolved inputs (Section 4.1, Figure 4
// step 2) and of the parent pointers that stand in for a call stack ("Graph execution stack").
//
// Counters that many threads bump at once are bumped once per workgroup (ballot + popcount per
// wave, combined in LDS; LDS histograms): atomics on one address are served one after the other.
#pragma once

#include "common.hpp"

namespace tl {

// Largest t with tree_off[t] <= n, by bisection over [0, n_trees).  Always returns an index in
// range, whatever the array holds.
__device__ inline int tree_of(const int32_t *tree_off, int n_trees, int n)
{
    int lo = 0, hi = n_trees - 1;
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if (tree_off[mid] <= n) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// Slot in an append-only list for every thread with pred set (-1 for the others): one atomic per
// workgroup of up to 1024 threads.  Must be called by
// all threads of the workgroup; s_cnt is shared scratch of APPEND_SCRATCH ints.
constexpr int APPEND_SCRATCH = 17;
template <typename T> __device__ inline int block_append(T *counter, bool pred, int *s_cnt)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = (blockDim.x + 63) >> 6;
    const unsigned long long mask = __ballot(pred);
    if (lane == 0) s_cnt[wave] = __popcll(mask);
    __syncthreads();
    if (threadIdx.x == 0) {
        int total = 0;
        for (int w = 0; w < n_waves; ++w) {
            const int c = s_cnt[w];
            s_cnt[w] = total;
            total += c;
        }
        s_cnt[16] = total ? (int)atomicAdd(counter, (T)total) : 0;
    }
    __syncthreads();
    const int slot = pred ? s_cnt[16] + s_cnt[wave] + __popcll(mask & ((1ull << lane) - 1ull)) : -1;
    __syncthreads();
    return slot;
}

// Threads per workgroup of the per-node kernels that append to lists.
constexpr int NODE_BLOCK = 1024;

// Data-flow scheduler: the rows that internal nodes will produce - c, and the h row their parents gather (the bf16
// copy when there is one) - show "not written" (all ones) in every element until they are.  One wave per row; called
// by all lanes of wave number `wave` of `n_waves`.
__device__ inline void flow_fill(const Fwd &f, size_t wave, size_t n_waves)
{
    const int H = f.H, lane = threadIdx.x & 63;
    const bool quad = (H & 3) == 0 && (((uintptr_t)f.h | (uintptr_t)f.c) & 15) == 0;
    const float ones = __uint_as_float(0xFFFFFFFFu);
    const floatx4 ones4 = floatx4{ones, ones, ones, ones};
    for (size_t n = wave; n < (size_t)f.n_nodes; n += n_waves) {
        if (f.left[n] < 0) continue;
        float *c = f.c ? f.c + n * H : nullptr, *h = f.hb ? nullptr : f.h + n * H;
        if (quad) {
            for (int e = lane * 4; e < H; e += 256) {
                if (c) *reinterpret_cast<floatx4 *>(c + e) = ones4;
                if (h) *reinterpret_cast<floatx4 *>(h + e) = ones4;
            }
        } else {
            for (int e = lane; e < H; e += 64) {
                if (c) c[e] = ones;
                if (h) h[e] = ones;
            }
        }
        if (f.hb) {
            unsigned short *hb = f.hb + n * f.hs;             // rows 16-byte aligned; what lies beyond H stays zero
            for (int e = lane * 8; e < H; e += 512) {
                if (e + 8 <= H) *reinterpret_cast<floatx4 *>(hb + e) = ones4;
                else for (int k = e; k < H; ++k) hb[k] = (unsigned short)0xFFFFu;
            }
        }
    }
}

// Resets the per-forward scheduler state.  A fill kernel rather than memsets so that a caller
// may capture the forward in a HIP graph.
__global__ void k_reset(Fwd f, int with_levels)
{
    const int N = f.n_nodes;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    const size_t ctl_words = sizeof(Ctl) / 4, gang_words = (size_t)MAX_GANGS * sizeof(GangBox) / 4;
    size_t total = (size_t)N + 1;
    if (total < ctl_words) total = ctl_words;
    if (total < gang_words) total = gang_words;
    if (f.rntn_done && total < (size_t)f.rntn_units * f.n_cg) total = (size_t)f.rntn_units * f.n_cg;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        if (i < (size_t)N) {
            f.parent[i] = -1;
            f.pending[i] = 0;
            if (with_levels) { f.height[i] = 0; f.arrive[i] = 0; f.level_fill[i] = 0; }
        }
        if (with_levels && i <= (size_t)N) f.level_cnt[i] = 0;
        if (i < (size_t)f.n_int) { f.q_rec[i].lo = 0; f.q_rec[i].hi = 0; }
        if (i < (size_t)f.n_trees) f.root_ws[i] = -1;
        if (f.rntn_done && i < (size_t)f.rntn_units * f.n_cg) f.rntn_done[i] = 0u;   // (a forward that gave up may have left counts)
        if (i < ctl_words) ((unsigned int *)f.ctl)[i] = 0;
        if (i < gang_words) ((unsigned int *)f.gangs)[i] = 0;
    }
    if (f.flow == 1) flow_fill(f, ((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6, stride >> 6);
}

// One thread per node: checks, parent scatter, leaf list, counters of unfinished children.
// Leaves are evaluated by a kernel of their own before any internal node, so pending[] counts
// internal children only, and an internal node whose children are both leaves starts ready.
__global__ __launch_bounds__(NODE_BLOCK) void k_scatter(Fwd f)
{
    __shared__ int s_cnt[APPEND_SCRATCH];
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    Ctl *ctl = f.ctl;
    if (n <= f.n_trees) {   // offsets: 0 = off[0] < off[1] < ... < off[B] = N
        int v = f.tree_off[n];
        bool ok = (n == 0) ? (v == 0) : (v > f.tree_off[n - 1]);
        if (n == f.n_trees) ok = ok && (v == f.n_nodes);
        if (!ok) latch_error(ctl, TL_ESTRUCT);
    }
    bool is_leaf = false, is_seed = false;
    int l = -1, r = -1;
    if (n < f.n_nodes) {
        const int t = tree_of(f.tree_off, f.n_trees, n);
        const int lo = f.tree_off[t], hi = f.tree_off[t + 1];
        l = f.left[n];
        r = f.right[n];
        if (n < lo || n >= hi) {
            latch_error(ctl, TL_ESTRUCT);
        } else if (l < 0 && r < 0) {
            const int w = f.word[n];
            if (w < 0 || w >= f.vocab) latch_error(ctl, TL_ESTRUCT); else is_leaf = true;
        } else if (l >= lo && l < hi && r >= lo && r < hi && l < f.n_nodes && r < f.n_nodes && l != r && l != n &&
                   r != n) {
            if (atomicCAS(&f.parent[l], -1, n) != -1) latch_error(ctl, TL_ESTRUCT);
            if (atomicCAS(&f.parent[r], -1, n) != -1) latch_error(ctl, TL_ESTRUCT);
            const int pend = (f.left[l] >= 0) + (f.left[r] >= 0);
            f.pending[n] = pend;
            is_seed = pend == 0;
        } else {
            latch_error(ctl, TL_ESTRUCT);
        }
    }
    const int leaf_slot = block_append(&ctl->n_leaf_seen, is_leaf, s_cnt);
    if (is_leaf && leaf_slot < f.n_leaf) f.leaf_list[leaf_slot] = n;
    const int seed_slot = block_append(&ctl->q_tail.v, is_seed, s_cnt);
    if (is_seed && seed_slot < f.n_int) qrec_store<false>(&f.q_rec[seed_slot], n, l, r);
}

// One thread per node: the node nobody points to is its tree's root; there must be exactly one.
__global__ __launch_bounds__(NODE_BLOCK) void k_roots(Fwd f)
{
    __shared__ int s_cnt[APPEND_SCRATCH];
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    Ctl *ctl = f.ctl;
    if (n == 0) {
        if (ctl->n_leaf_seen != f.n_leaf) latch_error(ctl, TL_ESTRUCT);
        ctl->n_seed = (int)ctl->q_tail.v;                // the first frontier: internal nodes over two leaves
    }
    const bool is_root = n < f.n_nodes && f.parent[n] == -1;
    if (is_root) {
        const int t = tree_of(f.tree_off, f.n_trees, n);
        if (atomicCAS(&f.root_ws[t], -1, n) != -1) latch_error(ctl, TL_ESTRUCT);     // a second root of the same tree
    }
    // no tree has two roots, so "as many roots as trees" means one each; later kernels compare the two
    // numbers (batch_rejected) and the root gather reports a mismatch
    block_append(&ctl->n_roots, is_root, s_cnt);
}

// ---- distance from the root (priority scheduling) -----------------------------------------
// One thread per node walks up the parent links and counts, giving up after DEPTH_CAP steps: the
// priority rule only asks whether a node is far from its root compared with the rest of the
// batch, so a distance of "DEPTH_CAP or more" is as good as the exact one, and the longest walk
// (which sets the duration of the kernel) stays short however deep a tree is.  The parent array
// of a batch fits the L2, so a step costs a cache hit.
constexpr int DEPTH_CAP = 128;

__global__ __launch_bounds__(NODE_BLOCK) void k_depth_walk(Fwd f)
{
    __shared__ unsigned s_sum[16];
    if (batch_rejected(f)) return;
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    unsigned d = 0;
    if (n < f.n_nodes) {
        int p = f.parent[n];
        while (p >= 0 && d < (unsigned)DEPTH_CAP) {
            d += 1;
            p = f.parent[p];
        }
        f.depth_root[n] = (int)d;
    }
    unsigned sum = d;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) sum += __shfl_xor(sum, o);
    if ((threadIdx.x & 63) == 0) s_sum[threadIdx.x >> 6] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long total = 0;
        for (int w = 0; w < (int)((blockDim.x + 63) >> 6); ++w) total += s_sum[w];
        if (total) atomicAdd(&f.ctl->depth_sum.v, total);
    }
}

// A node is critical when at least this many dependent steps are still above it: 32, or four times the
// batch's mean if that is more (then nothing is critical in a batch whose mean exceeds DEPTH_CAP / 4).
__device__ inline int critical_threshold(const Fwd &f)
{
    const unsigned long long mean4 = 4ull * f.ctl->depth_sum.v / (unsigned long long)f.n_nodes;
    return mean4 > 32ull ? (mean4 > 0x7fffffffull ? 0x7fffffff : (int)mean4) : 32;
}

// Rewrites the first n_seed records of the ready queue (the internal nodes over two leaves) with the
// critical ones at the front, the others filled in from the back.
__global__ __launch_bounds__(NODE_BLOCK) void k_seed_place(Fwd f)
{
    __shared__ int s_cnt[APPEND_SCRATCH];
    if (batch_rejected(f)) return;
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    Ctl *ctl = f.ctl;
    const int thr = critical_threshold(f);
    bool seed = false, crit = false;
    int l = -1, r = -1;
    if (n < f.n_nodes) {
        l = f.left[n];
        r = f.right[n];
        seed = l >= 0 && f.pending[n] == 0;
        crit = seed && f.depth_root[n] >= thr;
    }
    const int front = block_append(&ctl->seed_front.v, crit, s_cnt);
    const int back = block_append(&ctl->seed_back.v, seed && !crit, s_cnt);
    const int slot = crit ? front : ctl->n_seed - 1 - back;
    if (seed && slot >= 0 && slot < f.n_int) qrec_store<false>(&f.q_rec[slot], n, l, r);
}

// Heights by climbing: one thread per leaf walks towards the root; at every internal node the
// first child to arrive stops, the second continues with height 1 + max.  The walk passes each
// node once, so a thread's loop is bounded by the tree height.  The two children meet through one
// exchange on height[p] (zero before the pass): the first leaves 1 + its own height there and
// finds zero, the second finds the first one's value - the data travels in the word that is
// exchanged, so a step costs two memory round trips (the parent, the exchange) and no fence.
// arrive[p] = 2 marks the nodes whose height is final.
__global__ void k_climb(Fwd f)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (batch_rejected(f) || i >= f.n_leaf) return;
    int n = f.leaf_list[i];
    int hcur = 0;
    for (int guard = 0; guard < f.n_nodes; ++guard) {
        const int p = f.parent[n];
        if (p < 0) break;
        const int other = atomicExch(&f.height[p], hcur + 1);
        if (other == 0) break;                   // the sibling's subtree is not done yet: its thread will carry on
        hcur = other > hcur + 1 ? other : hcur + 1;
        f.height[p] = hcur;
        f.arrive[p] = 2;
        n = p;
    }
}

constexpr int HIST_BINS = 1024;

// One thread per node: histogram of the heights of the internal nodes that the climb reached
// (both children arrived), and the largest height.
__global__ void k_level_hist(Fwd f)
{
    __shared__ int s_hist[HIST_BINS];
    __shared__ int s_max;
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (batch_rejected(f)) return;
    for (int b = threadIdx.x; b < HIST_BINS; b += blockDim.x) s_hist[b] = 0;
    if (threadIdx.x == 0) s_max = 0;
    __syncthreads();
    if (n < f.n_nodes && f.left[n] >= 0 && f.arrive[n] == 2) {
        const int hgt = f.height[n];
        if (hgt < HIST_BINS) atomicAdd(&s_hist[hgt], 1); else atomicAdd(&f.level_cnt[hgt], 1);
        atomicMax(&s_max, hgt);
    }
    __syncthreads();
    for (int b = threadIdx.x; b < HIST_BINS; b += blockDim.x)
        if (s_hist[b]) atomicAdd(&f.level_cnt[b], s_hist[b]);
    if (threadIdx.x == 0 && s_max > 0) atomicMax(&f.ctl->max_height, s_max);
}

// Single workgroup: exclusive scan of the height histogram into level offsets.  Height 0 (the
// leaves) has no list: leaves are taken from leaf_list.
__global__ void k_scan_levels(Fwd f)
{
    __shared__ int s_part[1024];
    __shared__ int s_carry;
    Ctl *ctl = f.ctl;
    const int tid = threadIdx.x;
    if (batch_rejected(f)) {
        if (tid == 0) {
            ctl->n_levels = 0;
            latch_error(ctl, TL_ESTRUCT);
        }
        return;
    }
    const int n_levels = ctl->max_height + 1;
    if (tid == 0) s_carry = 0;
    __syncthreads();
    for (int base = 0; base < n_levels; base += 1024) {
        const int idx = base + tid;
        const int v = idx < n_levels ? f.level_cnt[idx] : 0;
        s_part[tid] = v;
        __syncthreads();
        for (int d = 1; d < 1024; d <<= 1) {
            int add = tid >= d ? s_part[tid - d] : 0;
            __syncthreads();
            s_part[tid] += add;
            __syncthreads();
        }
        const int carry = s_carry;
        if (idx < n_levels) f.level_off[idx] = carry + s_part[tid] - v;
        __syncthreads();
        if (tid == 1023) s_carry = carry + s_part[1023];
        __syncthreads();
    }
    if (tid == 0) {
        f.level_off[n_levels] = s_carry;
        ctl->n_levels = n_levels;
        ctl->reached = s_carry + f.n_leaf;
        if (s_carry != f.n_int) latch_error(ctl, TL_ESTRUCT);   // nodes no leaf leads to (cycle)
    }
}

// One thread per node: append every reached internal node to the list of its height.
__global__ void k_fill_levels(Fwd f)
{
    __shared__ int s_hist[HIST_BINS];
    __shared__ int s_base[HIST_BINS];
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (batch_rejected(f)) return;
    for (int b = threadIdx.x; b < HIST_BINS; b += blockDim.x) s_hist[b] = 0;
    __syncthreads();
    const bool mine = n < f.n_nodes && f.left[n] >= 0 && f.arrive[n] == 2;
    int hgt = 0, rank = 0;
    if (mine) {
        hgt = f.height[n];
        rank = hgt < HIST_BINS ? atomicAdd(&s_hist[hgt], 1) : atomicAdd(&f.level_fill[hgt], 1);
    }
    __syncthreads();
    for (int b = threadIdx.x; b < HIST_BINS; b += blockDim.x)
        if (s_hist[b]) s_base[b] = atomicAdd(&f.level_fill[b], s_hist[b]);
    __syncthreads();
    if (mine) {
        const int slot = f.level_off[hgt] + rank + (hgt < HIST_BINS ? s_base[hgt] : 0);
        if (slot < f.n_int) f.level_nodes[slot] = n;
    }
}

// h_root / c_root / root outputs.
__global__ void k_root_gather(Fwd f)
{
    if (batch_rejected(f)) {
        if (blockIdx.x == 0 && threadIdx.x == 0) latch_error(f.ctl, TL_ESTRUCT);    // a tree without a root
        return;
    }
    const int t = blockIdx.x;
    const int r = f.root_ws[t];
    if (r < 0) return;
    if (threadIdx.x == 0 && f.root_out) f.root_out[t] = r;
    for (int j = threadIdx.x; j < f.H; j += blockDim.x) {
        if (f.h_root) f.h_root[(size_t)t * f.H + j] = f.h[(size_t)r * f.H + j];
        if (f.c_root && f.c) f.c_root[(size_t)t * f.H + j] = f.c[(size_t)r * f.H + j];
    }
}

}  // namespace tl
