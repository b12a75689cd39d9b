// Shared definitions of the tree-network forward library (device + host).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "treelstm.h"

namespace tl {

// ---- tiling constants ---------------------------------------------------------------
// A tile is up to TILE_ROWS ready nodes times one column group of HU hidden units (all
// gates of those units, so that the gate epilogue stays in registers).  The contraction
// runs on v_mfma_f32_16x16x4_f32 / v_mfma_f32_16x16x32_bf16: 16 rows x 16 hidden units
// per wave, K consumed in chunks of KC staged through LDS.
constexpr int TILE_ROWS = 64;
constexpr int HU = 16;
constexpr int KC = 64;            // K elements per LDS chunk (4 MFMA k-steps of 16)
constexpr int STEP_K = 16;        // K elements per k-step (4 lane groups x 4)
constexpr int A_LD = KC + 4;      // LDS row stride of the A chunk in floats (pad: bank spread)
constexpr int WG_THREADS = 256;   // 4 waves
constexpr int MAX_GATES = 5;
constexpr int N_XCD = 8;          // L2 domains of the chip; workgroups are dealt to them round-robin

typedef float floatx4 __attribute__((ext_vector_type(4)));

// ---- scheduler control block (device memory, zeroed at the start of every forward) ---
struct Ctl {
    unsigned long long formed;    // low 32: ready-queue entries consumed into tiles; high 32: tiles formed
    unsigned int q_tail;          // ready-queue entries reserved by producers
    unsigned int tiles_done;      // tiles whose every column group has finished
    unsigned int part_next[N_XCD];// next (tile, column group) item of each column-group partition
    unsigned int bar_count;       // grid barrier arrivals (level scheduler)
    int status;                   // first latched tl_error
    int abort;                    // set when a waiting workgroup gives up; everybody leaves
    int n_leaf_seen;              // leaves counted by the structure pass
    int max_height;
    int n_levels;
    int reached;                  // nodes reached bottom-up from the leaves
    int pad;
};

// One contraction: rows gathered from `SEG` source rows of length L, times packed weights.
struct Gemm {
    const void *wp;     // packed weights, see pack.hpp
    const float *bp;    // packed bias [n_cg][NG][HU]
    int L;              // length of one source segment (E for leaves, H for internal nodes)
    int Lp;             // L rounded up to a multiple of 4
    int n_chunks;       // padded K / KC
};

// Everything a forward kernel needs, passed by value.
struct Fwd {
    int n_trees, n_nodes, n_leaf, n_int;
    const int32_t *tree_off, *left, *right, *word;
    float *h, *c;
    float *h_root, *c_root;
    int32_t *root_out;
    // model
    int cell, H, E, vocab, n_cg, bf16;
    const float *emb;           // fp32 embedding table (as given)
    const void *emb_lo;         // bf16 copy (bf16-operand mode)
    void *h_lo;                 // bf16 shadow of h, [n_nodes x H] (bf16-operand mode)
    Gemm leaf, inner;
    // workspace
    int32_t *parent, *pending, *leaf_list, *root_ws;
    int32_t *height, *arrive, *level_cnt, *level_off, *level_fill, *level_nodes;
    unsigned int *q_nodes;            // ready queue: node index + 1, 0 = slot not written yet
    unsigned long long *tile_desc;    // per formed tile: start | rows << 32 | 1 << 63
    unsigned int *tile_done;          // per formed tile: column groups finished
    Ctl *ctl;
    int spin_limit;
    int cap_tiles;                    // tiles the launched grid can work on at once
};

// ---- agent-scope atomics ---------------------------------------------------------------
template <typename T> __device__ inline T ld_relaxed(const T *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T> __device__ inline void st_release(T *p, T v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T> __device__ inline void st_relaxed(T *p, T v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T> __device__ inline T add_acq_rel(T *p, T v)
{
    return __hip_atomic_fetch_add(p, v, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T> __device__ inline T add_relaxed(T *p, T v)
{
    return __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T> __device__ inline bool cas_acq_rel(T *p, T *expected, T desired)
{
    return __hip_atomic_compare_exchange_strong(p, expected, desired, __ATOMIC_ACQ_REL, __ATOMIC_RELAXED,
                                                __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void fence_acquire() { __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent"); }
__device__ inline void fence_release() { __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent"); }

__device__ inline void latch_error(Ctl *ctl, int code)
{
    int expected = 0;
    __hip_atomic_compare_exchange_strong(&ctl->status, &expected, code, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_AGENT);
}

// Rows per tile when `avail` ready rows meet room for `free_tiles` more tiles: spread the rows
// over the free room in units of 16, at most TILE_ROWS; with no room only full tiles are worth
// forming (0 = wait for more rows).
__host__ __device__ inline int tile_rows_for(unsigned avail, unsigned free_tiles)
{
    if (avail == 0) return 0;
    if (free_tiles == 0) return avail >= (unsigned)TILE_ROWS ? TILE_ROWS : 0;
    unsigned per = (avail + free_tiles - 1) / free_tiles;
    unsigned m = (per + 15u) & ~15u;
    if (m < 16u) m = 16u;
    if (m > (unsigned)TILE_ROWS) m = TILE_ROWS;
    return (int)(m < avail ? m : avail);
}

// Column groups are split into min(n_cg, N_XCD) contiguous partitions; the workgroups of one
// L2 domain prefer one partition, so that its slice of the weights stays in that L2.
__host__ __device__ inline int part_start(int p, int n_cg, int n_parts) { return (int)((long long)p * n_cg / n_parts); }

}  // namespace tl
