// Shared definitions of the tree-network forward library (device + host).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "treelstm.h"

namespace tl {

// ---- tiling constants ---------------------------------------------------------------
// A tile is up to TILE_ROWS ready nodes times one column group of HU hidden units (all
// gates of those units, so that the gate epilogue stays in registers).  The contraction
// runs on v_mfma_f32_16x16x4_f32: 16 rows x 16 hidden units per wave and k-step of 16.
constexpr int TILE_ROWS = 64;
constexpr int HU = 16;
constexpr int KC = 64;            // K elements per LDS chunk (4 MFMA k-steps of 16)
constexpr int STEP_K = 16;        // K elements per k-step (4 lane groups x 4)
constexpr int A_LD = KC + 4;      // LDS row stride of the A chunk in floats (pad: bank spread)
constexpr int WG_THREADS = 256;   // 4 waves
constexpr int MAX_GATES = 5;
constexpr int N_XCD = 8;          // L2 domains of the chip; workgroups are dealt to them round-robin
constexpr int MAX_GANGS = 64;
constexpr int LINE = 128;         // bytes; every word that is polled or hammered gets its own line

typedef float floatx4 __attribute__((ext_vector_type(4)));

struct alignas(LINE) Line {
    unsigned int v;
    unsigned int pad[LINE / 4 - 1];
};
struct alignas(LINE) Line64 {
    unsigned long long v;
    unsigned long long pad[LINE / 8 - 1];
};

// ---- scheduler control block (device memory, zeroed at the start of every forward) ---
struct alignas(LINE) Ctl {
    // line 0: written rarely, read by the host
    int status;                   // first latched tl_error
    int n_leaf_seen;              // leaves counted by the structure pass
    int n_seed;                   // internal nodes that start ready (both children are leaves)
    int max_height;
    int n_levels;
    int reached;                  // nodes reached bottom-up from the leaves
    int tiles_formed;             // ready scheduler: tiles of ready nodes formed
    int n_roots;                  // nodes without a parent found by the structure pass (one per tree in a valid batch)
    int pad0[LINE / 4 - 8];
    Line abort;                   // set when a waiting workgroup gives up; everybody leaves
    Line q_head;                  // ready-queue entries consumed into tiles
    Line q_tail;                  // ready-queue entries reserved by producers
    Line tiles;                   // tiles formed (statistics only)
    Line direct;                  // nodes that a scheduler handed to its own gang without passing the queue
    Line truncated;               // top-down generation: nodes that would have expanded but found no free rows
    // top-down generation, data-flow form: rows reserved for children so far (low half; the roots' rows are not counted)
    // and rows whose decision has been taken and published (high half); the largest depth of a reserved row
    Line64 td_rows;
    Line td_depth;
    // priority variant of the ready scheduler: sum of all nodes' (capped) distances from their roots, and the
    // critical / other seeds placed so far
    Line64 depth_sum;
    Line seed_front;
    Line seed_back;
    // grid barrier of the level scheduler, one word per L2 domain: arrivals of the domain's workgroups in
    // the low half, ready-queue records they have appended (cumulative) in the high half
    Line64 bar_xcd[N_XCD];
    // large grids add a second level: arrivals of whole domains, and a flag per domain that the last
    // arrival raises (barrier number in the low half, length of the ready queue in the high half)
    Line bar_all;
    Line64 bar_flag[N_XCD];
};

// Mailbox of one gang: a scheduler workgroup plus workgroups that together cover all column
// groups of a tile.  The scheduler posts tiles into a ring of GANG_RING slots.  A slot holds, for
// each of the TILE_ROWS rows, the node index and its two source rows, every entry tagged with the
// tile's sequence number and row count: tag << 32 | value, tag = sequence << 8 | rows.  An entry
// is valid for tile number q exactly when its tag says so, so that a reader needs no separate
// "published" flag and may request the entry before it is known to be there.
constexpr int GANG_RING = 2;
constexpr int SLOT_ENTRIES = 3 * TILE_ROWS;
constexpr int VALUE_EXIT = -2;            // node value of row 0 in the "leave" message
struct alignas(LINE) GangBox {
    unsigned long long slot[GANG_RING][SLOT_ENTRIES];   // [0,64): node  [64,128): first source  [128,192): second source
    // compute workgroups that have finished the tiles of each ring slot (cumulative per slot).  One counter
    // for the whole ring would not do: a fast member's count for the tile after would stand in for a
    // slow member's count for this one.
    Line done[GANG_RING];
};

// Record of the ready queue: a node that has become ready, with its child rows, so that whoever
// takes it off the queue needs one memory round trip, not two.  Two 8-byte words, each written
// by one store: {node + 1, left} and {right, node + 1}; a record whose two tags agree and are not
// zero is complete (the queue is zeroed at the start of every forward).
struct QRec {
    unsigned long long lo, hi;
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
    unsigned short *hb;         // bf16 copy of h for the bf16 weight-stationary cell (row stride hs, pads zero); else null
    int hs;
    float *h_root, *c_root;
    int32_t *root_out;
    // model
    int cell, H, E, vocab, n_cg, bf16;
    const float *emb;           // fp32 embedding table (as given)
    const unsigned short *embb; // bf16 copy, rows of es elements (zero padded), for the bf16 weight-stationary leaf kernel
    int es;
    Gemm leaf, inner;
    // workspace
    int32_t *parent, *pending, *leaf_list, *root_ws;
    int32_t *height, *arrive, *level_cnt, *level_off, *level_fill, *level_nodes;
    int32_t *depth_root;              // priority scheduling: distance of every node from its root, capped
    float *rntn_part;                 // RNTN: parts of the sums over q, [unit][column group][part][64 rows x 16], see cell_rntn.hpp
    unsigned int *rntn_done;          // RNTN: parts finished per unit and column group (back at zero after every tile)
    int rntn_units;                   // units the two arrays have room for
    int priority;                     // ready scheduler: critical path first
    QRec *q_rec;                      // ready queue, append-only: one record per internal node
    GangBox *gangs;
    const float *zeros;               // 256 bytes of zeros (stand-in source for padded operand granules)
    Ctl *ctl;
    // backward pass only (null / zero in a forward)
    float *gates;                     // null, or [n_nodes x 5H]: gate activations kept by the forward for the backward pass
    float *dh, *dc;                   // [n_nodes x H]: gradient arriving at each node's h and c
    float *dg;                        // rows of gate-pre-activation gradients: [n_int x 5H] or [n_leaf x 3H], by list position
    float *d_x;                       // [n_nodes x E] out: gradient of the embedding row each leaf used
    Gemm bwd;                         // packed transposed weights of the "gradient to the operand" contraction
    int pos0;                         // list position of the first node of the list a static launch works on
    int out_cols;                     // columns of the contraction a backward kernel produces (2H or E)
    int spin_limit;
    int cap_tiles;                    // tiles the launched grid can work on at once
    int n_gangs, gang_size;           // ready scheduler: grid = n_gangs * gang_size compute + n_gangs scheduler workgroups
    // data-flow scheduler: per column group a counter of handed-out children per node [n_cg x n_nodes] and a list of
    // ready nodes {node, left, right, 0} [n_cg x n_int]; a workgroup uses the part that belongs to its slot's trees
    int32_t *flow_seen;
    int4 *flow_list;
    int flow_roots;                   // data-flow scheduler: roots are found and their states copied out by the cell kernels (no separate passes)
    int flow;                         // data-flow scheduler: who fills the rows of internal nodes with the "not written" pattern: 1 the reset kernel, 2 the leaf kernel
    int gang_parts;                   // ready scheduler, RNTN cell: workgroups per tile and column group (each adds up a part of the slices), 1 or RNTN_PARTS
    int pick;                         // batch of few large trees, both internal-node kernels launched: 1 this one runs if the trees are narrow, 2 if they are not (see internal_kernel_skipped)
};

// ---- device-scope accesses -------------------------------------------------------------
// Inside a persistent kernel data written by one workgroup is read by workgroups on other L2
// domains.  The L2s are not coherent with each other, so such data is written with
// device-scope write-through stores and read with device-scope loads (relaxed agent-scope
// atomics compile to exactly these: global_store/global_load with the sc1 bit), and a writer
// waits for its stores to be acknowledged (s_waitcnt) before it signals.  This avoids
// whole-L2 write-back / invalidate fences, which cost tens of microseconds under load.
template <typename T> __device__ inline T ld_dev(const T *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T> __device__ inline void st_dev(T *p, T v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T> __device__ inline T add_dev(T *p, T v)
{
    return __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T> __device__ inline bool cas_dev(T *p, T *expected, T desired)
{
    return __hip_atomic_compare_exchange_strong(p, expected, desired, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                                __HIP_MEMORY_SCOPE_AGENT);
}
// All earlier loads and stores of this wave have completed (stores: acknowledged by memory).
__device__ inline void wait_mem()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // compiler: keep earlier accesses before this point
    __builtin_amdgcn_s_waitcnt(0);
}

// bf16 (round to nearest even, done by the hardware conversion) of one value, as its 16 bits
__device__ inline unsigned short bf16_bits(float x)
{
    const __bf16 b = (__bf16)x;
    return __builtin_bit_cast(unsigned short, b);
}
template <bool COH> __device__ inline void st_h(unsigned short *p, unsigned short v)
{
    if (COH) st_dev(p, v); else *p = v;
}
template <bool COH> __device__ inline float ld_f(const float *p) { return COH ? ld_dev(p) : *p; }
template <bool COH> __device__ inline void st_f(float *p, float v)
{
    if (COH) st_dev(p, v); else *p = v;
}
// 16-byte aligned 4-float load
template <bool COH> __device__ inline floatx4 ld_f4(const float *p)
{
    if (!COH) return *reinterpret_cast<const floatx4 *>(p);
    const unsigned long long *q = reinterpret_cast<const unsigned long long *>(p);
    const unsigned long long a = ld_dev(q), b = ld_dev(q + 1);
    floatx4 v;
    v.x = __uint_as_float((unsigned)a);
    v.y = __uint_as_float((unsigned)(a >> 32));
    v.z = __uint_as_float((unsigned)b);
    v.w = __uint_as_float((unsigned)(b >> 32));
    return v;
}

// Rows of a table smaller than 4 GiB addressed as a raw buffer: a 32-bit byte offset per lane and the base in scalar
// registers, where a pointer per lane costs two vector registers and 64-bit arithmetic.  COH: device scope (the
// cache-policy bit that the device-scope loads and stores above carry as well).
__device__ inline __amdgpu_buffer_rsrc_t buf_of(const void *p, unsigned long long bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, p ? (unsigned)bytes : 0u, 0x00020000);
}
template <bool COH> __device__ inline float buf_ld_f(__amdgpu_buffer_rsrc_t r, unsigned off)
{
    return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, (int)off, 0, COH ? 16 : 0));
}
template <bool COH> __device__ inline void buf_st_f(__amdgpu_buffer_rsrc_t r, unsigned off, float v)
{
    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), r, (int)off, 0, COH ? 16 : 0);
}
template <bool COH> __device__ inline void buf_st_h(__amdgpu_buffer_rsrc_t r, unsigned off, unsigned short v)
{
    __builtin_amdgcn_raw_buffer_store_b16(v, r, (int)off, 0, COH ? 16 : 0);
}

__device__ inline unsigned long long pack2(unsigned lo32, unsigned hi32) { return (unsigned long long)hi32 << 32 | lo32; }
template <bool COH> __device__ inline void qrec_store(QRec *q, int node, int left, int right)
{
    const unsigned long long lo = pack2((unsigned)node + 1u, (unsigned)left), hi = pack2((unsigned)right, (unsigned)node + 1u);
    if (COH) { st_dev(&q->lo, lo); st_dev(&q->hi, hi); } else { q->lo = lo; q->hi = hi; }
}
// Device-scope read; false while the record is not (completely) there.
__device__ inline bool qrec_load(const QRec *q, int *node, int *left, int *right)
{
    const unsigned long long lo = ld_dev(&q->lo), hi = ld_dev(&q->hi);
    const unsigned tag = (unsigned)lo;
    *node = (int)tag - 1;
    *left = (int)(unsigned)(lo >> 32);
    *right = (int)(unsigned)hi;
    return tag != 0u && (unsigned)(hi >> 32) == tag;
}

__device__ inline void latch_error(Ctl *ctl, int code)
{
    int expected = 0;
    cas_dev(&ctl->status, &expected, code);
}

// After the structure pass: has it found anything wrong?  (A tree without a root shows as a root count
// below the number of trees; every other defect has been latched in status.)
// (Where the cell kernels look after the roots themselves, the root count is not taken beforehand; what must hold
// before any cell runs is that the leaf list is complete.)
__device__ inline bool batch_rejected(const Fwd &f)
{
    return f.ctl->status != 0 || (f.flow_roots ? f.ctl->n_leaf_seen != f.n_leaf : f.ctl->n_roots != f.n_trees);
}

__device__ inline void backoff() { __builtin_amdgcn_s_sleep(2); }

// A batch of fewer trees than the device has sets of workgroups, of large trees: the data-flow scheduler keeps a tree on
// one set, which is the faster way if the trees are deep and narrow (a step costs a round trip, not a barrier) and
// the slower one by the number of idle sets if they are bushy.  The host does not know the shapes; the structure pass
// does: the internal nodes over two leaves are the first frontier, and if that has no more than 16 rows per tree a
// tree's ready nodes fit the blocks of one set anyway.  Both kernels are launched and every workgroup takes the same
// decision from that count (n_seed, final since the root pass).
constexpr int FLOW_NARROW_SEEDS_PER_TREE = 16;
__device__ inline bool internal_kernel_skipped(const Fwd &f)
{
    if (f.pick == 0) return false;
    const bool narrow = (long long)f.ctl->n_seed <= (long long)FLOW_NARROW_SEEDS_PER_TREE * f.n_trees;
    return f.pick == 1 ? !narrow : narrow;
}

// Rows per tile when `avail` ready rows meet room for `free_tiles` more tiles: spread the rows
// over the free room in units of 16, at most TILE_ROWS.
__host__ __device__ inline int tile_rows_for(unsigned avail, unsigned free_tiles)
{
    if (avail == 0) return 0;
    if (free_tiles == 0) free_tiles = 1;
    unsigned per = (avail + free_tiles - 1) / free_tiles;
    unsigned m = (per + 15u) & ~15u;
    if (m < 16u) m = 16u;
    if (m > (unsigned)TILE_ROWS) m = TILE_ROWS;
    return (int)(m < avail ? m : avail);
}

// How one height's rows are cut into tiles for a grid with room for `cap` tiles at a time:
// whole rounds of full tiles first, then the remainder spread evenly over one more round in
// smaller tiles (a tile of <= 16 / <= 32 rows takes a quarter / half of a full tile's time).
struct LevelPlan {
    int n_full;     // tiles of TILE_ROWS rows
    int m_rem;      // rows per remainder tile
    int n_tiles;    // all tiles
};
__host__ __device__ inline LevelPlan plan_level(int rows, int cap)
{
    LevelPlan p;
    if (cap < 1) cap = 1;
    p.n_full = rows / TILE_ROWS / cap * cap;
    const int rem = rows - p.n_full * TILE_ROWS;
    p.m_rem = rem > 0 ? tile_rows_for((unsigned)rem, (unsigned)cap) : TILE_ROWS;
    p.n_tiles = p.n_full + (rem + p.m_rem - 1) / p.m_rem;
    return p;
}
__host__ __device__ inline void plan_tile(const LevelPlan &p, int rows, int tile, int *start, int *count)
{
    if (tile < p.n_full) {
        *start = tile * TILE_ROWS;
        *count = TILE_ROWS;
    } else {
        *start = p.n_full * TILE_ROWS + (tile - p.n_full) * p.m_rem;
        const int left = rows - *start;
        *count = left < p.m_rem ? left : p.m_rem;
    }
}

// Column group of member j of a gang of `gang_size` workgroups, pass i (a workgroup covers the
// column groups j, j + gang_size, ... when there are more column groups than gang members).
// Consecutive workgroups sit on consecutive L2 domains; when the count allows it, each domain
// is given a contiguous range of column groups so that its slice of the weights stays in its L2
// and neighbouring 64-byte pieces of an output row are written from the same L2.
__host__ __device__ inline int gang_cg(int j, int gang_size, int n_cg)
{
    if (gang_size == n_cg && n_cg % N_XCD == 0) return (j % N_XCD) * (n_cg / N_XCD) + j / N_XCD;
    return j;
}

}  // namespace tl
