// Weight-stationary form of the fused cell, for persistent kernels.
//
// Every internal node of every tree multiplies the same matrix U (Figure 2: one LSTM cell
// re-used at every recursive call).  A persistent workgroup therefore owns one column group of
// HU hidden units for the whole forward and keeps its slice of U in registers: the K axis is
// split between the four waves, and each wave holds SPW k-steps x NG gates of MFMA B operands
// (up to 16 x 5 x 4 = 320 VGPRs of the 512 a wave may use when one wave per SIMD is resident).
// The weights are read from memory once per forward instead of once per tile, which removes the
// L2 -> CU traffic that bounds small tiles, and a 16-row block costs SPW x NG x 4 MFMAs of
// latency however few rows are ready.
//
// Per block of 16 rows a wave
//   1. has requested its K range of the 16 gathered child rows one block earlier, with loads in
//      which consecutive lanes read consecutive 16 bytes of a row (a lane-per-row gather in MFMA
//      operand order costs one memory transaction per lane and throttles instruction issue);
//   2. parks them in its private LDS region and reads them back in MFMA operand order;
//   3. runs SPW x NG x 4 MFMAs on LDS-fed A and register-resident B operands;
//   4. meets the other three waves' partial sums in LDS and finishes four of the sixteen rows
//      (gate functions, c update, h/c stores).
//
// The summation order of a node is the one every data path uses (cell_tile.hpp, ksplit_reduce):
// wave w walks quarter w of the K axis in order, and the four quarter sums are added in wave
// order.  A node's result therefore does not depend on which rows happened to share its tile, on
// the scheduler, or on whether this form or the streaming form evaluated it.
#pragma once

#include <cstddef>

#include "cell_tile.hpp"

namespace tl {

constexpr int WS_MAX_SPW = 16;
constexpr int WS_RED_FLOATS = 4 * MAX_GATES * 4 * 64;     // one reduction buffer: [wave][gate][v][lane]
constexpr int WS_TABLE_ROWS = 256;                        // rows one call can take (a power of two)
constexpr int FLOW_ROOTS_KEPT = 192;                      // roots of a slot's trees that are remembered in LDS (more: found again by a second pass)
constexpr int FLOW_NXT_ROWS = 64;                         // rows of the next piece that the data-flow scheduler keeps in LDS

// LDS of the kernels that use this cell with SPW k-steps per wave.
template <int SPW> struct WsSmemT {
    static constexpr int A_LD = STEP_K * SPW + 4;   // LDS row stride of a wave's A block, floats
    float a[4][16 * A_LD];             // per wave: its K range of the block's 16 gathered rows
    float red[2][WS_RED_FLOATS];       // K-split partial sums, alternating per block
    int node[WS_TABLE_ROWS];           // row tables as in TileSmem, for up to WS_TABLE_ROWS rows
    int src0[WS_TABLE_ROWS];
    int src1[WS_TABLE_ROWS];
    int par[WS_TABLE_ROWS];            // data-flow scheduler: parent of each row's node (-1: none)
    int nxt[4][FLOW_NXT_ROWS];         // ... and the four tables of the piece after the current one, when that is a small one
    int roots[FLOW_ROOTS_KEPT];        // ... and the roots among the slot's nodes
    int cmd[8];
};

constexpr int WS_VGPR_STEPS = 5;   // k-steps whose weights stay in the vector registers when not all fit (see ws_load)
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
    // A wave has 256 vector registers and 256 accumulation registers; an MFMA takes its B operand from either
    // file.  With more weights than fit beside everything else in the first file, say which of them live in the
    // second: left to itself the compiler parks them there as well, but copies each back before its MFMA,
    // one vector instruction per MFMA operand and block.
    if constexpr (SPW * NG * 4 > 256) {
#pragma unroll
        for (int s = WS_VGPR_STEPS; s < SPW; ++s)
#pragma unroll
            for (int g = 0; g < NG; ++g)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float x = w.b[s][g][i];
                    asm volatile("" : "+a"(x));             // no instruction: a register-class constraint only
                    w.b[s][g][i] = x;
                }
    }
}

// Geometry of the coalesced row loads of one wave: its K range is 16*SPW floats = LPR lanes of
// 16 bytes; RPL rows fit into one 64-lane load; NL loads cover the 16 rows of a block.
template <int SPW> struct WsLoadGeom {
    static constexpr int LPR = 4 * SPW;
    static constexpr int RPL = 64 / LPR;
    static constexpr int NL = (16 + RPL - 1) / RPL;
};

// Requests of this wave's K range of 16 rows of the tile, with consecutive lanes on consecutive
// 16 bytes of a row.  T is the element type of the table the rows come from: float (16 elements
// per k-step) or 16-bit (bf16 rows, 32 elements per k-step); either way a k-step is 64 bytes of a
// row = 4 lanes.  A request is one 32-bit multiply-add (row * row bytes + this lane's offset in
// the row) and a load from a uniform base.  Lanes on the K padding meet zero weights; they
// re-read the last 16 bytes of the same row, which hold finite values (0 * garbage could be
// NaN).  Rows that do not exist (-1 in the row table) read row 0 instead: every MFMA output row
// depends on its own A row only, and the results of such rows are never stored.
// The caller guarantees rows < 2^24 and table bytes < 2^32.
// TAIL: fp32 rows whose length is even but not a multiple of 4 (so rows are 8-byte, not 16-byte
// aligned, which the two 8-byte loads of a device-scope request tolerate).  The last request of
// a row then covers two elements of the row and two of whatever follows it in memory; the lanes
// concerned take their second 8 bytes from a block of zeros instead.
template <int SEG, int SPW, typename T = float, bool TAIL = false> struct WsRowRequest {
    using G = WsLoadGeom<SPW>;
    static constexpr int EPL = 16 / (int)sizeof(T);             // elements per lane and load
    const char *table;
    const int *src;                                             // row table of this lane's segment (LDS)
    unsigned lane_off, row_bytes;
    int sub;
    unsigned off[G::NL];
    const char *hi_base;                                        // TAIL only: where the second 8 bytes come from
    unsigned hi_mask;
    __amdgpu_buffer_rsrc_t rsrc;                                // the table as a raw buffer (device-scope requests)

    // rows of `table` are `stride` elements apart; what a row holds between its data and `stride`
    // elements reads as zero
    template <typename Smem>
    __device__ inline void init(const Smem &sm, const Fwd &f, const T *__restrict__ table_, int table_rows, int Lp, int stride,
                                int wave, int lane)
    {
        table = reinterpret_cast<const char *>(table_);
        // the whole table; the caller guarantees that it is smaller than 4 GiB
        rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<T *>(table_), 0, (unsigned)table_rows * (unsigned)stride * (unsigned)sizeof(T),
                                                 0x00020000);
        sub = lane / G::LPR;                                    // which of the RPL rows of a load
        const int k = 4 * EPL * SPW * wave + (lane % G::LPR) * EPL;   // position on the padded K axis
        const int seg = (SEG == 2 && k >= Lp) ? 1 : 0;
        const int o = min(k - seg * Lp, (stride - EPL + 3) & ~3);
        if constexpr (SEG == 2) src = seg ? sm.src1 : sm.src0;
        else src = sm.src0;
        lane_off = (unsigned)o * (unsigned)sizeof(T);
        row_bytes = (unsigned)stride * (unsigned)sizeof(T);
        const bool tail = TAIL && o + EPL > stride;
        hi_base = tail ? reinterpret_cast<const char *>(f.zeros) : table + 8;
        hi_mask = tail ? 0u : ~0u;
    }
    // byte offsets of the requests of block [row0, row0 + 16): one batch of row-table reads
    __device__ inline void prepare(int row0)
    {
#pragma unroll
        for (int j = 0; j < G::NL; ++j) {
            const int row = (row0 + j * G::RPL + sub) & (WS_TABLE_ROWS - 1);
            off[j] = __umul24((unsigned)src[row], row_bytes) + lane_off;     // the tables hold row 0 for rows that do not exist
        }
    }
    template <bool COH> __device__ inline floatx4 issue(int j) const
    {
        if constexpr (!TAIL && COH) {
            // one 16-byte device-scope load (buffer_load_dwordx4 ... sc1)
            typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
            const uintx4 u = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)off[j], 0, 16);
            floatx4 v;
            v.x = __uint_as_float(u.x);
            v.y = __uint_as_float(u.y);
            v.z = __uint_as_float(u.z);
            v.w = __uint_as_float(u.w);
            return v;
        } else if constexpr (!TAIL) {
            return ld_f4<COH>(reinterpret_cast<const float *>(table + off[j]));
        } else {
            static_assert(sizeof(T) == 4, "tail handling is for fp32 rows");
            const unsigned long long a = ld_dev(reinterpret_cast<const unsigned long long *>(table + off[j]));
            const unsigned long long b = ld_dev(reinterpret_cast<const unsigned long long *>(hi_base + (off[j] & hi_mask)));
            floatx4 v;
            v.x = __uint_as_float((unsigned)a);
            v.y = __uint_as_float((unsigned)(a >> 32));
            v.z = __uint_as_float((unsigned)b);
            v.w = __uint_as_float((unsigned)(b >> 32));
            return v;
        }
    }
};

// Lane J of every group of four lanes, to all four.
template <int J> __device__ inline float quad_bcast(float x)
{
    return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(x), J * 0x55, 0xF, 0xF, true));
}

// ---- validity carried by the data itself (data-flow scheduler) -----------------------------
// Before the kernel starts, every row that an internal node will produce (its c row and the h row
// its parent gathers) is filled with a bit pattern that no cell ever stores: all ones, a NaN (h
// and c are finite whenever the parameters and embeddings are).  A consumer requests a child's
// row whenever it likes and looks at what arrives: a 16-byte piece that still shows the pattern in
// any of its elements has not been written (completely) yet, and the request is repeated.  No
// flag, counter or barrier stands between the producer's store and the consumer's load, and the
// producer does not wait for its stores to be acknowledged.  A row is written in pieces by the
// workgroups of several column groups and an element by one store, so every element is checked.
constexpr unsigned FLOW_SENTINEL = 0xFFFFFFFFu;             // fp32; a bf16 element shows 0xFFFF

template <typename T> __device__ inline unsigned flow_fold(unsigned m, const floatx4 &v)
{
    const unsigned a = __float_as_uint(v.x), b = __float_as_uint(v.y), c = __float_as_uint(v.z), d = __float_as_uint(v.w);
    if constexpr (sizeof(T) == 4) {
        return max(max(m, a), max(max(b, c), d));
    } else {
        typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));
        ushort2_t mm = __builtin_bit_cast(ushort2_t, m);
        mm = __builtin_elementwise_max(mm, __builtin_bit_cast(ushort2_t, a));
        mm = __builtin_elementwise_max(mm, __builtin_bit_cast(ushort2_t, b));
        mm = __builtin_elementwise_max(mm, __builtin_bit_cast(ushort2_t, c));
        mm = __builtin_elementwise_max(mm, __builtin_bit_cast(ushort2_t, d));
        return __builtin_bit_cast(unsigned, mm);
    }
}
template <typename T> __device__ inline bool flow_shows_sentinel(unsigned m)
{
    if constexpr (sizeof(T) == 4) return m == FLOW_SENTINEL;
    else return (m & 0xFFFFu) == 0xFFFFu || (m >> 16) == 0xFFFFu;
}
__device__ inline void flow_give_up(const Fwd &f)
{
    st_dev(&f.ctl->abort.v, 1u);
    latch_error(f.ctl, TL_ESTALL);
}
// The rows of one block (requested earlier, `req` still holds their offsets): repeats the requests until no piece
// this wave uses shows the pattern.  Bounded by the spin budget and the abort flag; returns false when it gave up.
template <typename T, bool COH, typename Req, int NL, int RPL>
__device__ inline bool flow_wait_rows(const Fwd &f, const Req &req, floatx4 (&rows)[NL], int sub)
{
    int spins = 0;
    unsigned aborted = 0u;
    for (;;) {
        unsigned m = 0u;
#pragma unroll
        for (int j = 0; j < NL; ++j)
            if (sub < RPL && j * RPL + sub < 16) m = flow_fold<T>(m, rows[j]);
        if (__ballot(flow_shows_sentinel<T>(m)) == 0ull) return true;
        if (++spins > f.spin_limit || aborted != 0u) {
            flow_give_up(f);
            return false;
        }
        backoff();
#pragma unroll
        for (int j = 0; j < NL; ++j) rows[j] = req.template issue<COH>(j);
        aborted = ld_dev(&f.ctl->abort.v);                  // arrives with the rows
    }
}
// One element of a child's c row.
template <bool COH> __device__ inline float flow_wait_c(const Fwd &f, __amdgpu_buffer_rsrc_t rs_c, unsigned off, float v)
{
    int spins = 0;
    while (__float_as_uint(v) == FLOW_SENTINEL) {
        if (++spins > f.spin_limit || ((spins & 63) == 0 && ld_dev(&f.ctl->abort.v) != 0u)) {
            flow_give_up(f);
            break;
        }
        backoff();
        v = buf_ld_f<COH>(rs_c, off);
    }
    return v;
}

// Parks requested rows in the wave's LDS region (row-major, stride Smem::A_LD).
template <int SPW, typename Smem>
__device__ inline void ws_park_rows(Smem &sm, const floatx4 (&regs)[WsLoadGeom<SPW>::NL], int wave, int lane)
{
    using G = WsLoadGeom<SPW>;
    const int sub = lane / G::LPR, kk = (lane % G::LPR) * 4;
#pragma unroll
    for (int j = 0; j < G::NL; ++j) {
        const int r = j * G::RPL + sub;
        if (sub < G::RPL && r < 16) *reinterpret_cast<floatx4 *>(&sm.a[wave][r * Smem::A_LD + kk]) = regs[j];
    }
}

// The row tables of this cell: sm.node holds -1 for rows that do not exist, sm.src0 / sm.src1 hold
// row 0 for them (so that a request needs no test).
// Evaluates the `count` <= WS_TABLE_ROWS rows in sm.node/src0/src1 for column group cg, 16 at a
// time, the requests of a block's rows always one block ahead.  All four waves call it together;
// a __syncthreads() has been passed since the row tables were written.
// `hook` lets the caller do memory work of its own beside the cell's, at points where waiting for what it requested
// earlier costs nothing: it is called with -1 once the first row requests are out, with rb when the rows of block rb
// have arrived and been parked, and with -2 after the last block's matrix instructions, before its rows are finished.
struct WsNoHook {
    __device__ inline void operator()(int) const {}
};
// Top-down generation, data-flow form (EPI_TD_CHILD with FLOW): a row of sm.node may hold WS_ROW_PENDING instead of the
// child's row: the parent (sm.src0) has been reserved but whether it gets children is not known yet.  Its contraction is
// computed all the same, and when the row is finished the hook says where the result goes: ahead_of(tile row) is what
// it asked for when the block's rows arrived, ask(parent) asks again; `undecided` is the answer "not known yet", -1 means
// no children, any other value is the left child's row, `side` is added for this workgroup's child.
constexpr int WS_ROW_PENDING = -3;
template <int EPI, bool COH, int SPW, bool TAIL = false, bool FLOW = false, typename Hook = WsNoHook>
__device__ inline void ws_tile(WsSmemT<SPW> &sm, const Fwd &f, const Gemm &gm, const float *__restrict__ table, int table_rows,
                               int count, int cg, const WsWeights<EpiTraits<EPI>::NG, SPW> &w, Hook hook = Hook())
{
    constexpr int NG = EpiTraits<EPI>::NG;
    constexpr int SEG = EpiTraits<EPI>::SEG;
    constexpr int NL = WsLoadGeom<SPW>::NL;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nrb = (count + 15) >> 4;
    const int H = f.H;
    const int hu = cg * HU + (lane & 15);
    const bool hu_ok = hu < H;
    const float *a_lane = &sm.a[wave][(lane & 15) * WsSmemT<SPW>::A_LD + (lane >> 4) * 4];   // + 16 s: this lane's operand of k-step s
    // h and c rows as raw buffers (the caller guarantees that they are smaller than 4 GiB)
    const __amdgpu_buffer_rsrc_t rs_h = buf_of(f.h, (unsigned long long)f.n_nodes * H * 4), rs_c = buf_of(f.c, (unsigned long long)f.n_nodes * H * 4);
    const unsigned row_b = (unsigned)H * 4u, hu_b = (unsigned)(hu_ok ? hu : 0) * 4u;

    // Second half of a block: the four K-range partial sums have met in LDS (a barrier has been
    // passed since they were written); wave w finishes accumulator row w of the block.
    auto finish = [&](const float *red, int enode, bool ev, float cl, float cr, int erow) {
        float gate[NG];
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            float sum = red[((0 * NG + g) * 4 + wave) * 64 + lane];
            sum += red[((1 * NG + g) * 4 + wave) * 64 + lane];
            sum += red[((2 * NG + g) * 4 + wave) * 64 + lane];
            sum += red[((3 * NG + g) * 4 + wave) * 64 + lane];
            gate[g] = sum + w.bias[g];
        }
        if constexpr (FLOW && EPI == EPI_TD_CHILD) {
            // The result of a row is stored the moment its own decision is known: a lane never holds a decided row back
            // while it waits for another row's decision (whoever decides that one may be waiting for this store).
            const bool pending = enode == WS_ROW_PENDING && hu_ok;
            if (ev || pending) {
                cl = flow_wait_c<COH>(f, rs_c, (unsigned)sm.src0[erow & (WS_TABLE_ROWS - 1)] * row_b + hu_b, cl);   // the parent's c element may arrive after its h row
                const float i = sigmoid_f(gate[0]), fg = sigmoid_f(gate[1]), og = sigmoid_f(gate[2]), u = tanh_f(gate[3]);
                const float cc = __builtin_fmaf(fg, cl, i * u);
                const float hh = og * tanh_f(cc);
                int child = pending ? hook.ahead_of(erow) : enode;
                bool open = true;
                // (The loop condition is the same for all lanes of the wave on purpose.  A loop that each lane leaves on its
                // own is compiled into one whose lanes meet again behind it, with the stores moved there: the coupling this
                // is meant to avoid.)
                for (int spins = 0;; ++spins) {
                    if (open && child != hook.undecided) {
                        if (child >= 0) {
                            const unsigned o = (unsigned)(pending ? child + hook.side : child) * row_b + hu_b;
                            buf_st_f<COH>(rs_c, o, cc);
                            buf_st_f<COH>(rs_h, o, hh);
                        }
                        open = false;
                    }
                    if (__ballot(open) == 0ull) break;
                    if (spins > f.spin_limit || ((spins & 63) == 63 && ld_dev(&f.ctl->abort.v) != 0u)) {
                        if (open) flow_give_up(f);
                        break;
                    }
                    backoff();
                    if (open) child = hook.ask(sm.src0[erow & (WS_TABLE_ROWS - 1)]);
                }
            }
            return;
        }
        if (ev) {
            const unsigned o = (unsigned)enode * row_b + hu_b;
            if constexpr (FLOW && EPI == EPI_LSTM_INNER) {      // a child's c element may arrive after its h row
                cl = flow_wait_c<COH>(f, rs_c, (unsigned)sm.src0[erow & (WS_TABLE_ROWS - 1)] * row_b + hu_b, cl);
                cr = flow_wait_c<COH>(f, rs_c, (unsigned)sm.src1[erow & (WS_TABLE_ROWS - 1)] * row_b + hu_b, cr);
            }
            if constexpr (EPI == EPI_LSTM_INNER) {
                float cc, hh;
                lstm_inner_out(gate[0], gate[1], gate[2], gate[3], gate[NG - 1], cl, cr, &cc, &hh, kept_gates(f, enode, hu), H);
                buf_st_f<COH>(rs_c, o, cc);
                buf_st_f<COH>(rs_h, o, hh);
            } else if constexpr (EPI == EPI_LSTM_LEAF) {
                float cc, hh;
                lstm_leaf_out(gate[0], gate[1], gate[NG - 1], &cc, &hh, kept_gates(f, enode, hu), H);
                buf_st_f<COH>(rs_c, o, cc);
                buf_st_f<COH>(rs_h, o, hh);
            } else if constexpr (EPI == EPI_TD_CHILD) {     // gates i, f, o, u of an LSTM step along the edge (as in cell_tile.hpp)
                const float i = sigmoid_f(gate[0]), fg = sigmoid_f(gate[1]), og = sigmoid_f(gate[2]), u = tanh_f(gate[3]);
                const float cc = __builtin_fmaf(fg, cl, i * u);
                buf_st_f<COH>(rs_c, o, cc);
                buf_st_f<COH>(rs_h, o, og * tanh_f(cc));
            } else {
                buf_st_f<COH>(rs_h, o, tanh_f(gate[0]));
            }
        }
    };

    WsRowRequest<SEG, SPW, float, TAIL> req;
    req.init(sm, f, table, table_rows, gm.Lp, gm.L, wave, lane);
    floatx4 rows[NL];
    req.prepare(0);
#pragma unroll
    for (int j = 0; j < NL; ++j) rows[j] = req.template issue<COH>(j);
    hook(-1);
    // The second half of block rb - 1 is done inside the MFMA phase of block rb (after its first
    // k-step): what it waits for (the barrier, LDS round trips, the c rows) has then had a k-step
    // of MFMAs to arrive, instead of leaving the matrix pipe idle between two blocks.
    int p_enode = -1;
    bool p_ev = false;
    float p_cl = 0.f, p_cr = 0.f;
    int p_erow = 0;
    constexpr int FINISH_AFTER = SPW > 1 ? 1 : 0;               // k-step after which the previous block is finished
    // A piece's last block with few rows takes the narrow form below the loop (data-flow scheduler only).
    constexpr int NARROW_MAX_RG = NG >= 3 ? 3 : 2;              // groups of four rows up to which that form is the faster one
    const int n_rg = (count - (nrb - 1) * 16 + 3) >> 2;         // groups of four rows in the last block
    // (not in top-down generation: there the place of a node in a tile depends on timing, and its bits must not)
    const bool last_narrow = FLOW && EPI != EPI_TD_CHILD && nrb > 0 && n_rg <= NARROW_MAX_RG;
    const int nrb_full = last_narrow ? nrb - 1 : nrb;
    for (int rb = 0; rb < nrb_full; ++rb) {
        float *red = sm.red[rb & 1];
        if constexpr (FLOW) {                               // the rows are there only when their producers have stored them
            if (!flow_wait_rows<float, COH, WsRowRequest<SEG, SPW, float, TAIL>, NL, WsLoadGeom<SPW>::RPL>(f, req, rows, req.sub))
                sm.cmd[7] = 1;
        }
        ws_park_rows<SPW>(sm, rows, wave, lane);            // waits for the requested rows
        // the next block's rows are requested between the k-steps below, one row load per step: the
        // memory path of a CU takes a 1 KB request every ~160 cycles, a k-step lasts 640
        req.prepare((rb + 1) * 16);
        hook(rb);
        // the row this lane finishes after the reduction, and its c operands
        const int erow = rb * 16 + (lane >> 4) * 4 + wave;
        const int enode = erow < count ? sm.node[erow] : -1;
        const bool ev = enode >= 0 && hu_ok;
        float cl = 0.f, cr = 0.f;
        if (EPI == EPI_LSTM_INNER) {                        // unused lanes read some existing element; the value is dropped
            cl = buf_ld_f<COH>(rs_c, (unsigned)sm.src0[erow & (WS_TABLE_ROWS - 1)] * row_b + hu_b);
            cr = buf_ld_f<COH>(rs_c, (unsigned)sm.src1[erow & (WS_TABLE_ROWS - 1)] * row_b + hu_b);
        } else if (EPI == EPI_TD_CHILD) {                   // the parent's c (src0 = the parent's row)
            cl = buf_ld_f<COH>(rs_c, (unsigned)sm.src0[erow & (WS_TABLE_ROWS - 1)] * row_b + hu_b);
        }
        __builtin_amdgcn_sched_barrier(0);                  // all requests are issued before the MFMAs start
        floatx4 acc[NG];
#pragma unroll
        for (int g = 0; g < NG; ++g) acc[g] = floatx4{0.f, 0.f, 0.f, 0.f};
        constexpr int LOADS_PER_STEP = (NL + SPW - 1) / SPW;
        // the A operand of a k-step is read from LDS one k-step ahead, so that its latency runs under MFMAs
        floatx4 av_next = *reinterpret_cast<const floatx4 *>(a_lane);
#pragma unroll
        for (int s = 0; s < SPW; ++s) {
            const floatx4 av = av_next;
            if (s + 1 < SPW) av_next = *reinterpret_cast<const floatx4 *>(a_lane + (s + 1) * STEP_K);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int g = 0; g < NG; ++g)
                    acc[g] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[i], w.b[s][g][i], acc[g], 0, 0, 0);
#pragma unroll
            for (int q = 0; q < LOADS_PER_STEP; ++q)
                if (s * LOADS_PER_STEP + q < NL) rows[s * LOADS_PER_STEP + q] = req.template issue<COH>(s * LOADS_PER_STEP + q);
            __builtin_amdgcn_sched_barrier(0);              // keep the request where it is
            if (s == FINISH_AFTER && rb > 0) {
                __syncthreads();                            // every wave has written its partial sums of block rb - 1
                finish(sm.red[(rb - 1) & 1], p_enode, p_ev, p_cl, p_cr, p_erow);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // this block's partial sums go to LDS; they are picked up one block later (or after the loop)
#pragma unroll
        for (int g = 0; g < NG; ++g)
#pragma unroll
            for (int v = 0; v < 4; ++v) red[((wave * NG + g) * 4 + v) * 64 + lane] = acc[g][v];
        p_enode = enode;
        p_ev = ev;
        p_cl = cl;
        p_cr = cr;
        p_erow = erow;
        // the two reduction buffers alternate: buffer rb & 1 is written again at the end of block
        // rb + 2, after every wave has passed the barrier inside block rb + 2, hence after it has
        // read this buffer (inside block rb + 1)
    }
    if constexpr (FLOW) {
        // The 16x16x4 instruction takes 32 cycles however many of its 16 rows exist, and the dependent steps of a deep tree
        // are blocks of one to four rows.  The 4x4x1 instruction (16 independent 4x4 products, 8 cycles) takes the same B
        // operands - lane l holds U[k(l >> 4)][l & 15] - when its 16 products are read as (k class l >> 4) x (four hidden
        // units): with A = a[4 rg + (l & 3)][k(l >> 4)] it accumulates, for rows 4 rg .. 4 rg + 3, the sum over the k of
        // class l >> 4.  A group of four rows so costs a quarter of a block (measured: 4.1 ns per instruction against
        // 14.6), and the four class sums of a wave are added when the row is finished.  A node's sum is then rounded in
        // another order than in a full block; which form evaluates a node depends on its place in the list alone, which
        // does not change from run to run.
        if (last_narrow) {
            const int rb = nrb - 1;
            // Lane l of wave w finishes row w of a group of four rows for hidden unit l >> 2, from wave (l & 3)'s four class
            // sums; the four lanes of a quad then add theirs in wave order.  (What is computed from the lane number here starts
            // from a copy the compiler cannot see through: held in registers across the whole kernel, these few values made it
            // spill others in the loop above.)
            int nl = lane;
            asm volatile("" : "+v"(nl));
            const int n_hu = cg * HU + (nl >> 2);
            const bool n_hu_ok = n_hu < H;
            const unsigned n_hu_b = (unsigned)(n_hu_ok ? n_hu : 0) * 4u;
            auto finish_narrow = [&](const float *red, int enode, bool ev, float cl, float cr, int erow, const float (&bias)[NG]) {
                float gate[NG];
#pragma unroll
                for (int g = 0; g < NG; ++g) {
                    const floatx4 p = *reinterpret_cast<const floatx4 *>(&red[(((((nl & 3) * NG + g) * 4 + wave) * 16) + (nl >> 2)) * 4]);
                    const float q = ((p.x + p.y) + p.z) + p.w;
                    gate[g] = (((quad_bcast<0>(q) + quad_bcast<1>(q)) + quad_bcast<2>(q)) + quad_bcast<3>(q)) + bias[g];
                }
                if (ev) {
                    const unsigned o = (unsigned)enode * row_b + n_hu_b;
                    if constexpr (FLOW && EPI == EPI_LSTM_INNER) {
                        cl = flow_wait_c<COH>(f, rs_c, (unsigned)sm.src0[erow & (WS_TABLE_ROWS - 1)] * row_b + n_hu_b, cl);
                        cr = flow_wait_c<COH>(f, rs_c, (unsigned)sm.src1[erow & (WS_TABLE_ROWS - 1)] * row_b + n_hu_b, cr);
                    }
                    const bool writer = (nl & 3) == 0;               // the four lanes of a quad hold the same result
                    if constexpr (EPI == EPI_LSTM_INNER) {
                        float cc, hh;
                        lstm_inner_out(gate[0], gate[1], gate[2], gate[3], gate[NG - 1], cl, cr, &cc, &hh, writer ? kept_gates(f, enode, n_hu) : nullptr, H);
                        if (writer) {
                            buf_st_f<COH>(rs_c, o, cc);
                            buf_st_f<COH>(rs_h, o, hh);
                        }
                    } else if constexpr (EPI == EPI_LSTM_LEAF) {
                        float cc, hh;
                        lstm_leaf_out(gate[0], gate[1], gate[NG - 1], &cc, &hh, writer ? kept_gates(f, enode, n_hu) : nullptr, H);
                        if (writer) {
                            buf_st_f<COH>(rs_c, o, cc);
                            buf_st_f<COH>(rs_h, o, hh);
                        }
                    } else if constexpr (EPI == EPI_TD_CHILD) {
                        const float i = sigmoid_f(gate[0]), fg = sigmoid_f(gate[1]), og = sigmoid_f(gate[2]), u = tanh_f(gate[3]);
                        const float cc = __builtin_fmaf(fg, cl, i * u);
                        if (writer) {
                            buf_st_f<COH>(rs_c, o, cc);
                            buf_st_f<COH>(rs_h, o, og * tanh_f(cc));
                        }
                    } else {
                        if (writer) buf_st_f<COH>(rs_h, o, tanh_f(gate[0]));
                    }
                }
            };

            int n_enode = -1, n_erow = 0;
            bool n_ev = false;
            float n_cl = 0.f, n_cr = 0.f, n_bias[NG];
            // the row a lane finishes in group rg, and its c operands (a value that shows "not written" is asked for again
            // when the row is finished)
            auto request_c = [&](int rg) {
                n_erow = rb * 16 + rg * 4 + wave;
                n_enode = n_erow < count ? sm.node[n_erow] : -1;
                n_ev = n_enode >= 0 && n_hu_ok;
                if (EPI == EPI_LSTM_INNER) {
                    n_cl = buf_ld_f<COH>(rs_c, (unsigned)sm.src0[n_erow & (WS_TABLE_ROWS - 1)] * row_b + n_hu_b);
                    n_cr = buf_ld_f<COH>(rs_c, (unsigned)sm.src1[n_erow & (WS_TABLE_ROWS - 1)] * row_b + n_hu_b);
                } else if (EPI == EPI_TD_CHILD) {
                    n_cl = buf_ld_f<COH>(rs_c, (unsigned)sm.src0[n_erow & (WS_TABLE_ROWS - 1)] * row_b + n_hu_b);
                }
            };
            if (!flow_wait_rows<float, COH, WsRowRequest<SEG, SPW, float, TAIL>, NL, WsLoadGeom<SPW>::RPL>(f, req, rows, req.sub))
                sm.cmd[7] = 1;
            ws_park_rows<SPW>(sm, rows, wave, lane);
            hook(rb);
            request_c(0);
#pragma unroll
            for (int g = 0; g < NG; ++g) n_bias[g] = __shfl(w.bias[g], nl >> 2);
#pragma unroll 1
            for (int rg = 0; rg < n_rg; ++rg) {
                if (rg > 0) {
                    __syncthreads();                        // every wave has written its partial sums of group rg - 1
                    finish_narrow(sm.red[(rb + rg - 1) & 1], n_enode, n_ev, n_cl, n_cr, n_erow, n_bias);
                    request_c(rg);
                }
                __builtin_amdgcn_sched_barrier(0);
                floatx4 acc[NG];
#pragma unroll
                for (int g = 0; g < NG; ++g) acc[g] = floatx4{0.f, 0.f, 0.f, 0.f};
                const float *a4 = &sm.a[wave][(rg * 4 + (nl & 3)) * WsSmemT<SPW>::A_LD + (nl >> 4) * 4];
                floatx4 av_next = *reinterpret_cast<const floatx4 *>(a4);
#pragma unroll
                for (int s = 0; s < SPW; ++s) {
                    const floatx4 av = av_next;
                    if (s + 1 < SPW) av_next = *reinterpret_cast<const floatx4 *>(a4 + (s + 1) * STEP_K);
#pragma unroll
                    for (int i = 0; i < 4; ++i)
#pragma unroll
                        for (int g = 0; g < NG; ++g)
                            acc[g] = __builtin_amdgcn_mfma_f32_4x4x1f32(av[i], w.b[s][g][i], acc[g], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    if (s == FINISH_AFTER && rg == 0 && rb > 0) {
                        __syncthreads();                    // every wave has written its partial sums of block rb - 1
                        finish(sm.red[(rb - 1) & 1], p_enode, p_ev, p_cl, p_cr, p_erow);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                // [wave][gate][row][hidden unit][k class]: the four class sums of an element lie side by side
                float *nred = sm.red[(rb + rg) & 1];
#pragma unroll
                for (int g = 0; g < NG; ++g)
#pragma unroll
                    for (int v = 0; v < 4; ++v) nred[((((wave * NG + g) * 4 + v) * 16) + (nl & 15)) * 4 + (nl >> 4)] = acc[g][v];
            }
            hook(-2);
            __syncthreads();
            finish_narrow(sm.red[(rb + n_rg - 1) & 1], n_enode, n_ev, n_cl, n_cr, n_erow, n_bias);
            __syncthreads();
            return;
        }
    }
    hook(-2);
    __syncthreads();
    if (nrb > 0) finish(sm.red[(nrb - 1) & 1], p_enode, p_ev, p_cl, p_cr, p_erow);
    __syncthreads();                                        // row tables and LDS may be rewritten after this call
}

// ---------------------------------------------------------------------------------------
// bf16-operand form (v_mfma_f32_16x16x32_bf16, fp32 accumulate, gates and state).
//
// A wave holds S k-steps of 32 x NG gates = S * NG * 4 registers of bf16 weights: half the fp32
// form's, so two workgroups fit on a CU and one computes while the other waits for rows or
// finishes gates.  The MFMAs of a block take a fraction of a microsecond here; what a block
// costs is the gather of its child rows, so those come from a bf16 copy of h (written next to
// the fp32 h by every epilogue, rows padded with zeros to a multiple of 8 elements): half the
// bytes, no conversion on the way into LDS, and the rounding of the operand (once per element,
// to nearest even) is the same as converting at gather time.
constexpr int WSB_MAX_S = 8;

// What only cells of internal nodes need in LDS: the second source of a row, and the data-flow scheduler's tables (see
// WsSmemT).  The leaf kernel, which is bound by the latency of a block's phases and gains from every further resident
// workgroup, does without them and with reduction buffers for its three gates: four workgroups fit on a CU.
template <bool INNER_TABLES> struct WsFlowTables {
    int src1[WS_TABLE_ROWS];
    int par[WS_TABLE_ROWS];
    int nxt[4][FLOW_NXT_ROWS];
    int roots[FLOW_ROOTS_KEPT];
};
template <> struct WsFlowTables<false> {};
template <int S, int NGM = MAX_GATES, bool FLOW_TABLES = true> struct WsSmemBfT : WsFlowTables<FLOW_TABLES> {
    static constexpr int A_LD = 32 * S + 8;                // LDS row stride of a wave's A block, bf16 elements
    unsigned short a[4][16 * A_LD];
    float red[2][4 * NGM * 4 * 64];    // K-split partial sums, alternating per block: [wave][gate][v][lane]
    int node[WS_TABLE_ROWS];
    int src0[WS_TABLE_ROWS];
    float bias[NGM * HU];              // the column group's bias (ws_load puts it here: a load of it from memory after the barrier would
                                       // have to wait for the row requests issued before it, and registers are short in this form)
    int cmd[8];
};

template <int NG, int S> struct WsWeightsBf {
    bf16x8 b[S][NG];
};
template <int NG> struct WsWeightsBf<NG, 0> {};

// k-steps (of 32) [wave*S, (wave+1)*S) of column group cg; the packed matrix has exactly 4*S of them.
// Called by all threads of the workgroup; a barrier must be passed before the first ws_tile (its own first barrier
// comes before the bias is read).
template <int NG, int S, int NGM, bool FT>
__device__ inline void ws_load(WsWeightsBf<NG, S> &w, WsSmemBfT<S, NGM, FT> &sm, const Gemm &gm, int cg, int wave, int lane)
{
    const bf16x8 *wp = reinterpret_cast<const bf16x8 *>(gm.wp) + ((size_t)cg * 4 * S + (size_t)wave * S) * NG * 64 + lane;
    // the bias is requested first: its way into LDS then waits for nothing but itself (loads return in order)
    const int t = wave * 64 + lane;
    float bias = 0.f;
    if (t < NG * HU) bias = gm.bp[cg * NG * HU + t];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int s = 0; s < S; ++s)
#pragma unroll
        for (int g = 0; g < NG; ++g) w.b[s][g] = wp[(size_t)(s * NG + g) * 64];
    if (t < NG * HU) sm.bias[t] = bias;
}

template <int EPI, bool COH, int S, bool FLOW = false, typename Hook = WsNoHook, int NGM = MAX_GATES, bool FT = true>
__device__ inline void ws_tile(WsSmemBfT<S, NGM, FT> &sm, const Fwd &f, const Gemm &gm, const unsigned short *__restrict__ table,
                               int table_rows, int stride, int count, int cg, const WsWeightsBf<EpiTraits<EPI>::NG, S> &w,
                               Hook hook = Hook())
{
    constexpr int NG = EpiTraits<EPI>::NG;
    static_assert(NG <= NGM, "reduction buffers and bias of the LDS layout are sized for NGM gates");
    constexpr int SEG = EpiTraits<EPI>::SEG;
    using G = WsLoadGeom<S>;
    constexpr int NL = G::NL;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nrb = (count + 15) >> 4;
    const int H = f.H;
    const int hu = cg * HU + (lane & 15);
    const bool hu_ok = hu < H;
    const unsigned short *a_lane = &sm.a[wave][(lane & 15) * WsSmemBfT<S, NGM, FT>::A_LD + (lane >> 4) * 8];   // + 32 s: operand of k-step s
    // h, c and the bf16 copy of h as raw buffers (the caller guarantees that they are smaller than 4 GiB)
    const __amdgpu_buffer_rsrc_t rs_h = buf_of(f.h, (unsigned long long)f.n_nodes * H * 4), rs_c = buf_of(f.c, (unsigned long long)f.n_nodes * H * 4),
                                 rs_hb = buf_of(f.hb, (unsigned long long)f.n_nodes * f.hs * 2);
    const unsigned row_b = (unsigned)H * 4u, hu_b = (unsigned)(hu_ok ? hu : 0) * 4u, hb_row_b = (unsigned)f.hs * 2u;

    WsRowRequest<SEG, S, unsigned short> req;
    req.init(sm, f, table, table_rows, stride, stride, wave, lane);
    floatx4 rows[NL];
    req.prepare(0);
#pragma unroll
    for (int j = 0; j < NL; ++j) rows[j] = req.template issue<COH>(j);
    hook(-1);
    for (int rb = 0; rb < nrb; ++rb) {
        float *red = sm.red[rb & 1];
        if constexpr (FLOW) {                               // the rows are there only when their producers have stored them
            if (!flow_wait_rows<unsigned short, COH, WsRowRequest<SEG, S, unsigned short>, NL, G::RPL>(f, req, rows, req.sub))
                sm.cmd[7] = 1;
        }
        {                                                   // park the requested rows (waits for them)
            const int sub = lane / G::LPR, kk = (lane % G::LPR) * 8;
#pragma unroll
            for (int j = 0; j < NL; ++j) {
                const int r = j * G::RPL + sub;
                if (sub < G::RPL && r < 16) *reinterpret_cast<floatx4 *>(&sm.a[wave][r * WsSmemBfT<S, NGM, FT>::A_LD + kk]) = rows[j];
            }
        }
        req.prepare((rb + 1) * 16);
        hook(rb);
        const int erow = rb * 16 + (lane >> 4) * 4 + wave;
        const int enode = erow < count ? sm.node[erow] : -1;
        const bool ev = enode >= 0 && hu_ok;
        // c operands of the row this lane finishes: requested before the MFMAs, used after them
        float cl = 0.f, cr = 0.f;
        if constexpr (EPI == EPI_LSTM_INNER) {
            cl = buf_ld_f<COH>(rs_c, (unsigned)sm.src0[erow & (WS_TABLE_ROWS - 1)] * row_b + hu_b);
            cr = buf_ld_f<COH>(rs_c, (unsigned)sm.src1[erow & (WS_TABLE_ROWS - 1)] * row_b + hu_b);
        }
        __builtin_amdgcn_sched_barrier(0);
        floatx4 acc[NG];
#pragma unroll
        for (int g = 0; g < NG; ++g) acc[g] = floatx4{0.f, 0.f, 0.f, 0.f};
        constexpr int LOADS_PER_STEP = (NL + S - 1) / S;
        bf16x8 av_next = *reinterpret_cast<const bf16x8 *>(a_lane);      // read one k-step ahead, as in the fp32 form
#pragma unroll
        for (int s = 0; s < S; ++s) {
            const bf16x8 av = av_next;
            if (s + 1 < S) av_next = *reinterpret_cast<const bf16x8 *>(a_lane + (s + 1) * 32);
#pragma unroll
            for (int g = 0; g < NG; ++g) acc[g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, w.b[s][g], acc[g], 0, 0, 0);
#pragma unroll
            for (int q = 0; q < LOADS_PER_STEP; ++q)
                if (s * LOADS_PER_STEP + q < NL) rows[s * LOADS_PER_STEP + q] = req.template issue<COH>(s * LOADS_PER_STEP + q);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int g = 0; g < NG; ++g)
#pragma unroll
            for (int v = 0; v < 4; ++v) red[((wave * NG + g) * 4 + v) * 64 + lane] = acc[g][v];
        if (rb == nrb - 1) hook(-2);
        __syncthreads();
        float gate[NG];
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            float sum = red[((0 * NG + g) * 4 + wave) * 64 + lane];
            sum += red[((1 * NG + g) * 4 + wave) * 64 + lane];
            sum += red[((2 * NG + g) * 4 + wave) * 64 + lane];
            sum += red[((3 * NG + g) * 4 + wave) * 64 + lane];
            gate[g] = sum + sm.bias[g * HU + (lane & 15)];
        }
        if (ev) {
            const unsigned o = (unsigned)enode * row_b + hu_b;
            float hh;
            if constexpr (FLOW && EPI == EPI_LSTM_INNER) {      // a child's c element may arrive after its h row
                cl = flow_wait_c<COH>(f, rs_c, (unsigned)sm.src0[erow & (WS_TABLE_ROWS - 1)] * row_b + hu_b, cl);
                cr = flow_wait_c<COH>(f, rs_c, (unsigned)sm.src1[erow & (WS_TABLE_ROWS - 1)] * row_b + hu_b, cr);
            }
            if constexpr (EPI == EPI_LSTM_INNER) {
                float cc;
                lstm_inner_out(gate[0], gate[1], gate[2], gate[3], gate[NG - 1], cl, cr, &cc, &hh);
                buf_st_f<COH>(rs_c, o, cc);
            } else if constexpr (EPI == EPI_LSTM_LEAF) {
                float cc;
                lstm_leaf_out(gate[0], gate[1], gate[NG - 1], &cc, &hh);
                buf_st_f<COH>(rs_c, o, cc);
            } else {
                hh = tanh_f(gate[0]);
            }
            buf_st_f<COH>(rs_h, o, hh);
            if (f.hb) buf_st_h<COH>(rs_hb, (unsigned)enode * hb_row_b + (hu_b >> 1), bf16_bits(hh));
        }
    }
    __syncthreads();
}

}  // namespace tl
