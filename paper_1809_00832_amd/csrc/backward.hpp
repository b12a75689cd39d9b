// Backward pass of the TreeLSTM forward (Section 4.2.2, recursive backpropagation): the gradient
// of a node's cell is applied to the node, then to its children, with the forward values of each
// node found by node index in the h / c rows.  Heights are walked from the roots down (a parent
// is always higher than its children), one pair of launches per height:
//   1. gate gradients: the forward contraction G = [h_l ; h_r] U + b is recomputed with the
//      streaming cell, and its epilogue turns (dh, dc, c, c_l, c_r, gates) into the gradient of
//      the five gate pre-activations (a row of 5H values per node, kept by list position) and
//      sends dc to the children; if the forward kept its gate activations, an elementwise
//      kernel does the same from those, without the contraction;
//   2. operand gradient: [dh_l ; dh_r] += dG U^T, the same streaming cell with the rows of dG as
//      the gathered operand and U^T as the packed weights; its epilogue adds the result to the
//      children's dh rows (every node has one parent, so plain read-modify-write).
// Leaves likewise (dG W_x^T gives the gradient of each leaf's embedding row).  The weight
// gradients dU = sum_n a_n^T dG_n, dW_x = sum_n x_n^T dG_n are two contractions over all nodes at
// the end (k_weight_grad), which also sums the columns of the dG rows it passes over (bias
// gradients).
#pragma once

#include "cell_tile.hpp"
#include "schedulers.hpp"

namespace tl {

// COH: the rows of dh that the operand gradient adds to are read by other workgroups of the same kernel (the
// persistent form below): device-scope accesses, as in the forward's persistent kernels.
template <int EPI, int NG, bool COH>
__device__ inline void bwd_epilogue(const TileSmem &sm, const Fwd &f, const Gemm &gm, const floatx4 (&acc)[NG], int rb,
                                    int count, int cg, int lane)
{
    const int col = cg * HU + (lane & 15);
    const int H = f.H;
    if constexpr (EPI == EPI_BWD_INNER_GATES || EPI == EPI_BWD_LEAF_GATES) {
        if (col >= H) return;
        float bias[NG];
#pragma unroll
        for (int g = 0; g < NG; ++g) bias[g] = gm.bp[(cg * NG + g) * HU + (lane & 15)];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int row = rb * 16 + (lane >> 4) * 4 + v;
            if (row >= count) continue;
            const int node = sm.node[row];
            if (node < 0) continue;
            const size_t o = (size_t)node * H + col;
            const float t = tanh_f(f.c[o]);
            const float dh = f.dh[o], dc = f.dc[o];
            float *dg = f.dg + (size_t)(sm.cmd[3] + row) * (NG * H) + col;
            if constexpr (EPI == EPI_BWD_INNER_GATES) {
                const int l = sm.src0[row], r = sm.src1[row];
                const float cl = f.c[(size_t)l * H + col], cr = f.c[(size_t)r * H + col];
                const float i = sigmoid_f(acc[0][v] + bias[0]), fl = sigmoid_f(acc[1][v] + bias[1]);
                const float fr = sigmoid_f(acc[2][v] + bias[2]), og = sigmoid_f(acc[3][v] + bias[3]);
                const float u = tanh_f(acc[4][v] + bias[4]);
                const float dct = dc + dh * og * (1.f - t * t);
                dg[0] = dct * u * i * (1.f - i);
                dg[H] = dct * cl * fl * (1.f - fl);
                dg[2 * H] = dct * cr * fr * (1.f - fr);
                dg[3 * H] = dh * t * og * (1.f - og);
                dg[4 * H] = dct * i * (1.f - u * u);
                f.dc[(size_t)l * H + col] = dct * fl;
                f.dc[(size_t)r * H + col] = dct * fr;
            } else {
                const float i = sigmoid_f(acc[0][v] + bias[0]), og = sigmoid_f(acc[1][v] + bias[1]);
                const float u = tanh_f(acc[2][v] + bias[2]);
                const float dct = dc + dh * og * (1.f - t * t);
                dg[0] = dct * u * i * (1.f - i);
                dg[H] = dh * t * og * (1.f - og);
                dg[2 * H] = dct * i * (1.f - u * u);
            }
        }
    } else {
        // operand gradient: the NG blocks of output columns of this column group start at g * (out_cols / NG)
        constexpr bool INNER = EPI == EPI_BWD_INNER_OPERAND || EPI == EPI_BWD_INNER_OPERAND4;
        const int block = f.out_cols / NG;
        if (col >= block) return;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int row = rb * 16 + (lane >> 4) * 4 + v;
            if (row >= count) continue;
            const int node = sm.node[row];
            if (node < 0) continue;
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                const int oc = g * block + col;
                if constexpr (INNER) {
                    const int child = oc < H ? f.left[node] : f.right[node];
                    float *p = f.dh + (size_t)child * H + (oc < H ? oc : oc - H);
                    // one contribution per element (a node has one parent): inside a persistent kernel it is added at the memory side
                    if constexpr (COH) (void)add_dev(p, acc[g][v]);
                    else *p += acc[g][v];
                } else {
                    f.d_x[(size_t)node * f.E + oc] = acc[g][v];
                }
            }
        }
    }
}

// Gate gradients from gate activations that the forward kept (Fwd::gates): the elementwise part
// of bwd_epilogue without the contraction in front of it.  One thread per (row of `list`, group of
// V hidden units); same outputs as the EPI_BWD_*_GATES epilogues (dg rows by list position from
// pos0 on, dc of the children).
// (COH: dh, dc and dg are exchanged between workgroups of one kernel, see the persistent form below.)
template <bool INNER, int V, bool COH>
__device__ inline void gate_grad_kept_rows(const Fwd &f, const int32_t *__restrict__ list, int n_rows, int pos0, long long first,
                                           long long stride)
{
    const int H = f.H, per_row = H / V;
    const int NG = INNER ? 5 : 3;
    const long long total = (long long)n_rows * per_row;
    for (long long e = first; e < total; e += stride) {
        const int row = (int)(e / per_row), col = (int)(e - (long long)row * per_row) * V;
        const int node = list[row];
        const size_t o = (size_t)node * H + col;
        const float *kept = f.gates + (size_t)node * (5 * H) + col;
        float *dg = f.dg + (size_t)(pos0 + row) * (NG * H) + col;
        int l = 0, r = 0;
        if (INNER) { l = f.left[node]; r = f.right[node]; }
        float cn[V], dh[V], dc[V], g[5][V], cl[V], cr[V], out[5][V], dcl[V], dcr[V];
        auto load = [&](float (&dst)[V], const float *src) {
            if constexpr (V == 4) { const floatx4 t = *reinterpret_cast<const floatx4 *>(src); dst[0] = t.x; dst[1] = t.y; dst[2] = t.z; dst[3] = t.w; }
            else dst[0] = *src;
        };
        auto load_x = [&](float (&dst)[V], const float *src) {      // what another workgroup may have written
            if constexpr (V == 4) { const floatx4 t = ld_f4<COH>(src); dst[0] = t.x; dst[1] = t.y; dst[2] = t.z; dst[3] = t.w; }
            else dst[0] = ld_f<COH>(src);
        };
        auto store = [&](float *dst, const float (&src)[V]) {       // ... and what another one will read
            if constexpr (V == 4 && COH) {
                st_dev(reinterpret_cast<unsigned long long *>(dst), pack2(__float_as_uint(src[0]), __float_as_uint(src[1])));
                st_dev(reinterpret_cast<unsigned long long *>(dst) + 1, pack2(__float_as_uint(src[2]), __float_as_uint(src[3])));
            } else if constexpr (V == 4) {
                *reinterpret_cast<floatx4 *>(dst) = floatx4{src[0], src[1], src[2], src[3]};
            } else {
                st_f<COH>(dst, src[0]);
            }
        };
        load(cn, f.c + o); load_x(dh, f.dh + o); load_x(dc, f.dc + o);
#pragma unroll
        for (int q = 0; q < NG; ++q) load(g[q], kept + (size_t)q * H);
        if (INNER) { load(cl, f.c + (size_t)l * H + col); load(cr, f.c + (size_t)r * H + col); }
#pragma unroll
        for (int v = 0; v < V; ++v) {
            const float t = tanh_f(cn[v]);
            if (INNER) {
                const float i = g[0][v], fl = g[1][v], fr = g[2][v], og = g[3][v], u = g[4][v];
                const float dct = dc[v] + dh[v] * og * (1.f - t * t);
                out[0][v] = dct * u * i * (1.f - i);
                out[1][v] = dct * cl[v] * fl * (1.f - fl);
                out[2][v] = dct * cr[v] * fr * (1.f - fr);
                out[3][v] = dh[v] * t * og * (1.f - og);
                out[4][v] = dct * i * (1.f - u * u);
                dcl[v] = dct * fl;
                dcr[v] = dct * fr;
            } else {
                const float i = g[0][v], og = g[1][v], u = g[2][v];
                const float dct = dc[v] + dh[v] * og * (1.f - t * t);
                out[0][v] = dct * u * i * (1.f - i);
                out[1][v] = dh[v] * t * og * (1.f - og);
                out[2][v] = dct * i * (1.f - u * u);
            }
        }
#pragma unroll
        for (int q = 0; q < NG; ++q) store(dg + (size_t)q * H, out[q]);
        if (INNER) { store(f.dc + (size_t)l * H + col, dcl); store(f.dc + (size_t)r * H + col, dcr); }
    }
}
template <bool INNER, int V>
__global__ __launch_bounds__(256) void k_gate_grad_kept(Fwd f, const int32_t *__restrict__ list, int n_rows, int pos0)
{
    gate_grad_kept_rows<INNER, V, false>(f, list, n_rows, pos0, (long long)blockIdx.x * blockDim.x + threadIdx.x,
                                         (long long)gridDim.x * blockDim.x);
}

// TreeRNN (h = tanh(a W + b), leaves h = x): the gradient of the pre-activation needs only the stored h,
// dpre = dh (1 - h^2), one row of H values per listed node (by list position from pos0 on).
template <int V, bool COH>
__device__ inline void rnn_gate_grad_rows(const Fwd &f, const int32_t *__restrict__ list, int n_rows, int pos0, long long first,
                                          long long stride)
{
    const int H = f.H, per_row = H / V;
    const long long total = (long long)n_rows * per_row;
    for (long long e = first; e < total; e += stride) {
        const int row = (int)(e / per_row), col = (int)(e - (long long)row * per_row) * V;
        const size_t o = (size_t)list[row] * H + col;
        float *dg = f.dg + (size_t)(pos0 + row) * H + col;
        if constexpr (V == 4) {
            const floatx4 hv = *reinterpret_cast<const floatx4 *>(f.h + o), dh = ld_f4<COH>(f.dh + o);
            const floatx4 out = {dh.x * (1.f - hv.x * hv.x), dh.y * (1.f - hv.y * hv.y), dh.z * (1.f - hv.z * hv.z),
                                 dh.w * (1.f - hv.w * hv.w)};
            if constexpr (COH) {
                st_dev(reinterpret_cast<unsigned long long *>(dg), pack2(__float_as_uint(out.x), __float_as_uint(out.y)));
                st_dev(reinterpret_cast<unsigned long long *>(dg) + 1, pack2(__float_as_uint(out.z), __float_as_uint(out.w)));
            } else {
                *reinterpret_cast<floatx4 *>(dg) = out;
            }
        } else {
            const float hv = f.h[o];
            st_f<COH>(dg, ld_f<COH>(f.dh + o) * (1.f - hv * hv));
        }
    }
}
template <int V>
__global__ __launch_bounds__(256) void k_rnn_gate_grad(Fwd f, const int32_t *__restrict__ list, int n_rows, int pos0)
{
    rnn_gate_grad_rows<V, false>(f, list, n_rows, pos0, (long long)blockIdx.x * blockDim.x + threadIdx.x,
                                 (long long)gridDim.x * blockDim.x);
}

// TreeRNN leaves: the embedding row is the state itself, so its gradient is the row of dh.
__global__ void k_rnn_leaf_grad(Fwd f)
{
    const size_t total = (size_t)f.n_leaf * f.H;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (size_t)gridDim.x * blockDim.x) {
        const int i = (int)(e / f.H), j = (int)(e - (size_t)i * f.H);
        const size_t o = (size_t)f.leaf_list[i] * f.H + j;
        f.d_x[o] = f.dh[o];
    }
}

// ---- RNTN (h_k = tanh(a^T V_k a + (a W)_k + b_k)) -----------------------------------------------
// With dz = dh (1 - h^2) and the row y = [ dz_k a_q for all (k, q) | dz ] of length d * 2d + d per node, both
// gradients are ordinary contractions that the kernels above already do:
//   da = y S          S[(k, q)][p] = V[k][p][q] + V[k][q][p],  S[d * 2d + k][p] = W[p][k]       (operand gradient)
//   sum_n a_n^T y_n   gives dV (as [p][(k, q)]) and dW (the last d columns), its column sums db   (weight gradient)
// k_rntn_build_s makes S from the parameters, k_rntn_rows the rows y of the listed nodes, k_rntn_unpack puts the
// weight-gradient contraction back into the layouts of V, W and b.
__global__ void k_rntn_build_s(const float *__restrict__ v, const float *__restrict__ w, float *__restrict__ s, int d)
{
    const int D2 = 2 * d;
    const size_t total = ((size_t)d * D2 + d) * D2;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (size_t)gridDim.x * blockDim.x) {
        const int p = (int)(e % D2);
        const size_t r = e / D2;
        if (r < (size_t)d * D2) {
            const int k = (int)(r / D2), q = (int)(r - (size_t)k * D2);
            s[e] = v[((size_t)k * D2 + p) * D2 + q] + v[((size_t)k * D2 + q) * D2 + p];
        } else {
            const int k = (int)(r - (size_t)d * D2);
            s[e] = w[(size_t)p * d + k];
        }
    }
}

__global__ __launch_bounds__(256) void k_rntn_rows(Fwd f, const int32_t *__restrict__ list, int n_rows, int pos0)
{
    const int d = f.H, D2 = 2 * d;
    const int L = d * D2 + d;
    const long long total = (long long)n_rows * L;
    for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (long long)gridDim.x * blockDim.x) {
        const int row = (int)(e / L), j = (int)(e - (long long)row * L);
        const int node = list[row];
        const int k = j < d * D2 ? j / D2 : j - d * D2;
        const float hv = f.h[(size_t)node * d + k];
        const float dz = f.dh[(size_t)node * d + k] * (1.f - hv * hv);
        float y = dz;
        if (j < d * D2) {
            const int q = j - k * D2;
            const int child = q < d ? f.left[node] : f.right[node];
            y = dz * f.h[(size_t)child * d + (q < d ? q : q - d)];
        }
        f.dg[(size_t)(pos0 + row) * L + j] = y;
    }
}

// acc [2d x (d * 2d + d)] = sum_n a_n^T y_n, colsum [d * 2d + d] = sum_n y_n  ->  d_v [d][2d][2d], d_w [2d][d], d_b [d]
__global__ void k_rntn_unpack(const float *__restrict__ acc, const float *__restrict__ colsum, float *__restrict__ d_v,
                              float *__restrict__ d_w, float *__restrict__ d_b, int d)
{
    const int D2 = 2 * d, L = d * D2 + d;
    const size_t n_v = (size_t)d * D2 * D2, total = n_v + (size_t)D2 * d + d;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (size_t)gridDim.x * blockDim.x) {
        if (e < n_v) {
            const int q = (int)(e % D2), p = (int)((e / D2) % D2), k = (int)(e / ((size_t)D2 * D2));
            d_v[e] = acc[(size_t)p * L + (size_t)k * D2 + q];
        } else if (e < n_v + (size_t)D2 * d) {
            const size_t r = e - n_v;
            const int k = (int)(r % d), p = (int)(r / d);
            d_w[r] = acc[(size_t)p * L + (size_t)d * D2 + k];
        } else {
            const int k = (int)(e - n_v - (size_t)D2 * d);
            d_b[k] = colsum[(size_t)d * D2 + k];
        }
    }
}

// out[r][c] = in[c][r] for a row-major [rows x cols] input
__global__ void k_transpose(const float *__restrict__ in, float *__restrict__ out, int rows, int cols)
{
    const size_t total = (size_t)rows * cols;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (size_t)gridDim.x * blockDim.x) {
        const size_t c = e / rows, r = e - c * rows;          // e indexes the output [cols x rows]
        out[e] = in[r * cols + c];
    }
}

// Weight gradient: out[k][j] += sum_q a_q[k] * dg[q][j] over the n_rows nodes of `list` (dg rows by
// list position), a_q = [h[left]; h[right]] (SEG 2, L = H) or the embedding row of the leaf's
// word (SEG 1, L = E).  K_out = SEG * L rows, n_cols columns, row-major; `out` is zero beforehand.
// One workgroup per 64 x 64 tile of the output and slice of the nodes (blockIdx.z; the slices'
// partial tiles are added with atomics: the node axis is long and the output small, so without
// slices there are too few workgroups to hide the latency of the gathers), wave w on the
// 32 x 32 quarter (w / 2, w % 2).  The contraction runs over the nodes, 16 at a time through LDS,
// on v_mfma_f32_16x16x4_f32 with the node index as the k of the instruction; the next 16 nodes'
// operands are requested into registers before the current ones are multiplied.
constexpr int WG_TILE = 64, WG_Q = 16, WG_LD = WG_TILE + 4;

template <int SEG, bool VEC4>
__global__ __launch_bounds__(256) void k_weight_grad(Fwd f, const int32_t *__restrict__ list, int n_rows,
                                                     const float *__restrict__ table, int L, const float *__restrict__ dg,
                                                     int n_cols, float *__restrict__ out, float *__restrict__ bias_out)
{
    __shared__ __align__(16) float as[2][WG_Q][WG_LD];         // two buffers each: a step's operands are parked while the
    __shared__ __align__(16) float bs[2][WG_Q][WG_LD];         // step before is still being multiplied (one barrier per step)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int k0 = blockIdx.x * WG_TILE, j0 = blockIdx.y * WG_TILE;
    const int K_out = SEG * L;
    const int wr = (wave >> 1) * 32, wc = (wave & 1) * 32;
    const int per = ((n_rows + (int)gridDim.z - 1) / (int)gridDim.z + WG_Q - 1) / WG_Q * WG_Q;
    const int q_lo = blockIdx.z * per, q_hi = min(n_rows, q_lo + per);
    if (q_lo >= q_hi) return;
    floatx4 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[a][b] = floatx4{0.f, 0.f, 0.f, 0.f};
    const int lq = tid >> 4, lk = (tid & 15) * 4;             // this thread stages 4 consecutive columns of row lq
    float ra[4], rb[4];
    // the workgroups of the first row of output tiles also sum the columns of dg they pass over (bias gradient)
    const bool with_bias = bias_out != nullptr && blockIdx.x == 0;
    float bsum[4] = {0.f, 0.f, 0.f, 0.f};
    // The operands of a step (16 nodes) hang on a chain of three loads: the node from the list, its source rows from
    // the child (or word) arrays, the data from those rows.  A step has only 16 MFMAs per wave to hide it, so the chain
    // is spread over three steps: step i requests the data of step i + 1, the source rows of step i + 2 and the node
    // of step i + 3, each from what the step before has requested.
    auto node_of = [&](int q0) {                              // stage 1
        const int q = q0 + lq;
        return q < q_hi ? list[q] : -1;
    };
    auto sources_of = [&](int node, int *s0, int *s1) {       // stage 2
        *s0 = *s1 = 0;
        if (node >= 0) {
            if (SEG == 2) { *s0 = f.left[node]; *s1 = f.right[node]; } else { *s0 = f.word[node]; }
        }
    };
    auto request = [&](int q0, int node, int s0, int s1) {    // stage 3: operands of nodes q0 .. q0 + 15 into registers
        const int q = q0 + lq;
        const bool live = node >= 0;
        if constexpr (VEC4) {      // L and n_cols multiples of 4, rows 16-byte aligned: 4 consecutive columns never leave a segment
            const int k = k0 + lk, j = j0 + lk;
            const int seg = (SEG == 2 && k >= L) ? 1 : 0;
            floatx4 a = floatx4{0.f, 0.f, 0.f, 0.f}, b = a;
            if (live && k < K_out) a = *reinterpret_cast<const floatx4 *>(table + (size_t)(seg ? s1 : s0) * L + (k - seg * L));
            if (live && j < n_cols) b = *reinterpret_cast<const floatx4 *>(dg + (size_t)q * n_cols + j);
#pragma unroll
            for (int e = 0; e < 4; ++e) { ra[e] = a[e]; rb[e] = b[e]; }
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int k = k0 + lk + e, j = j0 + lk + e;
                const int seg = (SEG == 2 && k >= L) ? 1 : 0;
                ra[e] = (live && k < K_out) ? table[(size_t)(seg ? s1 : s0) * L + (k - seg * L)] : 0.f;
                rb[e] = (live && j < n_cols) ? dg[(size_t)q * n_cols + j] : 0.f;
            }
        }
    };
    int node1 = node_of(q_lo), s0_1, s1_1;                    // step q_lo: all three stages at once
    sources_of(node1, &s0_1, &s1_1);
    request(q_lo, node1, s0_1, s1_1);
    node1 = node_of(q_lo + WG_Q);                             // step q_lo + 16: node and source rows
    sources_of(node1, &s0_1, &s1_1);
    int node2 = node_of(q_lo + 2 * WG_Q);                     // step q_lo + 32: node
    auto park = [&](int buf) {
        *reinterpret_cast<floatx4 *>(&as[buf][lq][lk]) = floatx4{ra[0], ra[1], ra[2], ra[3]};
        *reinterpret_cast<floatx4 *>(&bs[buf][lq][lk]) = floatx4{rb[0], rb[1], rb[2], rb[3]};
        if (with_bias) {
#pragma unroll
            for (int e = 0; e < 4; ++e) bsum[e] += rb[e];
        }
    };
    park(0);
    __syncthreads();
    int buf = 0;
    for (int q0 = q_lo; q0 < q_hi; q0 += WG_Q) {
        request(q0 + WG_Q, node1, s0_1, s1_1);                // (beyond the end: node -1, nothing is loaded)
        node1 = node2;
        sources_of(node1, &s0_1, &s1_1);
        node2 = node_of(q0 + 3 * WG_Q);
#pragma unroll
        for (int kk = 0; kk < WG_Q / 4; ++kk) {
            const int qq = kk * 4 + (lane >> 4);
            float a[2], b[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                a[t] = as[buf][qq][wr + t * 16 + (lane & 15)];
                b[t] = bs[buf][qq][wc + t * 16 + (lane & 15)];
            }
#pragma unroll
            for (int ta = 0; ta < 2; ++ta)
#pragma unroll
                for (int tb = 0; tb < 2; ++tb)
                    acc[ta][tb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[ta], b[tb], acc[ta][tb], 0, 0, 0);
        }
        // the other buffer was read in the step before this one, and every wave has passed the barrier since
        if (q0 + WG_Q < q_hi) park(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }
#pragma unroll
    for (int ta = 0; ta < 2; ++ta)
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int k = k0 + wr + ta * 16 + (lane >> 4) * 4 + v, j = j0 + wc + tb * 16 + (lane & 15);
                if (k < K_out && j < n_cols) atomicAdd(&out[(size_t)k * n_cols + j], acc[ta][tb][v]);
            }
    if (with_bias) {                                          // uniform per workgroup; the loop ended with a barrier
        *reinterpret_cast<floatx4 *>(&bs[0][lq][lk]) = floatx4{bsum[0], bsum[1], bsum[2], bsum[3]};
        __syncthreads();
        if (tid < WG_TILE && j0 + tid < n_cols) {
            float t = 0.f;
#pragma unroll
            for (int q = 0; q < WG_Q; ++q) t += bs[0][q][tid];
            atomicAdd(&bias_out[j0 + tid], t);
        }
    }
}

// Plain stochastic gradient descent, theta <- theta - lr * g (the product rounded, then the difference: the two
// roundings of the definition written as two operations), for up to four dense arrays in one launch.
struct SgdList {
    float *theta[4];
    const float *grad[4];
    size_t n[4];
};
__global__ void k_sgd_dense(SgdList z, float lr)
{
#pragma clang fp contract(off)          // two roundings, as the definition says: no fused multiply-add here
    const size_t stride = (size_t)gridDim.x * blockDim.x;
#pragma unroll
    for (int a = 0; a < 4; ++a)
        for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < z.n[a]; e += stride) {
            const float step = lr * z.grad[a][e];
            z.theta[a][e] = z.theta[a][e] - step;
        }
}

// The embedding table: row word[n] -= lr * d_x[n] for every leaf n.  Several leaves may share a word, so the
// rows are updated with atomics (the order of those additions is not fixed).
__global__ void k_sgd_embedding(float *__restrict__ emb, const float *__restrict__ d_x, const int32_t *__restrict__ left,
                                const int32_t *__restrict__ word, int n_nodes, int E, int vocab, float lr)
{
    const size_t total = (size_t)n_nodes * E;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (size_t)gridDim.x * blockDim.x) {
        const int n = (int)(e / E), j = (int)(e - (size_t)n * E);
        if (left[n] >= 0) continue;
        const int w = word[n];
        if (w < 0 || w >= vocab) continue;
        atomicAdd(&emb[(size_t)w * E + j], -(lr * d_x[e]));
    }
}

// ---- all heights in one launch ------------------------------------------------------------------
// The walk over the heights above as one persistent kernel: the per-height lists are on the device already (the
// counting sort of the structure pass), so the host needs neither the number of heights nor their sizes and
// tl_backward returns without waiting for the device.  Per height, from the roots down:
//   gate gradients   from the gate activations that the forward kept (TreeLSTM) or from h (TreeRNN), elementwise, the
//                    rows shared out over all threads of the grid
//   (grid barrier)
//   operand gradient tiles of the height's rows x column groups on the streaming cell, as in the per-height launches
//                    (four column blocks per group for heights of more than 64 rows, one otherwise)
//   (grid barrier)
// What one phase writes and the next reads on another workgroup (dg, dh, dc) goes through device-scope stores and
// loads; the barrier is the bounded one of the level scheduler.  (Gate gradients that recompute the forward
// contraction, and the RNTN cell, keep the per-height launches.)
struct BwdHeights {
    Gemm bwd4, bwd1;              // packed U^T with four column blocks per group / with one
    int ng_inner;                 // 4: both forms exist, 1: only bwd4 holds weights (one block per group)
    float *dg_int;
    int kept_v4;                  // rows of h, c, gates and dg are 16-byte aligned and H % 4 == 0
};

template <bool LSTM, bool VEC4>
__global__ __launch_bounds__(WG_THREADS, 2) void k_backward_heights(Fwd f, BwdHeights b)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    TileSmem &sm = *reinterpret_cast<TileSmem *>(smem_raw);
    if (batch_rejected(f)) return;
    const int tid = threadIdx.x;
    const int H = f.H;
    const int n_levels = f.ctl->n_levels;
    const long long first = (long long)blockIdx.x * blockDim.x + tid, stride = (long long)gridDim.x * blockDim.x;
    unsigned epoch = 0, unused = 0;
    Fwd g = f;
    g.dg = b.dg_int;
    g.out_cols = 2 * H;
    for (int lvl = n_levels - 1; lvl >= 1; --lvl) {         // roots first: a parent is always higher than its children
        const int lo = f.level_off[lvl], rows = f.level_off[lvl + 1] - lo;
        const int32_t *list = f.level_nodes + lo;
        g.pos0 = lo;
        if constexpr (LSTM) {
            if (b.kept_v4) gate_grad_kept_rows<true, 4, true>(g, list, rows, lo, first, stride);
            else gate_grad_kept_rows<true, 1, true>(g, list, rows, lo, first, stride);
        } else {
            if (b.kept_v4) rnn_gate_grad_rows<4, true>(g, list, rows, lo, first, stride);
            else rnn_gate_grad_rows<1, true>(g, list, rows, lo, first, stride);
        }
        if (!grid_barrier(sm, f, epoch, 0u, 0u, &unused)) return;
        const int ng = (b.ng_inner == 4 && rows > 64) ? 4 : 1;
        g.bwd = (b.ng_inner == 4 && ng == 1) ? b.bwd1 : b.bwd4;
        g.n_cg = (2 * H / ng + HU - 1) / HU;
        const LevelPlan plan = plan_level(rows, f.cap_tiles);
        for (int item = blockIdx.x; item < plan.n_tiles * g.n_cg; item += gridDim.x) {
            const int tile = item / g.n_cg, cg = item - tile * g.n_cg;
            int start, count;
            plan_tile(plan, rows, tile, &start, &count);
            __syncthreads();                                // the row tables are free
            tile_set_rows<EPI_BWD_INNER_OPERAND>(sm, g, tid, tid < count ? list[start + tid] : -1, lo + start + tid);
            if (tid == 0) sm.cmd[3] = lo + start;
            __syncthreads();
            if (ng == 4) cell_tile<EPI_BWD_INNER_OPERAND4, VEC4, true>(sm, g, g.bwd, g.dg, count, cg);
            else cell_tile<EPI_BWD_INNER_OPERAND, VEC4, true>(sm, g, g.bwd, g.dg, count, cg);
        }
        if (!grid_barrier(sm, f, epoch, 0u, 0u, &unused)) return;
    }
}

// The same walk with the operand gradient on weight-stationary workgroups (TreeLSTM from kept activations, 5 H a
// multiple of 128).  U^T is the one matrix that every height multiplies, so a workgroup owns 16 of the 2 H output
// columns for the whole call and keeps its slice of U^T in registers: the K axis (5 H) in four quarters, one per wave,
// 5 H / 64 k-steps x 4 registers each (160 at H = 512).  The rows of dG are long (5 H floats), so a block of 16 rows
// passes through LDS in two halves of each wave's quarter: while the matrix instructions of one half run, the other
// half (or the next block's first) is on its way.  A wave adds up its quarter in k order on one accumulator, the four
// quarters meet in LDS and are added in wave order: the order of every other data path, so the same bits.  Sets of
// 2 H / 16 workgroups share the blocks of a height.
template <int SPW2> struct OperandWsSmem {
    static constexpr int A_LD = STEP_K * SPW2 + 4;          // LDS row stride of half a quarter of a row, floats
    float a[4][16 * A_LD];
    float red[4 * 4 * 64];                                  // [wave][v][lane]
    int child[2][16];                                       // left / right child of the block's nodes
    int cmd[8];
};

// (LSTM = false: TreeRNN, whose rows of dG have H values, so K = H: a multiple of 128, SPW2 = H / 128.)
template <int SPW2, bool LSTM = true>
__global__ __launch_bounds__(WG_THREADS, 1) void k_backward_heights_ws(Fwd f, BwdHeights b)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    using Smem = OperandWsSmem<SPW2>;
    Smem &sm = *reinterpret_cast<Smem *>(smem_raw);
    if (batch_rejected(f)) return;
    constexpr int NLB = SPW2;                               // row loads per lane and half: 16 rows x 4 SPW2 pieces / 64 lanes
    constexpr int PPR = 4 * SPW2;                           // 16-byte pieces of a row in one half of a wave's quarter
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int H = f.H, K = (LSTM ? 5 : 1) * H;
    const int n_cg = 2 * H / HU;
    const int cg = (int)blockIdx.x % n_cg, slot = (int)blockIdx.x / n_cg, n_slots = (int)gridDim.x / n_cg;
    const int n_levels = f.ctl->n_levels;
    const long long first = (long long)blockIdx.x * blockDim.x + tid, stride = (long long)gridDim.x * blockDim.x;
    WsWeights<1, 2 * SPW2> w;
    {                                                       // (the grid is a whole number of sets)
        ws_load(w, b.bwd1, cg, wave, lane);
        // the weights live in the accumulation registers (a matrix instruction takes its B operand from either file), the
        // vector registers are for the rows in flight
#pragma unroll
        for (int s = 0; s < 2 * SPW2; ++s)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float x = w.b[s][0][i];
                asm volatile("" : "+a"(x));                     // no instruction: a register-class constraint only
                w.b[s][0][i] = x;
            }
    }
    const unsigned row_b = (unsigned)K * 4u;
    float *a_w = sm.a[wave];
    const float *a_lane = &a_w[(lane & 15) * Smem::A_LD + (lane >> 4) * 4];
    const __amdgpu_buffer_rsrc_t rs_dg = buf_of(b.dg_int, (unsigned long long)f.n_int * K * 4);
    // Rows in flight: one set of registers per half, so that a half is requested a whole block (both halves' matrix
    // instructions) before it is parked - the latency of a request is longer than one half's matrix instructions.
    floatx4 rows0[NLB], rows1[NLB];
    // 16 rows of dG from row `base` on, half `half` of this wave's quarter.  (Rows past the end of the height are other
    // nodes' rows, past the end of the table they read as zero; every output row depends on its own row only, and the
    // results of such rows are dropped.)
    // Piece j * 64 + lane of a half is piece c of row r, PPR pieces to a row: (r, c) is walked along with j instead of
    // being kept per piece (the registers are needed for the weights and the rows in flight).
    auto request = [&](floatx4 (&rows)[NLB], int base, int half) {
        const unsigned off = (unsigned)base * row_b + (unsigned)((wave * 2 + half) * SPW2 * STEP_K) * 4u;
        int r = lane / PPR, c = lane % PPR;
#pragma unroll
        for (int j = 0; j < NLB; ++j) {
            typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
            const uintx4 u = __builtin_amdgcn_raw_buffer_load_b128(rs_dg, (int)(off + (unsigned)r * row_b + (unsigned)c * 16u), 0, 16);
            rows[j] = floatx4{__uint_as_float(u.x), __uint_as_float(u.y), __uint_as_float(u.z), __uint_as_float(u.w)};
            c += 64;
            r += c / PPR;
            c %= PPR;
        }
    };
    auto park = [&](const floatx4 (&rows)[NLB]) {
        int r = lane / PPR, c = lane % PPR;
#pragma unroll
        for (int j = 0; j < NLB; ++j) {
            *reinterpret_cast<floatx4 *>(&a_w[r * Smem::A_LD + c * 4]) = rows[j];
            c += 64;
            r += c / PPR;
            c %= PPR;
        }
    };
    unsigned epoch = 0, unused = 0;
    Fwd g = f;
    g.dg = b.dg_int;
#pragma unroll 1
    for (int lvl = n_levels - 1; lvl >= 1; --lvl) {
        const int lo = f.level_off[lvl], n_rows = f.level_off[lvl + 1] - lo;
        const int32_t *list = f.level_nodes + lo;
        // (H % 128 == 0; the host has checked the alignment)
        if constexpr (LSTM) gate_grad_kept_rows<true, 4, true>(g, list, n_rows, lo, first, stride);
        else rnn_gate_grad_rows<4, true>(g, list, n_rows, lo, first, stride);
        if (!grid_barrier(sm, f, epoch, 0u, 0u, &unused)) return;
        const int n_blocks = (n_rows + 15) >> 4;
        if (slot < n_blocks) {
            request(rows0, lo + slot * 16, 0);
            request(rows1, lo + slot * 16, 1);
        }
#pragma unroll 1
        for (int blk = slot; blk < n_blocks; blk += n_slots) {
            const int cnt = min(16, n_rows - blk * 16);
            if (tid < 32) {                                 // the children that this block's results are added to
                const int r = tid & 15;
                const int node = r < cnt ? list[blk * 16 + r] : -1;
                sm.child[tid >> 4][r] = node < 0 ? -1 : (tid < 16 ? f.left[node] : f.right[node]);
            }
            floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                // (the last block asks for rows that nobody uses: past the end of the table they read as zero)
                if (half == 0) {
                    park(rows0);
                    request(rows0, lo + (blk + n_slots) * 16, 0);
                } else {
                    park(rows1);
                    request(rows1, lo + (blk + n_slots) * 16, 1);
                }
                __builtin_amdgcn_sched_barrier(0);
                floatx4 av_next = *reinterpret_cast<const floatx4 *>(a_lane);
#pragma unroll
                for (int s = 0; s < SPW2; ++s) {
                    const floatx4 av = av_next;
                    if (s + 1 < SPW2) av_next = *reinterpret_cast<const floatx4 *>(a_lane + (s + 1) * STEP_K);
#pragma unroll
                    for (int i = 0; i < 4; ++i) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av[i], w.b[half * SPW2 + s][0][i], acc, 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
#pragma unroll
            for (int v = 0; v < 4; ++v) sm.red[(wave * 4 + v) * 64 + lane] = acc[v];
            __syncthreads();
            {
                // wave w finishes accumulator row w of every group of four rows: the quarters in wave order
                float sum = sm.red[(0 * 4 + wave) * 64 + lane];
                sum += sm.red[(1 * 4 + wave) * 64 + lane];
                sum += sm.red[(2 * 4 + wave) * 64 + lane];
                sum += sm.red[(3 * 4 + wave) * 64 + lane];
                const int row = (lane >> 4) * 4 + wave, oc = cg * HU + (lane & 15);
                const int child = sm.child[oc < H ? 0 : 1][row];
                if (child >= 0) {
                    // (one contribution per element, from the node's only parent: an addition at the memory side gives the bits
                    // of load, add, store, and the wave does not wait for a load behind the rows it has requested ahead)
                    float *p = f.dh + (size_t)child * H + (oc < H ? oc : oc - H);
                    (void)add_dev(p, sum);
                }
            }
            __syncthreads();                                // red and child are free again
        }
        if (!grid_barrier(sm, f, epoch, 0u, 0u, &unused)) return;
    }
}

// Zeroes up to six arrays in one launch (outputs and workspace of the backward pass).
struct ZeroList {
    float *p[6];
    size_t n[6];
    const float *src;       // and one copy in the same launch: dst[0 .. n_copy) = src (n_copy = 0: none); a multiple of
    float *dst;             // four floats with both ends 16-byte aligned is moved 16 bytes at a time
    size_t n_copy;
};
__global__ void k_zero_many(ZeroList z)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x, first = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (z.n_copy % 4 == 0 && (((uintptr_t)z.src | (uintptr_t)z.dst) & 15) == 0) {
        const floatx4 *s4 = reinterpret_cast<const floatx4 *>(z.src);
        floatx4 *d4 = reinterpret_cast<floatx4 *>(z.dst);
        for (size_t e = first; e < z.n_copy / 4; e += stride) d4[e] = s4[e];
    } else {
        for (size_t e = first; e < z.n_copy; e += stride) z.dst[e] = z.src[e];
    }
#pragma unroll
    for (int a = 0; a < 6; ++a)
        for (size_t e = first; e < z.n[a]; e += stride) z.p[a][e] = 0.f;
}

}  // namespace tl
