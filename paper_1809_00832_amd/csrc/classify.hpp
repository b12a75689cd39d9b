// Per-node classifier head: probs[n] = softmax(h[n] W_s + b_s) for every row of h.
//
// Section 6.1: the evaluated networks label all nodes of a parse tree.  With a handful of classes
// the contraction is tiny ([N x H] x [H x C], C <= 32) and the kernel is bound by reading h once
// from memory, so it is written as a streaming reduction, not for the matrix cores: W_s sits in
// LDS (class-major), 16 lanes share a row (each lane reads 16 consecutive bytes of it per step,
// the 16 lanes 256 consecutive bytes), a wave works on 4 rows at a time, partial logits are
// combined with four butterfly steps inside the 16-lane group, and the softmax is evaluated in
// registers; the C probabilities of a row are written by consecutive lanes.
#pragma once

#include "common.hpp"

namespace tl {

constexpr int CLS_MAX_CLASSES = 32;

template <int CT>   // CT >= n_classes: accumulators per lane
__global__ __launch_bounds__(256) void k_classify(const float *__restrict__ h, const float *__restrict__ w_s,
                                                  const float *__restrict__ b_s, float *__restrict__ probs, int n_rows, int H,
                                                  int C)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    float *wt = reinterpret_cast<float *>(smem_raw);       // [C][Hp]: W_s transposed, rows padded to a multiple of 4
    const int Hp = (H + 3) & ~3;
    for (int e = threadIdx.x; e < C * Hp; e += blockDim.x) {
        const int c = e / Hp, k = e - c * Hp;
        wt[e] = k < H ? w_s[(size_t)k * C + c] : 0.f;
    }
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l16 = lane & 15, rslot = lane >> 4;
    const bool vec4 = (H & 3) == 0 && ((reinterpret_cast<uintptr_t>(h) & 15) == 0);
    float bias[CT];
#pragma unroll
    for (int c = 0; c < CT; ++c) bias[c] = c < C ? b_s[c] : 0.f;

    for (long long base = (long long)blockIdx.x * 16; base < n_rows; base += (long long)gridDim.x * 16) {
        const long long row = base + wave * 4 + rslot;
        const bool live = row < n_rows;
        const float *hr = h + (size_t)(live ? row : 0) * H;
        float acc[CT];
#pragma unroll
        for (int c = 0; c < CT; ++c) acc[c] = 0.f;
        // four 16-byte requests per lane are in flight before the first is used: with only a few
        // waves per SIMD the kernel is otherwise bound by memory latency, not bandwidth
        for (int kb = l16 * 4; kb < Hp; kb += 256) {
            floatx4 x[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int k0 = kb + 64 * u;
                if (vec4) {
                    x[u] = k0 < Hp ? *reinterpret_cast<const floatx4 *>(hr + k0) : floatx4{0.f, 0.f, 0.f, 0.f};
                } else {
                    x[u].x = k0 < H ? hr[k0] : 0.f;
                    x[u].y = k0 + 1 < H ? hr[k0 + 1] : 0.f;
                    x[u].z = k0 + 2 < H ? hr[k0 + 2] : 0.f;
                    x[u].w = k0 + 3 < H ? hr[k0 + 3] : 0.f;
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int k0 = kb + 64 * u;
                if (k0 < Hp) {
#pragma unroll
                    for (int c = 0; c < CT; ++c) {
                        if (c < C) {
                            const floatx4 w = *reinterpret_cast<const floatx4 *>(wt + c * Hp + k0);
                            acc[c] += x[u].x * w.x + x[u].y * w.y + x[u].z * w.z + x[u].w * w.w;
                        }
                    }
                }
            }
        }
        float m = -3.0e38f;
#pragma unroll
        for (int c = 0; c < CT; ++c) {
            if (c < C) {
#pragma unroll
                for (int o = 8; o >= 1; o >>= 1) acc[c] += __shfl_xor(acc[c], o);
                acc[c] += bias[c];
                m = fmaxf(m, acc[c]);
            }
        }
        float sum = 0.f;
#pragma unroll
        for (int c = 0; c < CT; ++c) {
            if (c < C) {
                acc[c] = __expf(acc[c] - m);
                sum += acc[c];
            }
        }
        const float inv = 1.f / sum;
        if (live) {
#pragma unroll
            for (int c = 0; c < CT; ++c)
                if (c < C && (c & 15) == l16) probs[(size_t)row * C + c] = acc[c] * inv;
        }
    }
}

// Backward of the head under a cross-entropy summed over the labelled rows (label in [0, C);
// any other value marks a row without label, which contributes nothing):
//   d_logits[n] = probs[n] - onehot(label[n]),   g_h[n] = d_logits[n] W_s^T,   loss += -log probs[n][label[n]].
// Same lane layout as k_classify (the logits are recomputed, h is read once); g_h is written by
// the lanes that hold the matching columns of W_s.  The loss is summed per workgroup first and
// added to *loss with one atomic per workgroup.  W_s^T d_logits sums (d_w_s, d_b_s) are left to
// k_head_weight_grad, which reads d_logits.
template <int CT>
__global__ __launch_bounds__(256) void k_classify_backward(const float *__restrict__ h, const float *__restrict__ w_s,
                                                           const float *__restrict__ b_s, const int32_t *__restrict__ label,
                                                           float *__restrict__ d_logits, float *__restrict__ g_h,
                                                           float *__restrict__ loss, int n_rows, int H, int C)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    __shared__ float s_loss[4];
    float *wt = reinterpret_cast<float *>(smem_raw);       // [C][Hp], as in k_classify
    const int Hp = (H + 3) & ~3;
    for (int e = threadIdx.x; e < C * Hp; e += blockDim.x) {
        const int c = e / Hp, k = e - c * Hp;
        wt[e] = k < H ? w_s[(size_t)k * C + c] : 0.f;
    }
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l16 = lane & 15, rslot = lane >> 4;
    const bool vec4 = (H & 3) == 0 && ((reinterpret_cast<uintptr_t>(h) & 15) == 0) && ((reinterpret_cast<uintptr_t>(g_h) & 15) == 0);
    float bias[CT];
#pragma unroll
    for (int c = 0; c < CT; ++c) bias[c] = c < C ? b_s[c] : 0.f;
    float my_loss = 0.f;

    for (long long base = (long long)blockIdx.x * 16; base < n_rows; base += (long long)gridDim.x * 16) {
        const long long row = base + wave * 4 + rslot;
        const bool live = row < n_rows;
        const float *hr = h + (size_t)(live ? row : 0) * H;
        int lab = live ? label[row] : -1;
        if (lab >= C) lab = -1;
        float acc[CT];
#pragma unroll
        for (int c = 0; c < CT; ++c) acc[c] = 0.f;
        for (int kb = l16 * 4; kb < Hp; kb += 256) {
            floatx4 x[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int k0 = kb + 64 * u;
                if (vec4) {
                    x[u] = k0 < Hp ? *reinterpret_cast<const floatx4 *>(hr + k0) : floatx4{0.f, 0.f, 0.f, 0.f};
                } else {
                    x[u].x = k0 < H ? hr[k0] : 0.f;
                    x[u].y = k0 + 1 < H ? hr[k0 + 1] : 0.f;
                    x[u].z = k0 + 2 < H ? hr[k0 + 2] : 0.f;
                    x[u].w = k0 + 3 < H ? hr[k0 + 3] : 0.f;
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int k0 = kb + 64 * u;
                if (k0 < Hp) {
#pragma unroll
                    for (int c = 0; c < CT; ++c) {
                        if (c < C) {
                            const floatx4 w = *reinterpret_cast<const floatx4 *>(wt + c * Hp + k0);
                            acc[c] += x[u].x * w.x + x[u].y * w.y + x[u].z * w.z + x[u].w * w.w;
                        }
                    }
                }
            }
        }
        float m = -3.0e38f, z_lab = 0.f;
#pragma unroll
        for (int c = 0; c < CT; ++c) {
            if (c < C) {
#pragma unroll
                for (int o = 8; o >= 1; o >>= 1) acc[c] += __shfl_xor(acc[c], o);
                acc[c] += bias[c];
                m = fmaxf(m, acc[c]);
                if (c == lab) z_lab = acc[c];
            }
        }
        float sum = 0.f;
#pragma unroll
        for (int c = 0; c < CT; ++c) {
            if (c < C) {
                acc[c] = __expf(acc[c] - m);
                sum += acc[c];
            }
        }
        const float inv = 1.f / sum;
        if (lab >= 0 && l16 == 0) my_loss += __logf(sum) - (z_lab - m);
        // acc becomes the gradient of the logits; zero for a row without label
#pragma unroll
        for (int c = 0; c < CT; ++c) {
            if (c < C) {
                acc[c] = lab >= 0 ? acc[c] * inv - (c == lab ? 1.f : 0.f) : 0.f;
                if (live && (c & 15) == l16) d_logits[(size_t)row * C + c] = acc[c];
            }
        }
        if (live) {
            float *gr = g_h + (size_t)row * H;
            for (int k0 = l16 * 4; k0 < Hp; k0 += 64) {
                floatx4 g = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int c = 0; c < CT; ++c) {
                    if (c < C) {
                        const floatx4 w = *reinterpret_cast<const floatx4 *>(wt + c * Hp + k0);
                        g.x += acc[c] * w.x; g.y += acc[c] * w.y; g.z += acc[c] * w.z; g.w += acc[c] * w.w;
                    }
                }
                if (vec4) {
                    *reinterpret_cast<floatx4 *>(gr + k0) = g;
                } else {
                    if (k0 < H) gr[k0] = g.x;
                    if (k0 + 1 < H) gr[k0 + 1] = g.y;
                    if (k0 + 2 < H) gr[k0 + 2] = g.z;
                    if (k0 + 3 < H) gr[k0 + 3] = g.w;
                }
            }
        }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) my_loss += __shfl_xor(my_loss, o);
    if (lane == 0) s_loss[wave] = my_loss;
    __syncthreads();
    if (threadIdx.x == 0) {
        const float total = (s_loss[0] + s_loss[1]) + (s_loss[2] + s_loss[3]);
        if (total != 0.f) atomicAdd(loss, total);
    }
}

// Zeroes the three sums of the head's backward pass in one launch.
__global__ void k_head_zero(float *__restrict__ d_w_s, int n_w, float *__restrict__ d_b_s, int n_b, float *__restrict__ loss)
{
    const int stride = gridDim.x * blockDim.x;
    for (int e = blockIdx.x * blockDim.x + threadIdx.x; e < n_w; e += stride) d_w_s[e] = 0.f;
    if (blockIdx.x == 0) {
        for (int e = threadIdx.x; e < n_b; e += blockDim.x) d_b_s[e] = 0.f;
        if (threadIdx.x == 0) *loss = 0.f;
    }
}

// d_w_s[k][c] += sum_n h[n][k] d_logits[n][c] and d_b_s[c] += sum_n d_logits[n][c]; both outputs
// are zero beforehand.  blockIdx.x picks 64 columns k of h (lane l owns column 64 blockIdx.x + l,
// so a wave reads 256 consecutive bytes of a row), blockIdx.y a slice of the rows.  The slice's
// d_logits rows are staged through LDS, 4 * HW_ROWS at a time; wave w takes the w-th group of
// HW_ROWS rows of every stage, 8 loads in flight per lane.  The four waves' partial sums are
// combined in LDS and added to the outputs with one atomic per element and workgroup.
constexpr int HW_ROWS = 32;

template <int CT>
__global__ __launch_bounds__(256) void k_head_weight_grad(const float *__restrict__ h, const float *__restrict__ d_logits,
                                                          float *__restrict__ d_w_s, float *__restrict__ d_b_s, int n_rows, int H,
                                                          int C)
{
    __shared__ float s_g[4 * HW_ROWS][CT];
    __shared__ float s_red[3][CT][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int per = (n_rows + gridDim.y - 1) / gridDim.y;
    const int lo = blockIdx.y * per, hi = min(n_rows, lo + per);
    if (lo >= hi) return;
    const int k = blockIdx.x * 64 + lane;
    const bool mine = k < H;
    float acc[CT];
#pragma unroll
    for (int c = 0; c < CT; ++c) acc[c] = 0.f;
    float bsum = 0.f;
    for (int r0 = lo; r0 < hi; r0 += 4 * HW_ROWS) {
        const int nr = min(4 * HW_ROWS, hi - r0);
        __syncthreads();
        for (int e = threadIdx.x; e < 4 * HW_ROWS * CT; e += 256) {
            const int r = e / CT, c = e - r * CT;
            s_g[r][c] = (r < nr && c < C) ? d_logits[(size_t)(r0 + r) * C + c] : 0.f;
        }
        __syncthreads();
        if (blockIdx.x == 0 && (int)threadIdx.x < C)
            for (int r = 0; r < nr; ++r) bsum += s_g[r][threadIdx.x];
        if (mine) {
            const int w0 = wave * HW_ROWS;
            for (int r = w0; r < w0 + HW_ROWS && r < nr; r += 8) {
                float x[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) x[u] = r + u < nr ? h[(size_t)(r0 + r + u) * H + k] : 0.f;
#pragma unroll
                for (int u = 0; u < 8; ++u)
#pragma unroll
                    for (int c = 0; c < CT; ++c)
                        if (c < C) acc[c] += x[u] * s_g[r + u][c];
            }
        }
    }
    if (wave > 0) {
#pragma unroll
        for (int c = 0; c < CT; ++c) s_red[wave - 1][c][lane] = acc[c];
    }
    __syncthreads();
    if (wave == 0 && mine) {
#pragma unroll
        for (int c = 0; c < CT; ++c)
            if (c < C) atomicAdd(&d_w_s[(size_t)k * C + c], (acc[c] + s_red[0][c][lane]) + (s_red[1][c][lane] + s_red[2][c][lane]));
    }
    if (blockIdx.x == 0 && (int)threadIdx.x < C) atomicAdd(&d_b_s[threadIdx.x], bsum);
}

}  // namespace tl
