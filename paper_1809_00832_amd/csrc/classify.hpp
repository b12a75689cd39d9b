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

}  // namespace tl
