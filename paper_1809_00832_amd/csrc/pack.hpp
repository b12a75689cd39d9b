// Re-packing of the caller's row-major parameters into the operand order of the MFMA tiles.
//
// The caller's matrix W is [SEG*L x NG*H] (NG gate blocks of H columns).  The packed copy is
// indexed [column group cg][k-step s][gate g][lane][i]:
//   fp32 (16x16x4 MFMA, i < 4):  k = 16 s + 4 (lane / 16) + i
//   bf16 (16x16x32 MFMA, i < 8): k = 32 s + 8 (lane / 16) + i
// holds W[row(k)][g*H + 16 cg + lane % 16], so that one 16-byte read per lane yields the B
// operands of consecutive MFMAs and the five gates of a hidden unit meet in one lane.
// k runs over the padded K axis: SEG segments of Lp = roundup(L, 4) rows each, then zeros up
// to a multiple of KC; padded rows and hidden units >= H hold zeros.
#pragma once

#include <hip/hip_bf16.h>

#include "common.hpp"

namespace tl {

__device__ inline unsigned short f32_to_bf16_rne(float x)
{
    unsigned int bits = __float_as_uint(x);
    bits += 0x7FFFu + ((bits >> 16) & 1u);
    return (unsigned short)(bits >> 16);
}

__device__ inline float pack_source(const float *w, int k, int g, int hu, int NG, int H, int SEG, int L, int Lp)
{
    int seg = k / Lp, off = k - seg * Lp;
    if (seg >= SEG || off >= L || hu >= H) return 0.f;
    return w[(size_t)(seg * L + off) * ((size_t)NG * H) + (size_t)g * H + hu];
}

__global__ void k_pack_f32(const float *__restrict__ w, float *__restrict__ wp, int NG, int H, int SEG, int L, int Lp,
                           int n_steps, int n_cg)
{
    size_t total = (size_t)n_cg * n_steps * NG * 64 * 4;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (size_t)gridDim.x * blockDim.x) {
        int i = (int)(e & 3);
        int lane = (int)((e >> 2) & 63);
        size_t r = e >> 8;
        int g = (int)(r % NG);
        r /= NG;
        int s = (int)(r % n_steps);
        int cg = (int)(r / n_steps);
        int k = 16 * s + 4 * (lane >> 4) + i;
        wp[e] = pack_source(w, k, g, cg * HU + (lane & 15), NG, H, SEG, L, Lp);
    }
}

__global__ void k_pack_bf16(const float *__restrict__ w, unsigned short *__restrict__ wp, int NG, int H, int SEG, int L,
                            int Lp, int n_steps32, int n_cg)
{
    size_t total = (size_t)n_cg * n_steps32 * NG * 64 * 8;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (size_t)gridDim.x * blockDim.x) {
        int i = (int)(e & 7);
        int lane = (int)((e >> 3) & 63);
        size_t r = e >> 9;
        int g = (int)(r % NG);
        r /= NG;
        int s = (int)(r % n_steps32);
        int cg = (int)(r / n_steps32);
        int k = 32 * s + 8 * (lane >> 4) + i;
        wp[e] = f32_to_bf16_rne(pack_source(w, k, g, cg * HU + (lane & 15), NG, H, SEG, L, Lp));
    }
}

__global__ void k_pack_bias(const float *__restrict__ b, float *__restrict__ bp, int NG, int H, int n_cg)
{
    int total = n_cg * NG * HU;
    for (int e = blockIdx.x * blockDim.x + threadIdx.x; e < total; e += gridDim.x * blockDim.x) {
        int j = e % HU, g = (e / HU) % NG, cg = e / (HU * NG);
        int hu = cg * HU + j;
        bp[e] = hu < H ? b[g * H + hu] : 0.f;
    }
}

// Several fp32 matrices packed over in one launch (the re-packing after a parameter update: the buffers exist, only their
// contents change).  A job is what k_pack_f32 and k_pack_bias do for one matrix; element (row, col) of the matrix to pack
// is src[row * rs + col * cs], so the transposed matrices of the backward pass are read straight from the parameters
// (rs = 1, cs = number of rows) with no transposed copy in between.
struct PackJob {
    const float *w;
    float *wp;
    const float *b;         // null: the bias is not touched (the backward pass's contractions have none)
    float *bp;
    int NG, H, SEG, L, Lp, n_steps, n_cg;
    long long rs, cs;
};
constexpr int PACK_JOBS = 6;
struct PackList {
    PackJob job[PACK_JOBS];
    int n;
};
__global__ void k_pack_many(PackList pl)
{
    for (int a = 0; a < pl.n; ++a) {
        const PackJob &j = pl.job[a];
        const size_t total = (size_t)j.n_cg * j.n_steps * j.NG * 64 * 4;
        for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (size_t)gridDim.x * blockDim.x) {
            const int i = (int)(e & 3), lane = (int)((e >> 2) & 63);
            size_t r = e >> 8;
            const int g = (int)(r % j.NG);
            r /= j.NG;
            const int s = (int)(r % j.n_steps), cg = (int)(r / j.n_steps);
            const int k = 16 * s + 4 * (lane >> 4) + i, hu = cg * HU + (lane & 15);
            const int seg = k / j.Lp, off = k - seg * j.Lp;
            float v = 0.f;
            if (seg < j.SEG && off < j.L && hu < j.H) v = j.w[(long long)(seg * j.L + off) * j.rs + (long long)(g * j.H + hu) * j.cs];
            j.wp[e] = v;
        }
        if (j.b) {
            const int nb = j.n_cg * j.NG * HU;
            for (int e = blockIdx.x * blockDim.x + threadIdx.x; e < nb; e += gridDim.x * blockDim.x) {
                const int q = e % HU, g = (e / HU) % j.NG, cg = e / (HU * j.NG);
                const int hu = cg * HU + q;
                j.bp[e] = hu < j.H ? j.b[g * j.H + hu] : 0.f;
            }
        }
    }
}

// bf16 copy of a row-major table with rows padded to Ls elements (pads zero)
__global__ void k_pad_bf16(const float *__restrict__ src, unsigned short *__restrict__ dst, size_t rows, int L, int Ls)
{
    const size_t total = rows * (size_t)Ls;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (size_t)gridDim.x * blockDim.x) {
        const size_t r = e / Ls;
        const int j = (int)(e - r * Ls);
        dst[e] = j < L ? f32_to_bf16_rne(src[r * L + j]) : (unsigned short)0;
    }
}

}  // namespace tl
