// HBM-bound helper kernels: the blocked tensor layouts of the paper's convolution listing
// (figure "The 2-D Convolution code": input[img][ifm_tile][h][w][ifm],
// filter[ofm_tile][ifm_tile][kj][ki][ifm][ofm]) and the separate element-wise operators that the
// fused epilogue replaces (section "Operator Fusion").
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "internal.hpp"

namespace polydl {

typedef float f4 __attribute__((ext_vector_type(4)));

// NCHW -> NCHWc.  One workgroup moves b channels x 256 pixels of one image: rows are read along
// the pixels (contiguous in NCHW), transposed in LDS, and written along (pixel, channel) which
// is contiguous in NCHWc.  Channels beyond C are written as zeros.
template <class V, bool TO_BLOCKED>
__global__ __launch_bounds__(256) void nchwc_kernel(const V *__restrict__ src, V *__restrict__ dst,
                                                    int C, int HW, int b, int Cb)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char tile_raw[];
    V *tile = reinterpret_cast<V *>(tile_raw);   // [b][257]
    const int t = threadIdx.x;
    const int hw0 = blockIdx.x * 256, cb = blockIdx.y, n = blockIdx.z;
    const int npix = min(256, HW - hw0);
    if (TO_BLOCKED) {
        for (int ci = 0; ci < b; ++ci) {
            int c = cb * b + ci;
            V v = 0;
            if (c < C && t < npix) v = src[((size_t)n * C + c) * HW + hw0 + t];
            tile[ci * 257 + t] = v;
        }
        __syncthreads();
        V *o = dst + (((size_t)n * Cb + cb) * HW + hw0) * b;
        for (int e = t; e < npix * b; e += 256) o[e] = tile[(e % b) * 257 + e / b];
    } else {
        const V *i = src + (((size_t)n * Cb + cb) * HW + hw0) * b;
        for (int e = t; e < npix * b; e += 256) tile[(e % b) * 257 + e / b] = i[e];
        __syncthreads();
        for (int ci = 0; ci < b; ++ci) {
            int c = cb * b + ci;
            if (c < C && t < npix) dst[((size_t)n * C + c) * HW + hw0 + t] = tile[ci * 257 + t];
        }
    }
}

// The same permutation for float tensors with 128-bit accesses on both sides: block sizes that are
// a multiple of 4 (up to 32), pixel planes a multiple of 4 floats, 16-byte aligned tensors.  One
// workgroup moves b channels x 256 pixels.  NCHW side: a thread moves four pixels of one channel;
// NCHWc side: four channels of one pixel, so consecutive threads touch consecutive 16 bytes.
// The LDS tile is [b][260]: rows stay 16-byte aligned and the strided side conflicts two-way.
template <bool TO_BLOCKED>
__global__ __launch_bounds__(256) void nchwc_wide_kernel(const float *__restrict__ src, float *__restrict__ dst,
                                                         int C, int HW, int b, int Cb)
{
    constexpr int PITCH = 260;
    extern __shared__ __attribute__((aligned(16))) unsigned char tile_raw[];
    float *tile = reinterpret_cast<float *>(tile_raw);   // [b][PITCH]
    typedef float f4 __attribute__((ext_vector_type(4)));
    const int t = threadIdx.x;
    const int hw0 = blockIdx.x * 256, cb = blockIdx.y, n = blockIdx.z;
    const int npix = min(256, HW - hw0);                 // a multiple of 4
    const int quads = b >> 2;                            // groups of four channels in a block
    const size_t blocked0 = (((size_t)n * Cb + cb) * HW + hw0) * b;
    if (TO_BLOCKED) {
        // rows of the NCHW tensor: unit u = (channel, group of four pixels)
        for (int u = t; u < b * 64; u += 256) {
            const int ci = u >> 6, g = u & 63, c = cb * b + ci;
            f4 v = {0.f, 0.f, 0.f, 0.f};
            if (c < C && g * 4 < npix) v = *reinterpret_cast<const f4 *>(src + ((size_t)n * C + c) * HW + hw0 + g * 4);
            *reinterpret_cast<f4 *>(tile + ci * PITCH + g * 4) = v;
        }
        __syncthreads();
        // blocked tensor: unit e = (pixel, group of four channels), consecutive in memory
        for (int e = t; e < npix * quads; e += 256) {
            const int px = e / quads, cj = e - px * quads;
            f4 v = {tile[(4 * cj) * PITCH + px], tile[(4 * cj + 1) * PITCH + px], tile[(4 * cj + 2) * PITCH + px],
                    tile[(4 * cj + 3) * PITCH + px]};
            *reinterpret_cast<f4 *>(dst + blocked0 + (size_t)e * 4) = v;
        }
    } else {
        for (int e = t; e < npix * quads; e += 256) {
            const int px = e / quads, cj = e - px * quads;
            const f4 v = *reinterpret_cast<const f4 *>(src + blocked0 + (size_t)e * 4);
            tile[(4 * cj) * PITCH + px] = v.x; tile[(4 * cj + 1) * PITCH + px] = v.y;
            tile[(4 * cj + 2) * PITCH + px] = v.z; tile[(4 * cj + 3) * PITCH + px] = v.w;
        }
        __syncthreads();
        for (int u = t; u < b * 64; u += 256) {
            const int ci = u >> 6, g = u & 63, c = cb * b + ci;
            if (c < C && g * 4 < npix)
                *reinterpret_cast<f4 *>(dst + ((size_t)n * C + c) * HW + hw0 + g * 4) =
                    *reinterpret_cast<const f4 *>(tile + ci * PITCH + g * 4);
        }
    }
}

// NCHW -> NCHW8c for 16-bit elements when H*W is a multiple of 8 and both tensors are 16-byte
// aligned.  One workgroup moves 8 channels x 512 pixels: a thread loads 16 bytes (8 pixels of one
// channel), the 8 x 512 tile is turned in LDS, and a thread stores 16 bytes (the 8 channels of one
// pixel): every access to memory is 128 bits wide.  Channels beyond C are zeros.
__global__ __launch_bounds__(256) void nchw8c_16bit_kernel(const uint16_t *__restrict__ src, uint16_t *__restrict__ dst,
                                                           int C, int HW, int Cb)
{
    constexpr int PIX = 512, PITCH = PIX + 8;            // pitch keeps rows 16-byte aligned
    __shared__ __attribute__((aligned(16))) uint16_t tile[8 * PITCH];
    typedef unsigned int u4 __attribute__((ext_vector_type(4)));
    const int t = threadIdx.x;
    const int hw0 = blockIdx.x * PIX, cb = blockIdx.y, n = blockIdx.z;
    const int npix = min(PIX, HW - hw0);                 // a multiple of 8
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int u = t + i * 256;                       // 8 channels x 64 groups of 8 pixels
        const int ci = u >> 6, g = u & 63, c = cb * 8 + ci;
        u4 v = {0u, 0u, 0u, 0u};
        if (c < C && g * 8 < npix) v = *reinterpret_cast<const u4 *>(src + ((size_t)n * C + c) * HW + hw0 + g * 8);
        *reinterpret_cast<u4 *>(tile + ci * PITCH + g * 8) = v;
    }
    __syncthreads();
    uint16_t *o = dst + (((size_t)n * Cb + cb) * HW + hw0) * 8;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int px = t + i * 256;
        if (px >= npix) continue;
        unsigned int w[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            w[j] = (unsigned int)tile[(2 * j) * PITCH + px] | ((unsigned int)tile[(2 * j + 1) * PITCH + px] << 16);
        u4 v = {w[0], w[1], w[2], w[3]};
        *reinterpret_cast<u4 *>(o + (size_t)px * 8) = v;
    }
}

// KCRS -> KCRSck: one thread per element of the blocked tensor (weights are small and packed
// once per tensor).  Elements whose channel indices fall beyond K or C are zeros.
template <class V>
__global__ void kcrsck_kernel(const V *__restrict__ wt, V *__restrict__ dst, int K, int C, int RS,
                              int bc, int bk, int Cb, size_t total)
{
    size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (o >= total) return;
    int ki = (int)(o % bk);
    size_t r1 = o / bk;
    int ci = (int)(r1 % bc);
    size_t r2 = r1 / bc;
    int rs = (int)(r2 % RS);
    size_t r3 = r2 / RS;
    int cblk = (int)(r3 % Cb);
    int kblk = (int)(r3 / Cb);
    int k = kblk * bk + ki, c = cblk * bc + ci;
    dst[o] = (k < K && c < C) ? wt[((size_t)k * C + c) * RS + rs] : (V)0;
}

// y[n][k][pq] += bias[k], in place.
__global__ void bias_add_kernel(float *__restrict__ y, const float *__restrict__ bias, int K, int PQ, size_t total)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t step = (size_t)gridDim.x * blockDim.x;
    for (; i < total; i += step) y[i] += bias[(i / PQ) % K];
}

// y = max(y, 0) or min(max(y, 0), 6), in place; 128-bit accesses on the aligned body.
__global__ void act_kernel(float *__restrict__ y, size_t total, int act)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t step = (size_t)gridDim.x * blockDim.x;
    size_t n4 = (((uintptr_t)y & 15) == 0) ? total / 4 : 0;
    f4 *y4 = reinterpret_cast<f4 *>(y);
    for (size_t j = i; j < n4; j += step) {
        f4 v = y4[j];
        for (int c = 0; c < 4; ++c) {
            float x = fmaxf(v[c], 0.f);
            v[c] = act == POLYDL_ACT_RELU6 ? fminf(x, 6.f) : x;
        }
        y4[j] = v;
    }
    for (size_t j = n4 * 4 + i; j < total; j += step) {
        float x = fmaxf(y[j], 0.f);
        y[j] = act == POLYDL_ACT_RELU6 ? fminf(x, 6.f) : x;
    }
}

// Inference batch normalisation with an optional activation in the same pass:
// y = act(gamma[k] * (x - mean[k]) / sqrt(var[k] + eps) + beta[k]) on an NKPQ tensor (y may be x).
// One thread handles four consecutive elements of one (n, k) plane when planes are a multiple of
// four floats and both tensors are 16-byte aligned, else one element.  Bound by HBM: one read and
// one write per element (the two integer divisions per thread are far below the ALU rate).
template <int V>
__global__ void bnorm_act_kernel(const float *__restrict__ x, float *__restrict__ y, const float *__restrict__ gamma,
                                 const float *__restrict__ beta, const float *__restrict__ mean,
                                 const float *__restrict__ var, float eps, uint32_t K, uint32_t PQ, uint32_t units,
                                 int act)
{
    uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    const uint32_t step = gridDim.x * blockDim.x;
    for (; i < units; i += step) {
        const uint32_t e = i * V;
        const uint32_t k = (e / PQ) % K;
        const float inv = 1.0f / sqrtf(var[k] + eps);
        const float g = gamma[k], m = mean[k], b = beta[k];
        float v[V];
        if constexpr (V == 4) {
            f4 t = *reinterpret_cast<const f4 *>(x + e);
            for (int c = 0; c < 4; ++c) v[c] = t[c];
        } else {
            v[0] = x[e];
        }
        for (int c = 0; c < V; ++c) {
            float r = g * ((v[c] - m) * inv) + b;
            if (act != POLYDL_ACT_NONE) r = fmaxf(r, 0.f);
            if (act == POLYDL_ACT_RELU6) r = fminf(r, 6.f);
            v[c] = r;
        }
        if constexpr (V == 4) {
            f4 t = {v[0], v[1], v[2], v[3]};
            *reinterpret_cast<f4 *>(y + e) = t;
        } else {
            y[e] = v[0];
        }
    }
}

hipError_t launch_bnorm_act(const float *x, float *y, const float *gamma, const float *beta, const float *mean,
                            const float *var, float eps, int K, int PQ, size_t total, int act, hipStream_t st)
{
    hipError_t le = hipSuccess;
    const bool vec = PQ % 4 == 0 && (((uintptr_t)x | (uintptr_t)y) & 15) == 0;
    const uint32_t units = (uint32_t)(vec ? total / 4 : total);
    const unsigned blocks = (unsigned)((units + 255) / 256 < 16384 ? (units + 255) / 256 : 16384);
    if (vec)
        le = launch_kernel((bnorm_act_kernel<4>), dim3(blocks), dim3(256), 0, st, x, y, gamma, beta, mean, var, eps,
                           (uint32_t)K, (uint32_t)PQ, units, act);
    else
        le = launch_kernel((bnorm_act_kernel<1>), dim3(blocks), dim3(256), 0, st, x, y, gamma, beta, mean, var, eps,
                           (uint32_t)K, (uint32_t)PQ, units, act);
    return le;
}

// elem_bytes: 4 (float) or 2 (bfloat16 bit patterns; a permutation does not look at the values)
hipError_t launch_nchwc(const void *src, void *dst, int N, int C, int HW, int b, bool to_blocked, int elem_bytes,
                        hipStream_t st)
{
    hipError_t le = hipSuccess;
    int Cb = (C + b - 1) / b;
    dim3 grid((unsigned)((HW + 255) / 256), (unsigned)Cb, (unsigned)N);
    size_t lds = (size_t)b * 257 * elem_bytes;
    if (elem_bytes == 4) {
        const float *s = static_cast<const float *>(src);
        float *d = static_cast<float *>(dst);
        if (b % 4 == 0 && HW % 4 == 0 && ((uintptr_t)src & 15) == 0 && ((uintptr_t)dst & 15) == 0) {
            const size_t wide_lds = (size_t)b * 260 * sizeof(float);
            if (to_blocked) le = launch_kernel((nchwc_wide_kernel<true>), grid, dim3(256), wide_lds, st, s, d, C, HW, b, Cb);
            else le = launch_kernel((nchwc_wide_kernel<false>), grid, dim3(256), wide_lds, st, s, d, C, HW, b, Cb);
            return le;
        }
        if (to_blocked) le = launch_kernel((nchwc_kernel<float, true>), grid, dim3(256), lds, st, s, d, C, HW, b, Cb);
        else le = launch_kernel((nchwc_kernel<float, false>), grid, dim3(256), lds, st, s, d, C, HW, b, Cb);
    } else {
        const uint16_t *s = static_cast<const uint16_t *>(src);
        uint16_t *d = static_cast<uint16_t *>(dst);
        if (to_blocked && b == 8 && HW % 8 == 0 && ((uintptr_t)src & 15) == 0 && ((uintptr_t)dst & 15) == 0) {
            dim3 g8((unsigned)((HW + 511) / 512), (unsigned)Cb, (unsigned)N);
            le = launch_kernel(nchw8c_16bit_kernel, g8, dim3(256), 0, st, s, d, C, HW, Cb);
            return le;
        }
        if (to_blocked) le = launch_kernel((nchwc_kernel<uint16_t, true>), grid, dim3(256), lds, st, s, d, C, HW, b, Cb);
        else le = launch_kernel((nchwc_kernel<uint16_t, false>), grid, dim3(256), lds, st, s, d, C, HW, b, Cb);
    }
    return le;
}

hipError_t launch_kcrsck(const void *wt, void *dst, int K, int C, int RS, int bc, int bk, int elem_bytes,
                         hipStream_t st)
{
    hipError_t le = hipSuccess;
    int Kb = (K + bk - 1) / bk, Cb = (C + bc - 1) / bc;
    size_t total = (size_t)Kb * Cb * RS * bc * bk;
    dim3 grid((unsigned)((total + 255) / 256));
    if (elem_bytes == 4)
        le = launch_kernel(kcrsck_kernel<float>, grid, dim3(256), 0, st, static_cast<const float *>(wt),
                           static_cast<float *>(dst), K, C, RS, bc, bk, Cb, total);
    else
        le = launch_kernel(kcrsck_kernel<uint16_t>, grid, dim3(256), 0, st, static_cast<const uint16_t *>(wt),
                           static_cast<uint16_t *>(dst), K, C, RS, bc, bk, Cb, total);
    return le;
}

hipError_t launch_bias_add(float *y, const float *bias, int K, int PQ, size_t total, hipStream_t st)
{
    hipError_t le = hipSuccess;
    unsigned blocks = (unsigned)((total + 255) / 256 < 8192 ? (total + 255) / 256 : 8192);
    le = launch_kernel(bias_add_kernel, dim3(blocks), dim3(256), 0, st, y, bias, K, PQ, total);
    return le;
}

hipError_t launch_act(float *y, size_t total, int act, hipStream_t st)
{
    hipError_t le = hipSuccess;
    size_t work = (total + 3) / 4;
    unsigned blocks = (unsigned)((work + 255) / 256 < 8192 ? (work + 255) / 256 : 8192);
    le = launch_kernel(act_kernel, dim3(blocks), dim3(256), 0, st, y, total, act);
    return le;
}

}  // namespace polydl
