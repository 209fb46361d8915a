// Pointwise convolution (R = S = 1, stride 1, no padding) with few input channels: the loop nest
// of figure "The 2-D Convolution code" (section "Convolutions") degenerates to
//   out[n][k][x] = sum_c wt[k][c] * in[n][c][x],   x = 0 .. H*W-1,
// a GEMM whose reduction (C <= 64) is so short that staging pixels through LDS, a barrier per
// stage and a tile prologue per workgroup cost more than the arithmetic.  Here
//   * the whole filter matrix sits in LDS for the life of the workgroup (K*C*4 <= 64 KB), laid
//     out so that a lane reads the four weights of four consecutive rank-2 updates as one vector;
//   * a wave owns 64 pixels at a time and loads their C channels from global memory straight
//     into the registers the matrix instruction reads -- lane j of each half-wave holds pixels
//     2j and 2j+1 (one 8-byte load per channel pair), the half-waves hold even and odd channels;
//   * with those registers it produces the output channels in groups of 32 (accumulators: two
//     blocks of 32x32, one per pixel of the lane's pair; groups of 64 measured 10 % slower), bias
//     and activation applied on the way out (section "Operator Fusion"), each lane storing its
//     two pixels of a channel row as one 8-byte store;
//   * (pixel tile, channel group) units are dealt to the waves of a grid that fits the chip once
//     in contiguous, equal runs, so a wave reloads pixels only when its run crosses a tile.
// No barrier after the filter is in LDS; waves never wait for each other.
#include <hip/hip_runtime.h>
#include "gemm_core.hpp"
#include "internal.hpp"

namespace polydl {

struct ConvPointKArgs {
    const float *in, *wt, *bias;
    float *out;
    int N, C, K, HW;
    int groups;             // K / 32
    uint32_t units;         // pixel tiles * groups
    uint32_t per, rem;      // units per wave; the first rem waves take one more
    uint32_t recip_groups, recip_HW;
    int act;
};

__device__ __forceinline__ v2f buf_load2(__amdgpu_buffer_rsrc_t r, uint32_t byte_off, uint32_t uniform_off)
{
    typedef int v2i __attribute__((ext_vector_type(2)));
    v2i v = __builtin_amdgcn_raw_buffer_load_b64(r, (int)byte_off, (int)uniform_off, 0);
    return __builtin_bit_cast(v2f, v);
}

// What a finished unit leaves behind until it is stored: its two accumulator blocks, the lane's 16
// bias values of its channel group, the lane's output offset and the group's first channel.
struct PointUnit {
    v16f acc[2];
    v4f bias[4];
    uint32_t vo;
    int k0;
};

// Stores first .. first + count - 1 (of 16) of a finished unit: accumulator registers 4q .. 4q+3 are
// four consecutive channels, the lane's two pixels of a channel row go out as one 8-byte store.
// Called from fully unrolled loops only, so every index is a constant.
template <int ACT>
__device__ __forceinline__ void point_store(__amdgpu_buffer_rsrc_t ro, uint32_t row_bytes, const PointUnit &u,
                                            int first, int count)
{
#pragma unroll
    for (int r = first; r < first + count; ++r) {
        const int q = r >> 2, i = r & 3;
        v2f v = {act_of<ACT>(u.acc[0][r] + u.bias[q][i]), act_of<ACT>(u.acc[1][r] + u.bias[q][i])};
        buf_store2(ro, u.vo, (uint32_t)(u.k0 + 8 * q + i) * row_bytes, v);
    }
}

// The products of one unit into `cur` and, PENDING, the 16 stores of the unit finished before it
// (`old`) dealt out between the groups of eight matrix instructions: a wave's stores leave while
// its own next matrix instructions run instead of after them, in a phase of their own in which
// the matrix core of the SIMD has nothing to do unless another wave happens to be out of step.
template <int C8, int ACT, bool PENDING>
__device__ __forceinline__ void point_unit(const v4f *a_base, int K, const v2f (&b)[C8 * 4], PointUnit &cur,
                                           __amdgpu_buffer_rsrc_t ro, uint32_t row_bytes, const PointUnit &old)
{
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) cur.acc[nb][r] = 0.f;
    constexpr int PER = 16 / C8;   // stores per group of eight matrix instructions
#pragma unroll
    for (int sg = 0; sg < C8; ++sg) {
        const v4f a = a_base[sg * 2 * K];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            cur.acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[4 * sg + i].x, cur.acc[0], 0, 0, 0);
            cur.acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[4 * sg + i].y, cur.acc[1], 0, 0, 0);
        }
        if constexpr (PENDING) {
            point_store<ACT>(ro, row_bytes, old, sg * PER, PER);
            // keep the stores where they are: left alone, the scheduler moves them all behind the
            // last matrix instruction
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// A wave's run of units [u, end).  Two unit records take turns: while one collects the products of
// unit i, the other, holding unit i - 1, is stored.
template <int C8, int ACT>
__device__ __forceinline__ void point_run(const ConvPointKArgs &p, const v4f *At, uint32_t u, uint32_t end, int half, int j)
{
    const int K = p.K, C = C8 * 8;
    const uint32_t HW = p.HW, total = (uint32_t)p.N * HW;
    const __amdgpu_buffer_rsrc_t ri = make_rsrc(p.in, (uint64_t)total * C * 4);
    const __amdgpu_buffer_rsrc_t ro = make_rsrc(p.out, (uint64_t)total * K * 4);
    const __amdgpu_buffer_rsrc_t rb = make_rsrc(p.bias, p.bias ? (uint64_t)K * 4 : 0);
    const uint32_t row_bytes = HW * 4u;

    uint32_t g;
    uint32_t tile = div_by(u, (uint32_t)p.groups, p.recip_groups, g);
    uint32_t have = 0xFFFFFFFFu, vo = kOobOffset;
    v2f b[C8 * 4];
    // pixels of a new tile, the unit's output offset and channel group, its bias values (zeros
    // without a bias; they are needed only when the unit is stored, one unit later)
    auto open_unit = [&](PointUnit &cur) {
        if (tile != have) {
            // the lane's two pixels: 2j and 2j+1 of the tile, in one image since H*W is even
            const uint32_t pix0 = tile * 64u + 2u * j;
            uint32_t x;
            const uint32_t n = div_by(pix0, HW, p.recip_HW, x);
            const bool ok = pix0 < total;
            const uint32_t vi = ok ? ((n * C + half) * HW + x) * 4u : kOobOffset;
            vo = ok ? ((n * K + 4u * half) * HW + x) * 4u : kOobOffset;
#pragma unroll
            for (int s = 0; s < C8 * 4; ++s) b[s] = buf_load2(ri, vi, (uint32_t)(2 * s) * row_bytes);
            have = tile;
        }
        cur.vo = vo;
        cur.k0 = (int)g * 32;
#pragma unroll
        for (int q = 0; q < 4; ++q) cur.bias[q] = buf_load4(rb, (uint32_t)(g * 32 + 8 * q + 4 * half) * 4u);
    };
    auto next_unit = [&]() {
        if (++g == (uint32_t)p.groups) { g = 0; ++tile; }
    };
    PointUnit A, B;
    uint32_t left = end - u;
    open_unit(A);
    point_unit<C8, ACT, false>(At + half * K + g * 32 + j, K, b, A, ro, row_bytes, A);
    next_unit();
    --left;
    while (left >= 2) {
        open_unit(B);
        point_unit<C8, ACT, true>(At + half * K + g * 32 + j, K, b, B, ro, row_bytes, A);
        next_unit();
        open_unit(A);
        point_unit<C8, ACT, true>(At + half * K + g * 32 + j, K, b, A, ro, row_bytes, B);
        next_unit();
        left -= 2;
    }
    if (left == 1) {
        open_unit(B);
        point_unit<C8, ACT, true>(At + half * K + g * 32 + j, K, b, B, ro, row_bytes, A);
        point_store<ACT>(ro, row_bytes, B, 0, 16);
    } else {
        point_store<ACT>(ro, row_bytes, A, 0, 16);
    }
}

// C8 = C / 8.  256 threads; LDS holds wt as float4 At[C8][2][K]:
// At[sg][h][k] = wt[k][8 sg + h + {0, 2, 4, 6}].
template <int C8>
__global__ __launch_bounds__(256, 2) void conv_point_kernel(const ConvPointKArgs p)
{
    __shared__ v4f At[4096];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // the same in all lanes: keeps unit bookkeeping scalar
    const int half = lane >> 5, j = lane & 31;
    const int K = p.K, C = C8 * 8;

    {
        // filter rows are read as they lie (16 bytes per lane, consecutive lanes consecutive addresses)
        // and scattered into the layout above one scalar at a time
        const __amdgpu_buffer_rsrc_t rw = make_rsrc(p.wt, (uint64_t)K * C * 4);
        float *At1 = reinterpret_cast<float *>(At);
        const int count = K * C8 * 2;                       // float4 units of wt
        for (int idx = tid; idx < count; idx += 256) {
            const int k = idx / (C8 * 2), c0 = (idx - k * (C8 * 2)) * 4;
            const v4f v = buf_load4(rw, (uint32_t)idx * 16u);
            const int sg = c0 >> 3, e0 = (c0 & 7) >> 1;     // c0 is a multiple of 4: components e0 and e0 + 1
            float *even = At1 + ((sg * 2 + 0) * K + k) * 4 + e0, *odd = At1 + ((sg * 2 + 1) * K + k) * 4 + e0;
            even[0] = v[0];
            odd[0] = v[1];
            even[1] = v[2];
            odd[1] = v[3];
        }
    }
    __syncthreads();

    const uint32_t w = blockIdx.x * 4u + wave;
    const uint32_t u = w * p.per + (w < p.rem ? w : p.rem);
    const uint32_t end = u + p.per + (w < p.rem ? 1u : 0u);
    if (u >= end) return;
    if (p.act == POLYDL_ACT_NONE) point_run<C8, POLYDL_ACT_NONE>(p, At, u, end, half, j);
    else if (p.act == POLYDL_ACT_RELU) point_run<C8, POLYDL_ACT_RELU>(p, At, u, end, half, j);
    else point_run<C8, POLYDL_ACT_RELU6>(p, At, u, end, half, j);
}

bool conv_point_fits(const ConvProblem &q)
{
    const int64_t HW = (int64_t)q.H * q.W;
    if (q.R != 1 || q.S != 1 || q.stride != 1 || q.pad != 0 || q.pre_act != POLYDL_ACT_NONE) return false;
    if (q.C != 16 && q.C != 32 && q.C != 64) return false;
    // at least four channel groups share the pixels a wave holds (with 64 output channels the kernel
    // measured no faster than the staged one); the filter has to fit the 64 KB of LDS
    if (q.K % 64 != 0 || q.K < 128 || (int64_t)q.K * q.C > 16384) return false;
    if (HW % 2 != 0) return false;
    // every byte offset, tile base and unit count stays below 2^31
    if ((int64_t)q.N * HW * q.C * 4 >= 0x7FFFFFF0ll || (int64_t)q.N * HW * q.K * 4 >= 0x7FFFFFF0ll) return false;
    return true;
}

// waves of the grid and units per wave for this problem
void conv_point_shape(const ConvProblem &q, int cus, uint32_t *units, uint32_t *workgroups)
{
    const int64_t total = (int64_t)q.N * q.H * q.W;
    const uint32_t tiles = (uint32_t)((total + 63) / 64);
    *units = tiles * (uint32_t)(q.K / 32);
    const uint32_t fit = (uint32_t)cus * 2u;                 // two workgroups per compute unit (LDS)
    const uint32_t need = (*units + 3) / 4;
    *workgroups = need < fit ? need : fit;
}

hipError_t conv_point_launch(const ConvProblem &q, hipStream_t stream)
{
    if (!conv_point_fits(q)) return hipErrorInvalidValue;
    ConvPointKArgs a;
    a.in = (const float *)q.in; a.wt = (const float *)q.wt; a.bias = q.bias; a.out = q.out;
    a.N = q.N; a.C = q.C; a.K = q.K; a.HW = q.H * q.W;
    a.groups = q.K / 32;
    uint32_t wgs;
    conv_point_shape(q, compute_units(), &a.units, &wgs);
    const uint32_t waves = wgs * 4;
    a.per = a.units / waves;
    a.rem = a.units % waves;
    a.recip_groups = div_recip((uint32_t)a.groups);
    a.recip_HW = div_recip((uint32_t)a.HW);
    a.act = q.act;
    hipError_t le = hipSuccess;
    if (q.C == 64) le = launch_kernel(conv_point_kernel<8>, dim3(wgs), dim3(256), 0, stream, a);
    else if (q.C == 32) le = launch_kernel(conv_point_kernel<4>, dim3(wgs), dim3(256), 0, stream, a);
    else le = launch_kernel(conv_point_kernel<2>, dim3(wgs), dim3(256), 0, stream, a);
    return le;
}

}  // namespace polydl
