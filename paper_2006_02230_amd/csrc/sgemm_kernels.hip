// SGEMM C += A*B on the fp32 matrix cores (figure "Matrix multiplication code", section
// "Notation"; two-level tiling as in figure "A code version generated for PolyDL").
#include "gemm_core.hpp"
#include "internal.hpp"
#include "variants.hpp"
#include <type_traits>

namespace polydl {

struct SgemmKArgs {
    const float *A, *B;
    float *C;
    int M, N, K;
    int tiles_m, tiles_n;
    int split_k, k_per_split;  // k_per_split is a multiple of the stage depth
    int raster;
    float alpha, beta;         // C = beta*C + alpha*A*B; beta == 0 writes C without reading it
    float *partials;           // split_k > 1: [tile][part][BM*BN] accumulator tiles in register order
    unsigned *counters;        // split_k > 1: per tile, how many of its reduction parts have finished
};

// AVEC / BVEC: 4 when the operand allows 128-bit loads, else 1.  CVEC: the lane's NB adjacent
// output columns are read and written as one vector when N % NB == 0 and C is 16-byte aligned.
template <class T, int AVEC, int BVEC, bool CVEC>
__global__ __launch_bounds__(T::NT, T::MIN_WAVES) void sgemm_kernel(SgemmKArgs p)
{
    __shared__ __attribute__((aligned(16))) float lds[T::LDS_FLOATS];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int tm, tn;
    tile_coords(blockIdx.x, p.raster, p.tiles_m, p.tiles_n, tm, tn);
    const int m0 = tm * T::BM, n0 = tn * T::BN;
    const int wm0 = (wave % T::WAVES_M) * T::WM, wn0 = (wave / T::WAVES_M) * T::WN;
    const int kbegin = blockIdx.y * p.k_per_split;
    const int kend = min(p.K, kbegin + p.k_per_split);

    ALoader<T, AVEC> al;
    BLoaderRows<T, BVEC> bl;
    al.init(p.A, tid, m0, p.M, p.K, p.K);
    bl.init(p.B, tid, n0, p.N, p.K, p.N);

    v16f acc[T::MB][T::NB];
#pragma unroll
    for (int bi = 0; bi < T::MB; ++bi)
#pragma unroll
        for (int bj = 0; bj < T::NB; ++bj)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[bi][bj][r] = 0.f;

    if (kbegin < kend) gemm_mainloop<T, T::SPLIT_STAGE>(lds, al, bl, acc, kbegin, kend, tid, wm0, wn0);

    // With the reduction split over blockIdx.y every part leaves its accumulator tile in scratch
    // memory (thread-contiguous, device-scope stores); the part that arrives last adds all parts
    // in index order and alone updates C, so the result does not depend on the order of arrival.
    // Nothing waits on another workgroup.
    if (p.split_k > 1) {
        __shared__ unsigned s_arrived;
        constexpr size_t TILE = (size_t)T::BM * T::BN;
        constexpr int NT = T::NT;
        float *tile0 = p.partials + (size_t)blockIdx.x * p.split_k * TILE;
        float *mine = tile0 + (size_t)blockIdx.y * TILE;
#pragma unroll
        for (int bi = 0; bi < T::MB; ++bi)
#pragma unroll
            for (int bj = 0; bj < T::NB; ++bj)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    __hip_atomic_store(mine + ((bi * T::NB + bj) * 16 + r) * NT + tid, acc[bi][bj][r], __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
        wait_vmcnt0();   // vmcnt(0): this wave's device-scope stores have completed
        __syncthreads();
        if (tid == 0)
            s_arrived = __hip_atomic_fetch_add(p.counters + blockIdx.x, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (__builtin_amdgcn_readfirstlane(s_arrived) != (unsigned)p.split_k - 1u) return;   // not the last part
        if (tid == 0)               // leave the counter at zero for the next launch
            __hip_atomic_store(p.counters + blockIdx.x, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sum_partial_tiles<T>(tile0, p.split_k, TILE, tid, acc);
    }
    // epilogue: C = beta*C + alpha*acc (alpha = beta = 1 rounds exactly like C += acc).  C is
    // addressed by a per-lane byte offset of the lane's first row and column inside the tile's row
    // panel plus a uniform offset per accumulator row, so a row costs no address arithmetic.
    const int col = n0 + wn0 + T::NB * (lane & 31);
    if (col >= p.N) return;
    const int krow = wm0 + 4 * (lane >> 5);   // row inside the tile of register 0; register r adds 8*(r/4) + r%4
    const uint64_t panel = (uint64_t)m0 * p.N * 4;
    __amdgpu_buffer_rsrc_t rc = make_rsrc(reinterpret_cast<char *>(p.C) + panel, (uint64_t)p.M * p.N * 4 - panel);
    const uint32_t off = ((uint32_t)krow * (uint32_t)p.N + (uint32_t)col) * 4u;
    const uint32_t row_bytes = (uint32_t)p.N * 4u;
    const float alpha = p.alpha, beta = p.beta;
    const bool readc = beta != 0.f;              // uniform
    const bool full = m0 + T::BM <= p.M;         // uniform: every row of the tile exists
    auto rows = [&](auto full_tag) __attribute__((always_inline)) {
        constexpr bool FULL = decltype(full_tag)::value;
#pragma unroll
        for (int bi = 0; bi < T::MB; ++bi)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int c = 32 * bi + 8 * (r >> 2) + (r & 3);
                if (!FULL && m0 + krow + c >= p.M) continue;
                const uint32_t uo = (uint32_t)c * row_bytes;
                if constexpr (CVEC && T::NB == 4) {
                    v4f v = {0.f, 0.f, 0.f, 0.f};
                    if (readc) v = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rc, (int)off, (int)uo, 0));
                    v.x = beta * v.x + alpha * acc[bi][0][r]; v.y = beta * v.y + alpha * acc[bi][1][r];
                    v.z = beta * v.z + alpha * acc[bi][2][r]; v.w = beta * v.w + alpha * acc[bi][3][r];
                    buf_store4(rc, off, uo, v);
                } else if constexpr (CVEC && T::NB == 2) {
                    v2f v = {0.f, 0.f};
                    if (readc) v = __builtin_bit_cast(v2f, __builtin_amdgcn_raw_buffer_load_b64(rc, (int)off, (int)uo, 0));
                    v.x = beta * v.x + alpha * acc[bi][0][r]; v.y = beta * v.y + alpha * acc[bi][1][r];
                    buf_store2(rc, off, uo, v);
                } else {
#pragma unroll
                    for (int bj = 0; bj < T::NB; ++bj)
                        if (col + bj < p.N) {
                            const float c0 = readc ? buf_load1(rc, off + 4u * bj, uo) : 0.f;
                            buf_store1(rc, off + 4u * bj, uo, beta * c0 + alpha * acc[bi][bj][r]);
                        }
                }
            }
    };
    if (full) rows(std::true_type{});
    else rows(std::false_type{});
}

template <class T>
static hipError_t sgemm_launch(const SgemmProblem &q, int split_k, int raster, hipStream_t stream)
{
    SgemmKArgs a;
    a.A = q.A; a.B = q.B; a.C = q.C;
    a.M = q.M; a.N = q.N; a.K = q.K;
    a.tiles_m = (q.M + T::BM - 1) / T::BM;
    a.tiles_n = (q.N + T::BN - 1) / T::BN;
    int stages = (q.K + T::BK - 1) / T::BK;
    if (split_k < 1) split_k = 1;
    if (split_k > stages) split_k = stages > 0 ? stages : 1;
    int stages_per = (stages + split_k - 1) / split_k;
    if (stages_per < 1) stages_per = 1;
    a.k_per_split = stages_per * T::BK;
    split_k = stages > 0 ? (stages + stages_per - 1) / stages_per : 1;
    a.split_k = split_k;
    a.raster = raster;
    a.alpha = q.alpha; a.beta = q.beta;
    a.partials = nullptr;
    a.counters = nullptr;
    hipError_t le = hipSuccess;
    if (split_k > 1) {
        const size_t bytes = (size_t)a.tiles_m * a.tiles_n * split_k * T::BM * T::BN * sizeof(float);
        hipError_t e = splitk_scratch(stream, q.arena, bytes, a.tiles_m * a.tiles_n, &a.partials, &a.counters);
        if (e != hipSuccess) return e;
    }
    dim3 grid((unsigned)(a.tiles_m * a.tiles_n), (unsigned)split_k), block(T::NT);
    const bool avec = (q.K % 4 == 0) && ((uintptr_t)q.A % 16 == 0);
    const bool bvec = (q.N % 4 == 0) && ((uintptr_t)q.B % 16 == 0);
    const bool cvec = (q.N % T::NB == 0) && ((uintptr_t)q.C % 16 == 0);
#define POLYDL_GO(AV, BV, CV) le = launch_kernel((sgemm_kernel<T, AV, BV, CV>), grid, block, 0, stream, a)
    if (avec && bvec && cvec) POLYDL_GO(4, 4, true);
    else if (avec && bvec) POLYDL_GO(4, 4, false);
    else if (avec && cvec) POLYDL_GO(4, 1, true);
    else if (avec) POLYDL_GO(4, 1, false);
    else if (bvec && cvec) POLYDL_GO(1, 4, true);
    else if (bvec) POLYDL_GO(1, 4, false);
    else if (cvec) POLYDL_GO(1, 1, true);
    else POLYDL_GO(1, 1, false);
#undef POLYDL_GO
    return le;
}

#define POLYDL_DEFINE_SGEMM(BM, BN, BK, WM, WN)                                                            \
    hipError_t sgemm_launch_##BM##x##BN##x##BK##_##WM##x##WN(const SgemmProblem &q, int s, int r,          \
                                                             hipStream_t st)                              \
    {                                                                                                     \
        return sgemm_launch<Tile<BM, BN, BK, WM, WN>>(q, s, r, st);                                        \
    }
POLYDL_TILE_FAMILY(POLYDL_DEFINE_SGEMM)

}  // namespace polydl
