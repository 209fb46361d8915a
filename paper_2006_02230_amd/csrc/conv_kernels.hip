// Forward convolution as an implicit GEMM on the fp32 matrix cores.
//
// The paper's convolution nest (figure "The 2-D Convolution code") contains a GEMM in its three
// inner loops; here the whole nest is one GEMM  out[K][N*P*Q] = wt[K][C*R*S] * X[C*R*S][N*P*Q]
// where X is the im2col view of the input, never materialised: its elements are gathered from
// the NCHW tensor while the B stage is filled.  Rows (output channels) come from the KCRS filter
// tensor, which already is a row-major K x (C*R*S) matrix.  Output columns (n, p, q) are
// contiguous in NKPQ for a fixed channel, so the accumulator tile is stored without a transpose.
// The element-wise tail (bias, ReLU / ReLU6) runs on the accumulators before the store: the
// peeled last reduction iteration of algorithm "Perform operator fusion".
#include "gemm_core.hpp"
#include "internal.hpp"
#include "variants.hpp"

namespace polydl {

struct ConvKArgs {
    const float *in, *wt, *bias;
    float *out;
    int C, H, W, K, R, S, stride, pad, P, Q;
    int PQ, RS, HW, CHW;
    int Kg, Ng;                 // reduction length C*R*S, number of output pixels N*P*Q
    uint32_t magic_C;           // GATHER_TAPMAJOR: exact division of a reduction index by C (C > 1)
    uint32_t magic_RS, magic_S; // exact division of a reduction index by R*S and by S,
    uint32_t one_RS, one_S;     // see fast_div(): magic multiplier and the all-ones mask for d == 1
    uint32_t recip_PQ, recip_Q; // for div_by(): pixel index -> (image, row, column)
    uint64_t in_bytes, out_bytes;
    int tiles_m, tiles_n;
    int split_k, k_per_split;
    // tail_parts > 1: one-dimensional grid; the first whole_tiles tiles run their reduction whole,
    // each later tile in tail_parts parts of tail_k reduction elements
    int whole_tiles, tail_parts, tail_k;
    uint32_t recip_tail;
    int raster, act;
    int pre_act;                // activation applied to every input element as its stage is filled
    float *partials;            // split_k > 1: [tile][part][BM*BN] accumulator tiles in register order
    unsigned *counters;         // split_k > 1: per tile, how many of its reduction parts have finished
};

// ---- B operand: on-the-fly im2col gather from NCHW --------------------------------------------
// A thread owns one output pixel (one column of the stage) for the whole reduction; per stage it
// loads BK / (NT/BN) reduction rows of that column.  The reduction row is the same for all lanes
// of a wave, so its split into (c, r, s) is scalar work.  Whether tap (r, s) falls inside the
// image for this pixel is kept as one bit per filter row and per filter column.
// n / d without a branch: (n * magic) >> 32 is exact for n*d < 2^32 when d > 1; for d == 1 the
// magic is 0 and the all-ones mask passes n through.
__device__ __forceinline__ uint32_t fast_div(uint32_t n, uint32_t magic, uint32_t ones_if_d1)
{
    return __umulhi(n, magic) + (n & ones_if_d1);
}

__device__ __forceinline__ uint32_t low_bits(int n) { return (uint32_t)((1ull << n) - 1ull); }   // 0 <= n <= 32
// Bits i of 0 .. n-1 with i < lo or i >= hi (n <= 32).
__device__ __forceinline__ uint32_t outside_bits(int lo, int hi, int n)
{
    lo = min(max(lo, 0), n);
    hi = min(max(hi, 0), n);
    return low_bits(lo) | (low_bits(n) & ~low_bits(hi));
}

// How a load finds its element and whether it lies inside the image:
//  GATHER_ANY   any filter: per-lane row and column bit masks, offset built per lane;
//  GATHER_POINT 1x1 filters without padding: reduction row k is channel k and every tap lies inside
//               the image, so the lane keeps the byte offset of its pixel and the channel offset
//               rides in the instruction's uniform offset -- no per-lane arithmetic per load;
//  GATHER_TAPS1 / GATHER_TAPS2  filters of at most 31 / 63 taps: the lane keeps one bit per tap
//               (set: outside the image) in one / two registers and the byte offset of tap (0,0);
//               the tap's distance is uniform and rides in the uniform offset, so a load costs a
//               bit extract and a merge of that bit into the top of the offset.
//  GATHER_TAPMAJOR  filters of 2 .. 63 taps whose channel count is a multiple of the stage depth, with
//               a second copy of the filter in the blocked layout [K][R][S][C] (KCRSck with
//               bc = C, bk = 1): the reduction is walked tap by tap, all channels of a tap before
//               the next tap (the order is free, section "Microkernel Specification"), so a whole
//               stage shares one tap: its validity bit and its distance are found once per stage,
//               not per element, and the channel rides in the uniform offset.  In that copy the
//               filter rows are contiguous in the walked order, so they load as in a plain GEMM.
//  GATHER_TABLE  filters of at most 63 taps with a short reduction (C*R*S + 2 stages at most kTableRows
//               rows; the stem layer): as GATHER_TAPS2, but the (c, r, s) split of a reduction row is
//               not redone by every wave for every element.  The workgroup writes (distance of the
//               row's tap and channel in bytes, tap number) of every row into LDS once; a load then
//               reads its row's entry (one address per stage, constant offsets), adds the distance
//               to the lane's offset and shifts the lane's 64 tap bits by the tap number.  Same
//               vector instructions per element as GATHER_TAPS2, a tenth of its scalar ones: the one
//               scalar unit of a compute unit serves four SIMDs, and at 18 scalar instructions per
//               matrix instruction (the stem layer) it, not the matrix cores, set the pace.
enum { GATHER_ANY = 0, GATHER_POINT = 1, GATHER_TAPS1 = 2, GATHER_TAPS2 = 3, GATHER_TAPMAJOR = 4, GATHER_TABLE = 5 };
constexpr int kTableRows = 512;   // 4 KB of LDS


template <class T, int MODE>
struct BLoaderIm2col {
    static constexpr bool POINT = MODE == GATHER_POINT;
    static constexpr bool TAPMAJOR = MODE == GATHER_TAPMAJOR;
    static constexpr bool TABLE = MODE == GATHER_TABLE;
    static constexpr bool TAPS = MODE == GATHER_TAPS1 || MODE == GATHER_TAPS2 || TAPMAJOR || TABLE;
    static constexpr int LAST_BIT = MODE == GATHER_TAPS1 ? 31 : 63;   // never a tap: always set
    static constexpr int KSTEP = T::NT / T::BN;  // reduction rows covered by one pass of the workgroup
    static constexpr int ITERS = T::BK / KSTEP;
    static_assert(T::BK % KSTEP == 0, "stage depth must be a multiple of the rows loaded per pass");
    float regs[2][ITERS];
    __amdgpu_buffer_rsrc_t rsrc;
    int pix_off;      // element offset of tap (0,0), channel 0 of this pixel from the descriptor base
    uint32_t rmask, smask;   // GATHER_TAPS*: the tap bits 0-31 and 32-63
    int krow0, lds_off;
    int RS, S, HW, W, pre_act, C;
    uint32_t magic_RS, magic_S, one_RS, one_S, magic_C;
    const uint2 *tab;   // GATHER_TABLE: per reduction row (byte distance, tap number), in LDS

    // GATHER_TABLE: the workgroup fills the table (rows at or past the end of the reduction get the
    // bit that is always set); the caller puts a barrier between this and the first load.
    __device__ __forceinline__ void fill_table(const ConvKArgs &p, int tid, uint2 *t)
    {
        tab = t;
        if constexpr (TABLE) {
            // every row a load can ask for: the reduction rounded up to whole stages and the two
            // stages the loads run ahead (the launcher checked that the table holds them)
            const int rows = ((p.Kg + T::BK - 1) / T::BK + 2) * T::BK;
            for (int kg = tid; kg < rows; kg += T::NT) {
                uint2 e = {0u, (uint32_t)LAST_BIT};
                if (kg < p.Kg) {
                    const uint32_t c = fast_div((uint32_t)kg, p.magic_RS, p.one_RS), rs = (uint32_t)kg - c * (uint32_t)p.RS;
                    const uint32_t r = fast_div(rs, p.magic_S, p.one_S), sx = rs - r * (uint32_t)p.S;
                    e.x = (c * (uint32_t)p.HW + r * (uint32_t)p.W + sx) * 4u;
                    e.y = rs;
                }
                t[kg] = e;
            }
        }
    }

    __device__ __forceinline__ void init(const ConvKArgs &p, int tid, int n0)
    {
        RS = p.RS; S = p.S; HW = p.HW; W = p.W; pre_act = p.pre_act; C = p.C; magic_C = p.magic_C;
        magic_RS = p.magic_RS; magic_S = p.magic_S; one_RS = p.one_RS; one_S = p.one_S;
        const int col = tid % T::BN;
        krow0 = __builtin_amdgcn_readfirstlane(tid / T::BN);
        lds_off = krow0 * T::LDB + col;
        // the descriptor starts at the first image this tile touches: offsets stay small
        uint32_t rem0;
        const int img0 = (int)div_by((uint32_t)n0, (uint32_t)p.PQ, p.recip_PQ, rem0);
        const uint64_t skip = (uint64_t)img0 * p.CHW * 4;
        // GATHER_TAPS*: per-lane offsets are those of tap (0,0), which lies up to pad rows and pad
        // columns before the image; the descriptor starts that much earlier so that they are not
        // negative (no load is made there: such taps are flagged outside)
        const int lead = TAPS ? (p.pad * p.W + p.pad) * 4 : 0;
        rsrc = make_rsrc(reinterpret_cast<const char *>(p.in) + skip - lead, p.in_bytes - skip + lead);
        const int colg = n0 + col;
        rmask = 0; smask = 0; pix_off = 0;
        if (colg < p.Ng) {
            uint32_t pq, oq;
            int img = (int)div_by((uint32_t)colg, (uint32_t)p.PQ, p.recip_PQ, pq);
            int op = (int)div_by(pq, (uint32_t)p.Q, p.recip_Q, oq);
            int ih0 = op * p.stride - p.pad, iw0 = (int)oq * p.stride - p.pad;
            pix_off = (img - img0) * p.CHW + ih0 * p.W + iw0;
            // filter rows r < -ih0 or r >= H - ih0 and columns s < -iw0 or s >= W - iw0 fall outside
            const uint32_t rows_out = outside_bits(-ih0, p.H - ih0, p.R);
            const uint32_t cols_out = outside_bits(-iw0, p.W - iw0, p.S);
            if constexpr (MODE == GATHER_ANY) {
                rmask = ~rows_out;
                smask = ~cols_out;
            }
            if constexpr (TAPS) {
                const uint32_t all_cols = low_bits(p.S);
                uint64_t taps = 0;
                for (int r = 0; r < p.R; ++r)
                    taps |= (uint64_t)((rows_out >> r) & 1u ? all_cols : cols_out) << (r * p.S);
                rmask = (uint32_t)taps;
                smask = (uint32_t)(taps >> 32);
                pix_off = pix_off * 4 + lead;
            }
        } else if constexpr (TAPS) {
            rmask = 0xFFFFFFFFu; smask = 0xFFFFFFFFu;
        }
        if constexpr (TAPS) { if (MODE == GATHER_TAPS1) rmask |= 1u << 31; else smask |= 1u << 31; }
        (void)C; (void)magic_C;
        if constexpr (POINT) pix_off = colg < p.Ng ? pix_off * 4 : (int)kOobOffset;   // bytes, or out of range
    }
    template <int SET>
    __device__ __forceinline__ void load(int k0, int kend)
    {
        if constexpr (POINT) {
            // A row at or past kend meets zeros in the filter operand; it reads the last real
            // channel so that what it multiplies is a finite input value of the same image
#pragma unroll
            for (int i = 0; i < ITERS; ++i) {
                int kg = min(k0 + krow0 + i * KSTEP, kend - 1);  // wave-uniform
                regs[SET][i] = buf_load1(rsrc, (uint32_t)pix_off, (uint32_t)(kg * HW) * 4u);
            }
            return;
        }
        if constexpr (TAPMAJOR) {
            // one tap for the whole stage: its bit and its distance once, the channel in the uniform offset
            const uint32_t kk = k0 < kend ? (uint32_t)k0 : 0u;
            const uint32_t tap = __umulhi(kk, magic_C), c0 = kk - tap * (uint32_t)C;
            const uint32_t r = fast_div(tap, magic_S, one_S), sx = tap - r * (uint32_t)S;
            const uint32_t t = k0 < kend ? tap : (uint32_t)LAST_BIT;
            const uint32_t word = t < 32u ? rmask : smask;
            const uint32_t off = (uint32_t)pix_off | (((word >> (t & 31u)) & 1u) << 31);
            uint32_t koff = ((c0 + (uint32_t)krow0) * (uint32_t)HW + r * (uint32_t)W + sx) * 4u;
#pragma unroll
            for (int i = 0; i < ITERS; ++i) {
                regs[SET][i] = buf_load1(rsrc, off, koff);
                koff += (uint32_t)(KSTEP * HW) * 4u;
            }
            return;
        }
        if constexpr (TABLE) {
            // one LDS address per stage; the rows of this thread lie KSTEP entries apart.  Rows at or
            // past kend are either past the reduction's end (entry: always outside) or belong to a
            // look-ahead stage of a split reduction, whose values are never multiplied.
            const uint2 *row = tab + (k0 + krow0);
            const uint64_t taps = ((uint64_t)smask << 32) | rmask;
#pragma unroll
            for (int i = 0; i < ITERS; ++i) {
                const uint2 e = row[i * KSTEP];
                const uint32_t outside = (uint32_t)(taps >> e.y);      // bit 0 counts: the shift below drops the rest
                regs[SET][i] = buf_load1(rsrc, ((uint32_t)pix_off + e.x) | (outside << 31));
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < ITERS; ++i) {
            uint32_t kg = (uint32_t)(k0 + krow0 + i * KSTEP);  // wave-uniform
            uint32_t c = fast_div(kg, magic_RS, one_RS);
            uint32_t rs = kg - c * (uint32_t)RS;
            uint32_t r = fast_div(rs, magic_S, one_S);
            uint32_t s = rs - r * (uint32_t)S;
            int koff = (int)c * HW + (int)r * W + (int)s;
            if constexpr (TAPS) {
                // a row at or past kend takes the bit that is always set
                const uint32_t t = (int)kg < kend ? rs : (uint32_t)LAST_BIT;
                uint32_t word = rmask;
                if constexpr (MODE == GATHER_TAPS2) word = t < 32u ? rmask : smask;
                const uint32_t outside = (word >> (t & 31u)) & 1u;
                regs[SET][i] = buf_load1(rsrc, (uint32_t)pix_off | (outside << 31), (uint32_t)koff * 4u);
                continue;
            }
            uint32_t ok = (uint32_t)((int)kg < kend) & (rmask >> r) & (smask >> s) & 1u;
            // not ok -> set the top bit: at or beyond 2^31 every descriptor reads as zero
            uint32_t off = ((uint32_t)(pix_off + koff) * 4u) | ((ok ^ 1u) << 31);
            regs[SET][i] = buf_load1(rsrc, off);
        }
    }
    // The element-wise operator that precedes the convolution is applied where its operand is
    // first touched (the symmetric case of section "Operator Fusion": fused with the first iteration
    // of the heavy operator's reduction loops); zero fill stays zero under ReLU and ReLU6.
    template <int SET>
    __device__ __forceinline__ void store(float *Bs, int)
    {
        if (pre_act != POLYDL_ACT_NONE) {   // uniform
#pragma unroll
            for (int i = 0; i < ITERS; ++i) {
                float v = fmaxf(regs[SET][i], 0.f);
                regs[SET][i] = pre_act == POLYDL_ACT_RELU6 ? fminf(v, 6.f) : v;
            }
        }
#pragma unroll
        for (int i = 0; i < ITERS; ++i) Bs[lds_off + i * KSTEP * T::LDB] = regs[SET][i];
    }
};

__device__ __forceinline__ float apply_act(float v, int act)
{
    if (act != POLYDL_ACT_NONE) v = fmaxf(v, 0.f);
    if (act == POLYDL_ACT_RELU6) v = fminf(v, 6.f);
    return v;
}

template <class T, int AVEC, int MODE>
__global__ __launch_bounds__(T::NT) void conv_kernel(ConvKArgs p)
{
    __shared__ __attribute__((aligned(16))) float lds[T::LDS_FLOATS];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int tm, tn;
    // which tile, and which part of its reduction (uniform)
    int tile = blockIdx.x, part = blockIdx.y, parts = p.split_k, kps = p.k_per_split, first_split_tile = 0;
    if (p.tail_parts > 1) {
        part = 0; parts = 1; first_split_tile = p.whole_tiles;
        if (tile >= p.whole_tiles) {
            uint32_t rem;
            tile = p.whole_tiles + (int)div_by((uint32_t)(tile - p.whole_tiles), (uint32_t)p.tail_parts, p.recip_tail, rem);
            part = (int)rem; parts = p.tail_parts; kps = p.tail_k;
        }
    }
    tile_coords(tile, p.raster, p.tiles_m, p.tiles_n, tm, tn);
    const int m0 = tm * T::BM, n0 = tn * T::BN;
    const int wm0 = (wave % T::WAVES_M) * T::WM, wn0 = (wave / T::WAVES_M) * T::WN;
    const int kbegin = part * kps;
    const int kend = min(p.Kg, kbegin + kps);

    // AVEC = 1 stands for filter rows that are not a multiple of four floats long or not 16-byte
    // aligned: vector loads all the same, with the reduction's tail masked
    ALoader<T, 4, AVEC == 1> al;
    BLoaderIm2col<T, MODE> bl;
    __shared__ uint2 ktab[MODE == GATHER_TABLE ? kTableRows : 1];
    bl.fill_table(p, tid, ktab);
    al.init(p.wt, tid, m0, p.K, p.Kg, p.Kg);
    bl.init(p, tid, n0);
    if constexpr (MODE == GATHER_TABLE) __syncthreads();

    v16f acc[T::MB][T::NB];
#pragma unroll
    for (int bi = 0; bi < T::MB; ++bi)
#pragma unroll
        for (int bj = 0; bj < T::NB; ++bj)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[bi][bj][r] = 0.f;

    gemm_mainloop<T, false>(lds, al, bl, acc, kbegin, kend, tid, wm0, wn0);

    // With the reduction of a tile split over several workgroups every part leaves its accumulator tile in scratch
    // memory (thread-contiguous, device-scope stores); the part that arrives last adds all parts
    // in index order and runs the fused epilogue.  Nothing waits on another workgroup.
    if (parts > 1) {
        __shared__ unsigned s_arrived;
        constexpr size_t TILE = (size_t)T::BM * T::BN;
        constexpr int NT = T::NT;
        const int slot = tile - first_split_tile;   // scratch tiles and counters are numbered over the split tiles
        float *tile0 = p.partials + (size_t)slot * parts * TILE;
        float *mine = tile0 + (size_t)part * TILE;
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
            s_arrived = __hip_atomic_fetch_add(p.counters + slot, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (__builtin_amdgcn_readfirstlane(s_arrived) != (unsigned)parts - 1u) return;   // not the last part
        if (tid == 0)               // leave the counter at zero for the next launch
            __hip_atomic_store(p.counters + slot, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sum_partial_tiles<T>(tile0, parts, TILE, tid, acc);
    }
    // epilogue.  The lane owns NB adjacent pixels starting at colg for 16*MB output channels.
    // Addresses are a per-lane byte offset from the first image the tile touches plus a uniform
    // offset per channel row, so a store costs no address arithmetic.
    const int colg = n0 + wn0 + T::NB * (lane & 31);
    if (colg >= p.Ng) return;
    const int krow = m0 + wm0 + 4 * (lane >> 5);   // channel of register 0; register r adds 8*(r/4) + r%4
    const uint32_t KPQ = (uint32_t)p.K * (uint32_t)p.PQ;
    uint32_t rem0, pq;
    const uint32_t img0 = div_by((uint32_t)n0, (uint32_t)p.PQ, p.recip_PQ, rem0);   // uniform
    const uint32_t img = div_by((uint32_t)colg, (uint32_t)p.PQ, p.recip_PQ, pq);
    const uint64_t skip = (uint64_t)img0 * KPQ * 4;
    __amdgpu_buffer_rsrc_t ro = make_rsrc(reinterpret_cast<char *>(p.out) + skip, p.out_bytes - skip);
    // bias of channels at or past K reads as zero (as does every channel without a bias vector)
    __amdgpu_buffer_rsrc_t rb = make_rsrc(p.bias, p.bias ? (uint64_t)p.K * 4 : 0);
    float bias[T::MB][16];
#pragma unroll
    for (int bi = 0; bi < T::MB; ++bi)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            bias[bi][r] = buf_load1(rb, (uint32_t)(krow + 32 * bi + 8 * (r >> 2) + (r & 3)) * 4u);
    const uint32_t row_bytes = (uint32_t)p.PQ * 4u;
    // the NB pixels are one vector store when they lie in one image and keep the alignment
    const bool vec = (p.PQ % T::NB == 0) && (((uintptr_t)p.out & 15) == 0);
    if (vec) {
        const uint32_t off = ((img - img0) * KPQ + (uint32_t)krow * (uint32_t)p.PQ + pq) * 4u;
        store_rows_by<T>(p.act, m0 + T::BM <= p.K, ro, off, row_bytes, acc, bias, krow, p.K);
    } else {
#pragma unroll
        for (int bj = 0; bj < T::NB; ++bj) {
            if (colg + bj >= p.Ng) break;
            // pixel bj of the lane: same image, or among the first pixels of a following one
            uint32_t q = pq + bj, im = img - img0;
            while (q >= (uint32_t)p.PQ) { q -= (uint32_t)p.PQ; ++im; }
            const uint32_t off = (im * KPQ + (uint32_t)krow * (uint32_t)p.PQ + q) * 4u;
#pragma unroll
            for (int bi = 0; bi < T::MB; ++bi)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int c = 32 * bi + 8 * (r >> 2) + (r & 3);
                    if (krow + c >= p.K) continue;
                    buf_store1(ro, off, (uint32_t)c * row_bytes, apply_act(acc[bi][bj][r] + bias[bi][r], p.act));
                }
        }
    }
}

template <class T>
static hipError_t conv_launch(const ConvProblem &q, int split_k, int raster, hipStream_t stream)
{
    ConvKArgs a;
    a.in = static_cast<const float *>(q.in); a.wt = static_cast<const float *>(q.wt);
    a.bias = q.bias; a.out = q.out;
    a.C = q.C; a.H = q.H; a.W = q.W; a.K = q.K; a.R = q.R; a.S = q.S;
    a.stride = q.stride; a.pad = q.pad; a.P = q.P; a.Q = q.Q;
    a.PQ = q.P * q.Q; a.RS = q.R * q.S; a.HW = q.H * q.W; a.CHW = q.C * q.H * q.W;
    a.Kg = q.C * q.R * q.S;
    a.Ng = q.N * a.PQ;
    a.magic_C = div_magic((uint32_t)q.C);
    a.magic_RS = div_magic((uint32_t)a.RS);
    a.magic_S = div_magic((uint32_t)q.S);
    a.one_RS = a.RS == 1 ? 0xFFFFFFFFu : 0u;
    a.one_S = q.S == 1 ? 0xFFFFFFFFu : 0u;
    a.in_bytes = (uint64_t)q.N * a.CHW * 4;
    a.out_bytes = (uint64_t)q.N * q.K * a.PQ * 4;
    a.recip_PQ = div_recip((uint32_t)a.PQ);
    a.recip_Q = div_recip((uint32_t)q.Q);
    a.tiles_m = (q.K + T::BM - 1) / T::BM;
    a.tiles_n = (a.Ng + T::BN - 1) / T::BN;
    int stages = (a.Kg + T::BK - 1) / T::BK;
    if (split_k < 1) split_k = 1;
    if (split_k > stages) split_k = stages;
    int stages_per = (stages + split_k - 1) / split_k;
    a.k_per_split = stages_per * T::BK;
    a.split_k = (stages + stages_per - 1) / stages_per;
    const bool tail = raster >= 2;   // rasters 2 and 3: tile order of raster 0 and 1, leftover tiles split
    a.raster = raster & 1;
    a.act = q.act;
    a.pre_act = q.pre_act;
    a.partials = nullptr;
    a.counters = nullptr;
    hipError_t le = hipSuccess;
    const int tiles = a.tiles_m * a.tiles_n;
    a.whole_tiles = tiles; a.tail_parts = 1; a.tail_k = a.k_per_split; a.recip_tail = 0;
    dim3 grid((unsigned)tiles, (unsigned)a.split_k), block(T::NT);
    if (a.split_k > 1) {
        const size_t bytes = (size_t)tiles * a.split_k * T::BM * T::BN * sizeof(float);
        hipError_t e = splitk_scratch(stream, q.arena, bytes, tiles, &a.partials, &a.counters);
        if (e != hipSuccess) return e;
    } else {
        // rasters 2, 3: an unsplit grid whose last round would leave most compute units idle has the
        // tiles of that round split
        const TailSplit ts = tail ? tail_split(tiles, stages, compute_units()) : TailSplit{0, 1, stages};
        if (ts.parts > 1) {
            a.whole_tiles = tiles - ts.tiles; a.tail_parts = ts.parts; a.tail_k = ts.stages_per_part * T::BK;
            a.recip_tail = div_recip((uint32_t)ts.parts);
            const size_t bytes = (size_t)ts.tiles * ts.parts * T::BM * T::BN * sizeof(float);
            hipError_t e = splitk_scratch(stream, q.arena, bytes, ts.tiles, &a.partials, &a.counters);
            if (e != hipSuccess) return e;
            grid = dim3((unsigned)(a.whole_tiles + ts.tiles * ts.parts), 1u);
        }
    }
    const bool avec = (a.Kg % 4 == 0) && ((uintptr_t)q.wt % 16 == 0);
    // tile layout 2: the filter comes as [K][R][S][C], 16-byte aligned (its rows load as vectors)
    const bool tapmajor = q.wt_tap != nullptr;
    if (tapmajor) {
        if (!gather_tap_major_fits(q, T::BK) || ((uintptr_t)q.wt_tap & 15)) return hipErrorInvalidValue;
        a.wt = q.wt_tap;
    }
    // the table covers every row a load can ask for: the reduction rounded up to whole stages and the
    // two stages the loads run ahead
    const bool table = a.RS <= 63 && (stages + 2) * T::BK <= kTableRows;
    const int mode = (q.R == 1 && q.S == 1 && q.pad == 0) ? GATHER_POINT
                     : tapmajor ? GATHER_TAPMAJOR
                     : table ? GATHER_TABLE
                     : a.RS <= 31 ? GATHER_TAPS1 : a.RS <= 63 ? GATHER_TAPS2 : GATHER_ANY;
#define POLYDL_GO(AV, MODE) le = launch_kernel((conv_kernel<T, AV, MODE>), grid, block, 0, stream, a)
    if (mode == GATHER_TAPMAJOR) {
        POLYDL_GO(4, GATHER_TAPMAJOR);
    } else if (avec) {
        if (mode == GATHER_POINT) POLYDL_GO(4, GATHER_POINT);
        else if (mode == GATHER_TABLE) POLYDL_GO(4, GATHER_TABLE);
        else if (mode == GATHER_TAPS1) POLYDL_GO(4, GATHER_TAPS1);
        else if (mode == GATHER_TAPS2) POLYDL_GO(4, GATHER_TAPS2);
        else POLYDL_GO(4, GATHER_ANY);
    } else {
        if (mode == GATHER_POINT) POLYDL_GO(1, GATHER_POINT);
        else if (mode == GATHER_TABLE) POLYDL_GO(1, GATHER_TABLE);
        else if (mode == GATHER_TAPS1) POLYDL_GO(1, GATHER_TAPS1);
        else if (mode == GATHER_TAPS2) POLYDL_GO(1, GATHER_TAPS2);
        else POLYDL_GO(1, GATHER_ANY);
    }
#undef POLYDL_GO
    return le;
}

#define POLYDL_DEFINE_CONV(BM, BN, BK, WM, WN)                                                            \
    hipError_t conv_launch_##BM##x##BN##x##BK##_##WM##x##WN(const ConvProblem &q, int s, int r,           \
                                                            hipStream_t st)                              \
    {                                                                                                    \
        return conv_launch<Tile<BM, BN, BK, WM, WN>>(q, s, r, st);                                        \
    }
POLYDL_TILE_FAMILY(POLYDL_DEFINE_CONV)

}  // namespace polydl
