// Forward convolution on the fp32 matrix cores with the input staged through LDS as row patches.
//
// Same GEMM view as conv_kernels.hip: out[K][N*P*Q] = wt[K][C*R*S] * X[C*R*S][N*P*Q].  Here the
// im2col matrix X is not gathered element by element from HBM.  A workgroup owns BN consecutive
// output pixels (a run of output rows, possibly crossing into the next images); per stage it
// copies, for CB input channels, exactly the input rows those pixels need into LDS, each row
// widened by the zero padding so no tap ever needs a bounds test.  The R*S taps are then formed
// while the matrix-core operand is read from LDS: a lane's pixel has one base address in the
// patch and tap (r, s) of channel c is at a wave-uniform offset from it.  Every input element is
// fetched from HBM/L2 once per workgroup instead of once per tap -- the reuse the paper's outer
// loop tiling is after (section "Working set size computation": a reuse is realised when the
// data touched between source and target iteration stays in the fast memory).
//
// Reduction order inside a stage: channel pairs outermost, then filter row, filter column.  One
// v_mfma_f32_32x32x2_f32 consumes one tap of one channel pair: lanes 0-31 carry the even
// channel, lanes 32-63 the odd one.  The filter rows of the workgroup's BM output channels are
// copied as they lie in KCRS (C*R*S contiguous per output channel); the LDS row pitch is odd so
// that 32 lanes reading one column of 32 rows hit 32 different banks.
#include "gemm_core.hpp"
#include "internal.hpp"
#include "variants.hpp"

namespace polydl {

// The reduction element the kernel moves and multiplies.
// ElemF32:   one float; an MFMA step (v_mfma_f32_32x32x2_f32) consumes one tap of a channel pair.
// ElemBF16x8: eight consecutive bfloat16 channels (16 bytes, the NCHW8c / KCRS8c unit); an MFMA
//            step (v_mfma_f32_32x32x16_bf16, fp32 accumulate) consumes one tap of a pair of units.
// "Channel" below means one such unit.
struct ElemF32 {
    static constexpr int BYTES = 4;
    typedef float unit_t;
    typedef float frag_t;
    static __device__ __forceinline__ frag_t read(const unit_t *p) { return *p; }
    static __device__ __forceinline__ v16f mfma(frag_t a, frag_t b, v16f c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
    }
};
struct ElemBF16x8 {
    static constexpr int BYTES = 16;
    typedef v4f unit_t;
#if defined(__HIP_DEVICE_COMPILE__)
    typedef __bf16 frag_t __attribute__((ext_vector_type(8)));
    static __device__ __forceinline__ frag_t read(const unit_t *p) { return __builtin_bit_cast(frag_t, *p); }
    static __device__ __forceinline__ v16f mfma(frag_t a, frag_t b, v16f c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
#else
    // the host pass only needs the kernel's signature; bfloat16 vectors do not exist there
    typedef v4f frag_t;
    static frag_t read(const unit_t *p) { return *p; }
    static v16f mfma(frag_t, frag_t, v16f c) { return c; }
#endif
};

struct ConvPatchKArgs {
    const void *in, *wt;
    const float *bias;
    float *out;
    int C, H, W, K, R, S, stride, pad, P, Q;
    int PQ, RS, HW, CHW, Kg, Ng;
    int Wp;          // pitch of a patch row: W + 2*pad, or Q when S == 1 (only the columns used)
    int prs, irs;    // patch rows per output-row step, input rows per patch row: (stride, 1), or
                     // (1, stride) when R == 1 so that rows no tap reads are not staged
    int pcs, ics;    // the same for columns: (stride, 1), or (1, stride) when S == 1
    int CB;          // input channels per stage (even)
    // Filter rows per stage.  Rp = R: a stage holds all R*S taps of its CB channels.  Rp = 1 (large
    // filters): a stage holds ONE filter row of its CB channels -- S taps per channel, and of the
    // input only the rows that filter row reads (one per output row) -- so that the LDS need of a
    // stage does not grow with R; the R filter rows of a channel block are consecutive stages.
    int Rp, nr;      // nr = R / Rp stages per channel block
    int RSp;         // Rp*S: taps of one channel in a stage
    int nstages;     // ceil(C / CB) * nr
    int D;           // CB*Rp*S: reduction elements per stage
    int LDA;         // LDS pitch of a filter row: D + 1 (odd, so a column read has no bank conflict)
    int rows_full;   // patch rows one whole image contributes: (P-1)*prs + R
    int a_stage;     // floats reserved per LDS filter stage (BM*LDA rounded up to the workgroup size)
    int b_stage;     // floats reserved per LDS patch stage (rounded up likewise)
    uint32_t magic_Wp, one_Wp, magic_rf, one_rf, magic_lda, magic_S, one_S, magic_nr, one_nr;
    uint32_t recip_PQ, recip_Q, recip_split;   // for div_by()
    uint64_t in_bytes, wt_bytes, out_bytes;
    int tiles_m, tiles_n, raster, act;
    // split_k > 1: every tile's reduction is cut into split_k parts of stages_per_split stages;
    // workgroup t*split_k + y takes part y of tile t
    int split_k, stages_per_split;
    float *partials;      // split_k > 1: [tile][split][BM*BN] accumulator tiles in register order
    unsigned *counters;   // split_k > 1: per tile, how many of its reduction parts have finished
    int nbuf;        // LDS stage buffers: 2, or 1 when a workgroup runs a single stage
    int single;      // 1: the whole reduction is ONE unit (CB == 1): the upper half-wave, which would
                     // carry the pair's second unit, takes the NEXT TAP of the same unit instead (two taps
                     // per matrix instruction; a last odd tap, and every tap of a filter whose size is
                     // not known at compile time, multiplies a zero kept in LDS)
};

__device__ __forceinline__ uint32_t fdiv(uint32_t n, uint32_t magic, uint32_t ones_if_d1)
{
    return __umulhi(n, magic) + (n & ones_if_d1);
}

__device__ __forceinline__ float act_apply(float v, int act)
{
    if (act != POLYDL_ACT_NONE) v = fmaxf(v, 0.f);
    if (act == POLYDL_ACT_RELU6) v = fminf(v, 6.f);
    return v;
}

// One channel pair of a stage: R*S taps, each one rank-2 update of every accumulator block.
// With the filter size known at compile time (RC, SC > 0) the taps are unrolled, so the LDS
// reads of later taps are in flight while the matrix cores work on earlier ones.
template <class E, class T, int RC, int SC>
__device__ __forceinline__ void patch_pair(const typename E::unit_t *__restrict__ A,
                                           const typename E::unit_t *__restrict__ B,
                                           const int (&a_base)[T::MB], const int (&b_base)[T::NB],
                                           int ka, int kb, int R, int S, int Wp, v16f (&acc)[T::MB][T::NB],
                                           int bmul = 1)
{
    constexpr int MB = T::MB, NB = T::NB;
    // bmul is 1, or per lane 0 where the lane's pixel operand must stay on one (zero) LDS unit;
    // only the 16-byte element path pays for the multiply
    auto boff = [&](int o) { return E::BYTES == 16 ? o * bmul : o; };
    if constexpr (RC > 0) {
#pragma unroll
        for (int r = 0; r < RC; ++r)
#pragma unroll
            for (int s = 0; s < SC; ++s) {
                typename E::frag_t fa[MB], fb[NB];
#pragma unroll
                for (int bi = 0; bi < MB; ++bi) fa[bi] = E::read(A + a_base[bi] + ka + r * SC + s);
#pragma unroll
                for (int bj = 0; bj < NB; ++bj) fb[bj] = E::read(B + b_base[bj] + boff(kb + r * Wp + s));
#pragma unroll
                for (int bi = 0; bi < MB; ++bi)
#pragma unroll
                    for (int bj = 0; bj < NB; ++bj) acc[bi][bj] = E::mfma(fa[bi], fb[bj], acc[bi][bj]);
            }
    } else {
        for (int r = 0; r < R; ++r) {
            for (int s = 0; s < S; ++s) {
                typename E::frag_t fa[MB], fb[NB];
#pragma unroll
                for (int bi = 0; bi < MB; ++bi) fa[bi] = E::read(A + a_base[bi] + ka);
#pragma unroll
                for (int bj = 0; bj < NB; ++bj) fb[bj] = E::read(B + b_base[bj] + boff(kb + s));
#pragma unroll
                for (int bi = 0; bi < MB; ++bi)
#pragma unroll
                    for (int bj = 0; bj < NB; ++bj) acc[bi][bj] = E::mfma(fa[bi], fb[bj], acc[bi][bj]);
                ++ka;
            }
            kb += Wp;
        }
    }
}

// Loads go straight from HBM/L2 into LDS (buffer_load ... lds): lane i of a wave instruction
// fills LDS dword base + i, so a workgroup-wide pass fills NT consecutive dwords and the LDS
// image is simply "dword e of the stage" for e = thread + pass*NT.  No staging registers, no
// ds_write, and the data of stage t+1 streams in while the matrix cores work on stage t.
// Out-of-range lanes (padding, rows outside the image, channel or filter tails) read as zero.
// MAXA / MAXP: passes a thread may need for the filter block / the input patch of one stage.
// RC, SC: filter size when known at compile time, 0 for any size.
typedef __attribute__((address_space(3))) void *lds_ptr_t;

// One direct-to-LDS buffer load of BYTES (4 or 16) per lane.  Device pass only: the 16-byte form
// exists on gfx950 alone and the host pass has no such target to check it against.
template <int BYTES, class U>
__device__ __forceinline__ void lds_dma(__amdgpu_buffer_rsrc_t rsrc, U *lds_dst, uint32_t byte_off)
{
#if defined(__HIP_DEVICE_COMPILE__)
    // the size operand must be a literal, not a template-dependent value
    if constexpr (BYTES == 16)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr_t)lds_dst, 16, (int)byte_off, 0, 0, 0);
    else
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr_t)lds_dst, 4, (int)byte_off, 0, 0, 0);
#else
    (void)rsrc; (void)lds_dst; (void)byte_off;
#endif
}

// ROWS: one filter row per stage (p.nr > 1); RC, SC then describe that row (RC = 1).
template <class E, class T, int MAXA, int MAXP, int RC, int SC, bool ROWS = false>
__global__ __launch_bounds__(T::NT) void conv_patch_kernel(ConvPatchKArgs p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    typedef typename E::unit_t unit_t;
    unit_t *lds = reinterpret_cast<unit_t *>(lds_raw);
    constexpr int NT = T::NT, MB = T::MB, NB = T::NB;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, lh = lane >> 5;
    const bool cut = p.split_k > 1;   // uniform
    int tile = blockIdx.x, part = 0;
    if (cut) {
        uint32_t rem;
        tile = (int)div_by(blockIdx.x, (uint32_t)p.split_k, p.recip_split, rem);
        part = (int)rem;
    }
    const int cut_tile = tile;
    int tm, tn;
    tile_coords(tile, p.raster, p.tiles_m, p.tiles_n, tm, tn);
    const int m0 = tm * T::BM, n0 = tn * T::BN;
    const int wm0 = (wave % T::WAVES_M) * T::WM, wn0 = (wave / T::WAVES_M) * T::WN;

    // ---- geometry of this workgroup's pixel run (uniform) ---------------------------------
    const int nlast = min(n0 + T::BN, p.Ng) - 1;
    uint32_t pq_a, pq_b, q_a, q_b;
    const int img_a = (int)div_by((uint32_t)n0, (uint32_t)p.PQ, p.recip_PQ, pq_a);
    const int p_a = (int)div_by(pq_a, (uint32_t)p.Q, p.recip_Q, q_a);
    const int img_b = (int)div_by((uint32_t)nlast, (uint32_t)p.PQ, p.recip_PQ, pq_b);
    const int p_b = (int)div_by(pq_b, (uint32_t)p.Q, p.recip_Q, q_b);
    int nrows0, total_rows;
    if (img_a == img_b) {
        nrows0 = (p_b - p_a) * p.prs + p.Rp;
        total_rows = nrows0;
    } else {
        nrows0 = (p.P - 1 - p_a) * p.prs + p.Rp;
        total_rows = nrows0 + (img_b - img_a - 1) * p.rows_full + p_b * p.prs + p.Rp;
    }
    const int ihb0 = p_a * p.stride - p.pad;       // first input row held for the first image
    const int chs = total_rows * p.Wp;             // patch floats per channel
    const int patch_elems = p.CB * chs;
    // Multiplier for e / chs, e < MAXP*NT < 2^14: any value from 2^32/chs up to 2^18/chs above it
    // divides exactly, so the single-precision reciprocal, nudged upwards, is good enough.
    const uint32_t magic_chs = chs > 1 ? (uint32_t)(4294967296.0f * __frcp_rn((float)chs) * (1.0f + 0x1p-21f)) + 1u : 0u;
    const uint32_t one_chs = chs > 1 ? 0u : 0xFFFFFFFFu;

    const int a_stage = p.a_stage;                 // units: BM rows of pitch LDA, rounded up to NT
    unit_t *As = lds;                              // [2][a_stage]
    unit_t *Bs = lds + p.nbuf * a_stage;           // [nbuf][b_stage], then one zero unit
    const int a_elems = T::BM * p.LDA;

    // ---- per-thread patch elements: LDS dword e <-> one input element or a zero -------------
    // ROWS: the input row of an element moves down by one per filter-row stage, so whether it lies
    // inside the image is decided per stage from p_row (its row for filter row 0; far below zero
    // for an element that is never valid); p_goff then holds the signed offset for filter row 0.
    uint32_t p_goff[MAXP];
    int p_row[ROWS ? MAXP : 1];
#pragma unroll
    for (int i = 0; i < MAXP; ++i) {
        if (i * NT >= patch_elems) {   // uniform: no pass of the workgroup reaches this entry
            p_goff[i] = kOobOffset;
            if constexpr (ROWS) p_row[i] = -0x40000000;
            continue;
        }
        uint32_t e = (uint32_t)(tid + i * NT);
        uint32_t c_l = fdiv(e, magic_chs, one_chs);
        uint32_t rem = e - c_l * (uint32_t)chs;
        uint32_t row = fdiv(rem, p.magic_Wp, p.one_Wp);
        int col = (int)(rem - row * (uint32_t)p.Wp);
        int ii = 0, rr = (int)row, ihb = ihb0;
        if ((int)row >= nrows0) {
            uint32_t d = row - (uint32_t)nrows0;
            uint32_t j = fdiv(d, p.magic_rf, p.one_rf);
            ii = 1 + (int)j;
            rr = (int)(d - j * (uint32_t)p.rows_full);
            ihb = -p.pad;
        }
        int ih = ihb + rr * p.irs, iw = col * p.ics - p.pad;
        if constexpr (ROWS) {
            const bool okc = ((int)e < patch_elems) && iw >= 0 && iw < p.W;
            p_row[i] = okc ? ih : -0x40000000;
            p_goff[i] = (uint32_t)(((ii * p.C + (int)c_l) * p.HW + ih * p.W + iw) * E::BYTES);
        } else {
            bool ok = ((int)e < patch_elems) && ih >= 0 && ih < p.H && iw >= 0 && iw < p.W;
            p_goff[i] = ok ? (uint32_t)(((ii * p.C + (int)c_l) * p.HW + ih * p.W + iw) * E::BYTES) : kOobOffset;
        }
    }

    // ---- per-thread filter elements: LDS dword e = m*LDA + kk <-> wt[m0+m][k0+kk] ------------
    uint32_t a_goff[MAXA];
#pragma unroll
    for (int i = 0; i < MAXA; ++i) {
        if (i * NT >= a_elems) {   // uniform
            a_goff[i] = kOobOffset;
            continue;
        }
        uint32_t e = (uint32_t)(tid + i * NT);
        uint32_t m = fdiv(e, p.magic_lda, 0u);
        int kk = (int)(e - m * (uint32_t)p.LDA);
        bool ok = (int)e < a_elems && m0 + (int)m < p.K && kk < p.D;
        int col = kk;
        if constexpr (ROWS) {   // stage column kk = (channel, s) -> KCRS column channel*R*S + s (+ r*S per stage)
            const int c_l = (int)fdiv((uint32_t)kk, p.magic_S, p.one_S);
            col = c_l * p.RS + (kk - c_l * p.S);
        }
        a_goff[i] = ok ? (uint32_t)(((int)m * p.Kg + col) * E::BYTES) : kOobOffset;
    }

    // ---- per-lane operand bases ---------------------------------------------------------------
    // filter operand: row wm0 + 32*bi + lane%32, column offset (lane/32)*RS selects the odd channel
    int a_base[MB];
#pragma unroll
    for (int bi = 0; bi < MB; ++bi) a_base[bi] = (wm0 + 32 * bi + li) * p.LDA + (p.single ? 0 : lh * p.RSp);
    const int zero_unit = p.nbuf * p.b_stage;      // relative to Bs
    const int bmul = (p.single && lh) ? 0 : 1;   // run-time filter sizes only, see the main loop
    if (tid == 0) {
        unit_t z = {};
        Bs[zero_unit] = z;                          // visible after the first barrier below
    }
    // pixel operand: the lane's NB blocks are NB adjacent pixels (so the epilogue stores them as
    // one vector); patch position of tap (0,0), channel parity lane/32
    int b_base[NB];
    int px_img[NB], px_pq[NB];
#pragma unroll
    for (int bj = 0; bj < NB; ++bj) {
        int colg = n0 + wn0 + NB * li + bj;
        int base = 0;
        px_img[bj] = -1;
        px_pq[bj] = 0;
        if (colg < p.Ng) {
            uint32_t upq, uoq;
            int img = (int)div_by((uint32_t)colg, (uint32_t)p.PQ, p.recip_PQ, upq);
            int op = (int)div_by(upq, (uint32_t)p.Q, p.recip_Q, uoq);
            int pq = (int)upq, oq = (int)uoq;
            int ii = img - img_a;
            int slot0 = ii == 0 ? 0 : nrows0 + (ii - 1) * p.rows_full;
            int p_lo = ii == 0 ? p_a : 0;
            base = (slot0 + (op - p_lo) * p.prs) * p.Wp + oq * p.pcs;
            px_img[bj] = img;
            px_pq[bj] = pq;
        }
        b_base[bj] = p.single ? base : base + lh * chs;
    }

    v16f acc[MB][NB];
#pragma unroll
    for (int bi = 0; bi < MB; ++bi)
#pragma unroll
        for (int bj = 0; bj < NB; ++bj)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[bi][bj][r] = 0.f;

    auto load_stage = [&](int t, int buf) {
        const int cblk = ROWS ? (int)fdiv((uint32_t)t, p.magic_nr, p.one_nr) : t;
        const int frow = ROWS ? t - cblk * p.nr : 0;     // filter row of this stage
        const int c0 = cblk * p.CB;
        const int k0 = c0 * p.RS + frow * p.S;
        const int crem = p.C - c0;      // channels that exist from c0 on
        const int krem = crem * p.RSp;  // stage columns that exist
        const uint64_t a_skip = ((uint64_t)m0 * p.Kg + k0) * E::BYTES;
        __amdgpu_buffer_rsrc_t ra = make_rsrc(reinterpret_cast<const char *>(p.wt) + a_skip, p.wt_bytes - a_skip);
        unit_t *A = As + buf * a_stage + wave * 64;
        if (krem >= p.D) {
#pragma unroll
            for (int i = 0; i < MAXA; ++i)
                if (i * NT < a_elems) lds_dma<E::BYTES>(ra, A + i * NT, a_goff[i]);
        } else {
            // last stage of a channel count that is no multiple of CB: columns past the end are zero
#pragma unroll
            for (int i = 0; i < MAXA; ++i)
                if (i * NT < a_elems) {
                    uint32_t e = (uint32_t)(tid + i * NT);
                    uint32_t m = fdiv(e, p.magic_lda, 0u);
                    int kk = (int)(e - m * (uint32_t)p.LDA);
                    lds_dma<E::BYTES>(ra, A + i * NT, kk < krem ? a_goff[i] : kOobOffset);
                }
        }
        const uint64_t b_skip = ((uint64_t)img_a * p.C + c0) * p.HW * E::BYTES;
        __amdgpu_buffer_rsrc_t rb = make_rsrc(reinterpret_cast<const char *>(p.in) + b_skip, p.in_bytes - b_skip);
        unit_t *B = Bs + buf * p.b_stage + wave * 64;
        if constexpr (ROWS) {
            const int shift = frow * p.W * E::BYTES;
#pragma unroll
            for (int i = 0; i < MAXP; ++i)
                if (i * NT < patch_elems) {
                    bool ok = (uint32_t)(p_row[i] + frow) < (uint32_t)p.H;
                    if (crem < p.CB) ok = ok && (int)fdiv((uint32_t)(tid + i * NT), magic_chs, one_chs) < crem;
                    lds_dma<E::BYTES>(rb, B + i * NT, ok ? p_goff[i] + (uint32_t)shift : kOobOffset);
                }
        } else if (crem >= p.CB) {
#pragma unroll
            for (int i = 0; i < MAXP; ++i)
                if (i * NT < patch_elems) lds_dma<E::BYTES>(rb, B + i * NT, p_goff[i]);
        } else {
#pragma unroll
            for (int i = 0; i < MAXP; ++i)
                if (i * NT < patch_elems) {
                    uint32_t c_l = fdiv((uint32_t)(tid + i * NT), magic_chs, one_chs);
                    lds_dma<E::BYTES>(rb, B + i * NT, (int)c_l < crem ? p_goff[i] : kOobOffset);
                }
        }
    };

    const int npairs = (p.CB + 1) >> 1;

    const int t_begin = cut ? part * p.stages_per_split : 0;
    const int t_end = cut ? min(p.nstages, t_begin + p.stages_per_split) : p.nstages;
    load_stage(t_begin, 0);
    wait_vmcnt0();   // vmcnt(0): this wave's direct-to-LDS loads have landed
    __syncthreads();
    // The one-unit form below gets a stage loop of its own instead of a branch inside the common
    // loop: with two alternative bodies in one loop the compiler keeps the accumulators in two
    // register sets and copies all of them across twice per stage.
    // A reduction of one unit, filter size compiled in: the two halves of the matrix instruction's
    // reduction take two TAPS of that unit -- lanes 0-31 tap t, lanes 32-63 tap t+1 -- instead of two
    // units.  The upper half of a last odd tap multiplies the zero column behind the filter row
    // (LDA > D) with the zero unit.
    auto one_unit_taps = [&](const unit_t *A, const unit_t *B, int buf) {
        if constexpr (RC > 0) {
            const int zb = zero_unit - buf * p.b_stage;   // the zero unit, relative to this stage's patch
#pragma unroll
            for (int t = 0; t < RC * SC; t += 2) {
                const bool tail = t + 1 >= RC * SC;
                const int r0 = t / SC, s0 = t % SC;
                const int r1 = tail ? 0 : (t + 1) / SC, s1 = tail ? 0 : (t + 1) % SC;
                const int a_off = t + lh;
                const int b_off = lh ? r1 * p.Wp + s1 : r0 * p.Wp + s0;
                typename E::frag_t fa[MB], fb[NB];
#pragma unroll
                for (int bi = 0; bi < MB; ++bi) fa[bi] = E::read(A + a_base[bi] + a_off);
#pragma unroll
                for (int bj = 0; bj < NB; ++bj) fb[bj] = E::read(B + ((tail && lh) ? zb : b_base[bj] + b_off));
#pragma unroll
                for (int bi = 0; bi < MB; ++bi)
#pragma unroll
                    for (int bj = 0; bj < NB; ++bj) acc[bi][bj] = E::mfma(fa[bi], fb[bj], acc[bi][bj]);
            }
        } else {
            // filter size known only at run time: tap by tap, the upper half on the zero unit
            int bz[NB];
#pragma unroll
            for (int bj = 0; bj < NB; ++bj) bz[bj] = lh ? zero_unit - buf * p.b_stage : b_base[bj];
            patch_pair<E, T, RC, SC>(A, B, a_base, bz, 0, 0, p.Rp, p.S, p.Wp, acc, bmul);
        }
    };
    auto pairs = [&](const unit_t *A, const unit_t *B, int) {
        if constexpr (RC == 1 && SC == 1) {
            // 1x1 filters: a pair is a single tap, so unroll over pairs instead
            int cp = 0;
            for (; cp + 4 <= npairs; cp += 4) {
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    patch_pair<E, T, 1, 1>(A, B, a_base, b_base, (cp + u) * 2, (cp + u) * 2 * chs, 1, 1, p.Wp, acc, bmul);
            }
            for (; cp < npairs; ++cp)
                patch_pair<E, T, 1, 1>(A, B, a_base, b_base, cp * 2, cp * 2 * chs, 1, 1, p.Wp, acc, bmul);
        } else {
            for (int cp = 0; cp < npairs; ++cp)
                patch_pair<E, T, RC, SC>(A, B, a_base, b_base, cp * 2 * p.RSp, cp * 2 * chs, p.Rp, p.S, p.Wp, acc, bmul);
        }
    };
    bool one_unit = false;   // uniform
    if constexpr (E::BYTES == 16) one_unit = p.single != 0;
    if (one_unit) {
        for (int t = t_begin; t < t_end; ++t) {
            const int buf = (t - t_begin) & 1;
            // buffer buf^1 was last read in stage t-1, which every wave has left (barrier below)
            if (t + 1 < t_end) load_stage(t + 1, buf ^ 1);
            one_unit_taps(As + buf * a_stage, Bs + buf * p.b_stage, buf);
            wait_vmcnt0();   // vmcnt(0)
            __syncthreads();
        }
    } else {
        for (int t = t_begin; t < t_end; ++t) {
            const int buf = (t - t_begin) & 1;
            if (t + 1 < t_end) load_stage(t + 1, buf ^ 1);
            pairs(As + buf * a_stage, Bs + buf * p.b_stage, buf);
            wait_vmcnt0();   // vmcnt(0)
            __syncthreads();
        }
    }

    // ---- epilogue: bias, activation, store NKPQ ------------------------------------------------
    // The lane's NB pixels are one vector store when they lie in one image and keep the alignment.
    // A lane holds 16*MB output channels; their biases are fetched together before any store.
    const bool vec = NB == 1 || ((p.PQ % NB == 0) && (((uintptr_t)p.out & 15) == 0));
    const bool full_rows = m0 + T::BM <= p.K;   // uniform: no channel of this tile is outside K
    if (cut) {
        // Every reduction part leaves its accumulator tile in scratch memory, register by register
        // (thread-contiguous, so the stores coalesce).  The part that finishes last -- whichever
        // it is -- adds all parts up in their fixed order and goes on to the fused epilogue, so
        // the result does not depend on the order of arrival and no pass over the output follows.
        __shared__ unsigned s_arrived;
        constexpr size_t TILE = (size_t)T::BM * T::BN;
        float *tile0 = p.partials + (size_t)cut_tile * p.split_k * TILE;
        float *mine = tile0 + (size_t)part * TILE;
#pragma unroll
        for (int bi = 0; bi < MB; ++bi)
#pragma unroll
            for (int bj = 0; bj < NB; ++bj)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    __hip_atomic_store(mine + ((bi * NB + bj) * 16 + r) * NT + tid, acc[bi][bj][r], __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
        // The tile is written and read back with device-scope accesses, which go past the caches
        // that are not shared by the whole device.  A full release/acquire fence pair would do
        // too, but costs a write-back of the whole L2 per workgroup.  Instead: wait until this
        // wave's stores have completed (at device scope), meet the other waves, then count the
        // arrival; whoever sees the last count knows every part's stores completed before it.
        wait_vmcnt0();   // vmcnt(0)
        __syncthreads();
        if (tid == 0)
            s_arrived = __hip_atomic_fetch_add(p.counters + cut_tile, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (__builtin_amdgcn_readfirstlane(s_arrived) != (unsigned)p.split_k - 1u) return;   // not the last part
        if (tid == 0)               // leave the counter at zero for the next launch
            __hip_atomic_store(p.counters + cut_tile, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sum_partial_tiles<T>(tile0, p.split_k, TILE, tid, acc);
    }
    // Addresses are a per-lane byte offset from the first image the tile touches plus a uniform
    // offset per channel row; biases of channels at or past K (and of a missing bias vector) read
    // as zero.
    const int krow = m0 + wm0 + 4 * lh;   // channel of register 0; register r adds 8*(r/4) + r%4
    const uint32_t KPQ = (uint32_t)p.K * (uint32_t)p.PQ;
    const uint64_t o_skip = (uint64_t)img_a * KPQ * 4;
    __amdgpu_buffer_rsrc_t ro = make_rsrc(reinterpret_cast<char *>(p.out) + o_skip, p.out_bytes - o_skip);
    __amdgpu_buffer_rsrc_t rbias = make_rsrc(p.bias, p.bias ? (uint64_t)p.K * 4 : 0);
    float bias[MB][16];
#pragma unroll
    for (int bi = 0; bi < MB; ++bi)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            bias[bi][r] = buf_load1(rbias, (uint32_t)(krow + 32 * bi + 8 * (r >> 2) + (r & 3)) * 4u);
    const uint32_t row_bytes = (uint32_t)p.PQ * 4u;
    if (px_img[0] < 0) return;
    if (vec && px_img[NB - 1] >= 0) {
        const uint32_t off = ((uint32_t)(px_img[0] - img_a) * KPQ + (uint32_t)krow * (uint32_t)p.PQ + (uint32_t)px_pq[0]) * 4u;
        store_rows_by<T>(p.act, full_rows, ro, off, row_bytes, acc, bias, krow, p.K);
    } else {
#pragma unroll
        for (int bj = 0; bj < NB; ++bj) {
            if (px_img[bj] < 0) continue;
            const uint32_t off = ((uint32_t)(px_img[bj] - img_a) * KPQ + (uint32_t)krow * (uint32_t)p.PQ + (uint32_t)px_pq[bj]) * 4u;
#pragma unroll
            for (int bi = 0; bi < MB; ++bi)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int c = 32 * bi + 8 * (r >> 2) + (r & 3);
                    if (krow + c >= p.K) continue;
                    buf_store1(ro, off, (uint32_t)c * row_bytes, act_apply(acc[bi][bj][r] + bias[bi][r], p.act));
                }
        }
    }
}

// LDS one workgroup may take: the whole 160 KB of a compute unit.
static constexpr size_t kMaxLdsBytes = 160 * 1024 - 256;   // less the kernel's few static words

// Input rows a run of bn consecutive output pixels can need at most (all images it touches).
static int patch_rows_bound(const ConvProblem &q, int bn, int Rp)
{
    const long PQ = (long)q.P * q.Q, Ng = (long)q.N * PQ;
    long run = bn < Ng ? bn : Ng;
    long rows_out = (run - 1 + q.Q - 1) / q.Q + 1;
    if (rows_out > (long)q.N * q.P) rows_out = (long)q.N * q.P;
    long imgs = (run - 1 + PQ - 1) / PQ + 1;
    if (imgs > q.N) imgs = q.N;
    // an image with n output rows in the run holds (n-1)*prs + R patch rows
    long prs = Rp == 1 ? 1 : q.stride;
    long extra = Rp > prs ? Rp - prs : 0;
    long bound = rows_out * prs + imgs * extra;
    return (int)bound;
}

// q.C counts reduction units of E (channels for fp32, blocks of eight channels for bf16) and
// q.in / q.wt point at tensors made of such units.
template <class E, class T, int MAXA, int MAXP>
static hipError_t conv_patch_launch(const ConvProblem &q, int cb, int split_k, int raster, hipStream_t stream,
                                    bool dry)
{
    ConvPatchKArgs a;
    a.in = q.in; a.wt = q.wt; a.bias = q.bias; a.out = q.out;
    a.C = q.C; a.H = q.H; a.W = q.W; a.K = q.K; a.R = q.R; a.S = q.S;
    a.stride = q.stride; a.pad = q.pad; a.P = q.P; a.Q = q.Q;
    a.PQ = q.P * q.Q; a.RS = q.R * q.S; a.HW = q.H * q.W; a.CHW = q.C * q.H * q.W;
    a.Kg = q.C * a.RS;
    a.Ng = q.N * a.PQ;
    a.Wp = q.S == 1 ? q.Q : q.W + 2 * q.pad;
    // filters of five rows or more are staged one filter row at a time
    const bool rows = q.R >= 5;
    a.Rp = rows ? 1 : q.R;
    a.nr = q.R / a.Rp;
    a.RSp = a.Rp * q.S;
    a.prs = a.Rp == 1 ? 1 : q.stride; a.irs = a.Rp == 1 ? q.stride : 1;
    a.pcs = q.S == 1 ? 1 : q.stride; a.ics = q.S == 1 ? q.stride : 1;
    // a reduction of one 16-byte unit runs unpaired instead of staging a second unit of zeros
    a.single = (E::BYTES == 16 && q.C == 1) ? 1 : 0;
    if (a.single) cb = 1;
    a.CB = cb;
    a.nstages = (q.C + cb - 1) / cb * a.nr;
    a.D = cb * a.RSp;
    a.LDA = (a.D + 1) | 1;   // odd pitch (D is even unless single), at least 3
    a.rows_full = (q.P - 1) * a.prs + a.Rp;
    const int rows_alloc = patch_rows_bound(q, T::BN, a.Rp);
    a.a_stage = (T::BM * a.LDA + T::NT - 1) / T::NT * T::NT;
    a.b_stage = (cb * rows_alloc * a.Wp + T::NT - 1) / T::NT * T::NT;
    a.magic_Wp = div_magic((uint32_t)a.Wp); a.one_Wp = a.Wp == 1 ? 0xFFFFFFFFu : 0u;
    a.magic_rf = div_magic((uint32_t)a.rows_full); a.one_rf = a.rows_full == 1 ? 0xFFFFFFFFu : 0u;
    a.magic_lda = div_magic((uint32_t)a.LDA);
    a.magic_S = div_magic((uint32_t)q.S); a.one_S = q.S == 1 ? 0xFFFFFFFFu : 0u;
    a.magic_nr = div_magic((uint32_t)a.nr); a.one_nr = a.nr == 1 ? 0xFFFFFFFFu : 0u;
    a.recip_PQ = div_recip((uint32_t)a.PQ);
    a.recip_Q = div_recip((uint32_t)q.Q);
    a.in_bytes = (uint64_t)q.N * a.CHW * E::BYTES;
    a.wt_bytes = (uint64_t)q.K * a.Kg * E::BYTES;
    a.out_bytes = (uint64_t)q.N * q.K * a.PQ * 4;
    a.tiles_m = (q.K + T::BM - 1) / T::BM;
    a.tiles_n = (a.Ng + T::BN - 1) / T::BN;
    a.raster = raster;
    a.act = q.act;
    // what one thread may hold, and the LDS a workgroup may take
    if ((long)a.a_stage > (long)MAXA * T::NT) return hipErrorInvalidConfiguration;
    if ((long)a.b_stage > (long)MAXP * T::NT) return hipErrorInvalidConfiguration;
    const int tiles = a.tiles_m * a.tiles_n;
    if (split_k < 1) split_k = 1;
    if (split_k > a.nstages) split_k = a.nstages;
    a.stages_per_split = (a.nstages + split_k - 1) / split_k;
    a.split_k = (a.nstages + a.stages_per_split - 1) / a.stages_per_split;
    a.recip_split = div_recip((uint32_t)a.split_k);
    if (a.split_k > 65535) return hipErrorInvalidConfiguration;
    // one stage buffer is enough when no workgroup runs more than one stage
    a.nbuf = a.stages_per_split > 1 ? 2 : 1;
    // the stage buffers and the zero unit behind them (kept a whole 64-unit row for alignment)
    const size_t lds_bytes = ((size_t)a.nbuf * ((size_t)a.a_stage + a.b_stage) + 64) * E::BYTES;
    if (lds_bytes > kMaxLdsBytes) return hipErrorInvalidConfiguration;
    // 31-bit byte offsets: filter rows of one tile, and the images one pixel run touches (input and output)
    const long PQl = a.PQ;
    const long imgs = (T::BN - 1 + PQl - 1) / PQl + 1;
    if ((long)T::BM * a.Kg * E::BYTES >= 0x7FFFFFF0l || (imgs * q.C + cb) * (long)a.HW * E::BYTES >= 0x7FFFFFF0l ||
        (imgs + 1) * (long)q.K * PQl * 4 >= 0x7FFFFFF0l)
        return hipErrorInvalidConfiguration;
    if (dry) return hipSuccess;
    hipError_t le = hipSuccess;
    a.partials = nullptr;
    a.counters = nullptr;
    const int cut_tiles = a.split_k > 1 ? tiles : 0;
    if (cut_tiles > 0) {
        const size_t bytes = (size_t)cut_tiles * a.split_k * T::BM * T::BN * sizeof(float);
        hipError_t e = splitk_scratch(stream, q.arena, bytes, cut_tiles, &a.partials, &a.counters);
        if (e != hipSuccess) return e;
    }
    const long nwg = (long)(tiles - cut_tiles) + (long)cut_tiles * a.split_k;
    if (nwg > 0x7FFFFFFFl) return hipErrorInvalidConfiguration;
    dim3 grid((unsigned)nwg, 1u), block(T::NT);
    void (*kern)(ConvPatchKArgs) = conv_patch_kernel<E, T, MAXA, MAXP, 0, 0>;
    if (q.R == 1 && q.S == 1) kern = conv_patch_kernel<E, T, MAXA, MAXP, 1, 1>;
    else if (q.R == 3 && q.S == 3) kern = conv_patch_kernel<E, T, MAXA, MAXP, 3, 3>;
    if (rows) {
        kern = conv_patch_kernel<E, T, MAXA, MAXP, 0, 0, true>;
        if (q.S == 7) kern = conv_patch_kernel<E, T, MAXA, MAXP, 1, 7, true>;
    }
    if (lds_bytes > 64 * 1024) {
        // more than the default per-workgroup LDS window has to be asked for, per kernel
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
    }
    le = launch_kernel(kern, grid, block, lds_bytes, stream, a);
    return le;
}

#define POLYDL_DEFINE_CONV_PATCH(BM, BN, BK, WM, WN)                                                     \
    hipError_t conv_patch_launch_##BM##x##BN##_##WM##x##WN(const ConvProblem &q, int cb, int sk, int r,    \
                                                           hipStream_t st, bool dry)                     \
    {                                                                                                    \
        /* the instantiation with fewer per-thread passes needs fewer registers: more waves per SIMD */ \
        if (conv_patch_launch<ElemF32, Tile<BM, BN, 8, WM, WN>, 6, 4>(q, cb, sk, r, st, true) == hipSuccess)         \
            return conv_patch_launch<ElemF32, Tile<BM, BN, 8, WM, WN>, 6, 4>(q, cb, sk, r, st, dry);                 \
        if (conv_patch_launch<ElemF32, Tile<BM, BN, 8, WM, WN>, 12, 8>(q, cb, sk, r, st, true) == hipSuccess)        \
            return conv_patch_launch<ElemF32, Tile<BM, BN, 8, WM, WN>, 12, 8>(q, cb, sk, r, st, dry);                \
        return conv_patch_launch<ElemF32, Tile<BM, BN, 8, WM, WN>, 40, 32>(q, cb, sk, r, st, dry);                   \
    }
POLYDL_PATCH_FAMILY(POLYDL_DEFINE_CONV_PATCH)

// bfloat16 (units of eight channels) launchers: same kernel, 16-byte elements
#define POLYDL_DEFINE_CONV_PATCH_BF16(BM, BN, BK, WM, WN)                                                \
    hipError_t conv_patch_bf16_launch_##BM##x##BN##_##WM##x##WN(const ConvProblem &q, int cb, int sk,      \
                                                                int r, hipStream_t st, bool dry)         \
    {                                                                                                    \
        return conv_patch_launch<ElemBF16x8, Tile<BM, BN, 8, WM, WN>, 16, 16>(q, cb, sk, r, st, dry);        \
    }
POLYDL_PATCH_BF16_FAMILY(POLYDL_DEFINE_CONV_PATCH_BF16)

// 2 or 1 if the problem runs in an instantiation with few per-thread passes (fewer registers,
// more waves per SIMD; 2 is the smallest), 0 if it needs the large one, -1 if none holds it.
#define POLYDL_DEFINE_PATCH_CLASS(BM, BN, BK, WM, WN)                                                   \
    int conv_patch_class_##BM##x##BN##_##WM##x##WN(const ConvProblem &q, int cb)                         \
    {                                                                                                    \
        if (conv_patch_launch<ElemF32, Tile<BM, BN, 8, WM, WN>, 6, 4>(q, cb, 1, 0, nullptr, true) == hipSuccess)    \
            return 2;                                                                                    \
        if (conv_patch_launch<ElemF32, Tile<BM, BN, 8, WM, WN>, 12, 8>(q, cb, 1, 0, nullptr, true) == hipSuccess)   \
            return 1;                                                                                    \
        return conv_patch_launch<ElemF32, Tile<BM, BN, 8, WM, WN>, 40, 32>(q, cb, 1, 0, nullptr, true) == hipSuccess \
                   ? 0 : -1;                                                                             \
    }
POLYDL_PATCH_FAMILY(POLYDL_DEFINE_PATCH_CLASS)

}  // namespace polydl
