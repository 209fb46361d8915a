// Tiled matrix-core GEMM main loop shared by the SGEMM and implicit-GEMM convolution kernels.
//
// Structure (figure "A code version generated for PolyDL", section "GEMM"): the outer tiling
// level is the workgroup tile BM x BN x BK staged through LDS, the inner level is the wave tile
// WM x WN held in accumulator registers for the whole reduction -- the role of the register
// resident microkernel of algorithm "The GEMM Microkernel" (load C once, a chain of rank-k
// updates, store C once).  Each rank-2 update is one v_mfma_f32_32x32x2_f32.
//
// Operand order inside a stage: the microkernel may visit the reduction in any order as long as
// both operands agree (section "Microkernel Specification": only the data set touched has to be
// the same).  A lane therefore reads four consecutive k of A with one 128-bit LDS read and uses
// them in four successive MFMAs; the lane's upper half (lane/32) takes the next four k.  B is
// read with k-slot (lane/32)*4+t to match.  Columns are permuted the same way: one LDS read of
// NB consecutive columns feeds the NB column blocks of the wave, so a lane ends up owning NB
// adjacent output columns and the epilogue stores them as one vector.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/polydl.h"

namespace polydl {

typedef float v2f __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef int v4i __attribute__((ext_vector_type(4)));

// Offset that is out of range for every buffer descriptor built here (num_records < 2^31):
// a raw buffer load at or beyond num_records returns zero, which is how padding, ragged tile
// edges and the reduction tail are filled without branches.
static constexpr uint32_t kOobOffset = 0x80000000u;
static constexpr uint64_t kMaxRecords = 0x7FFFFFF0ull;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, uint64_t bytes)
{
    uint32_t rec = bytes > kMaxRecords ? (uint32_t)kMaxRecords : (uint32_t)bytes;
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), (short)0, (int)rec, 0x00020000);
}
__device__ __forceinline__ float buf_load1(__amdgpu_buffer_rsrc_t r, uint32_t byte_off)
{
    // the builtin returns the raw 32 bits as an integer
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, (int)byte_off, 0, 0));
}
__device__ __forceinline__ v4f buf_load4(__amdgpu_buffer_rsrc_t r, uint32_t byte_off)
{
    v4i v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_off, 0, 0);
    return __builtin_bit_cast(v4f, v);
}
// byte_off is per lane and the only part that is range-checked; uniform_off (the same for the
// whole wave) is added to the address after the check
__device__ __forceinline__ float buf_load1(__amdgpu_buffer_rsrc_t r, uint32_t byte_off, uint32_t uniform_off)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, (int)byte_off, (int)uniform_off, 0));
}
__device__ __forceinline__ void buf_store1(__amdgpu_buffer_rsrc_t r, uint32_t byte_off, uint32_t uniform_off, float v)
{
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, v), r, (int)byte_off, (int)uniform_off, 0);
}
__device__ __forceinline__ void buf_store2(__amdgpu_buffer_rsrc_t r, uint32_t byte_off, uint32_t uniform_off, v2f v)
{
    typedef int v2i __attribute__((ext_vector_type(2)));
    __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(v2i, v), r, (int)byte_off, (int)uniform_off, 0);
}
__device__ __forceinline__ void buf_store4(__amdgpu_buffer_rsrc_t r, uint32_t byte_off, uint32_t uniform_off, v4f v)
{
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4i, v), r, (int)byte_off, (int)uniform_off, 0);
}

// Blocks the wave until every vector-memory operation it has issued (loads, stores, direct-to-LDS
// loads) has completed: s_waitcnt vmcnt(0), the other counters left alone.  The immediate is the
// gfx9-family encoding (vmcnt in bits 3:0 and 15:14, expcnt 6:4 = 7, lgkmcnt 11:8 = 15), where
// stores count in vmcnt too; this library is built for gfx950 only.
__device__ __forceinline__ void wait_vmcnt0()
{
#if defined(__HIP_DEVICE_COMPILE__) && !defined(__gfx950__)
#error "s_waitcnt encoding and counter semantics below are those of gfx950"
#endif
    __builtin_amdgcn_s_waitcnt(0x0F70);
}

// n / d and n % d for any 32-bit n and d >= 1, given recip = floor(2^32 / d) (0xFFFFFFFF for
// d == 1): umulhi(n, recip) is the quotient or one below it, which one comparison settles.
__device__ __forceinline__ uint32_t div_by(uint32_t n, uint32_t d, uint32_t recip, uint32_t &rem)
{
    uint32_t q = __umulhi(n, recip);
    uint32_t r = n - q * d;
    if (r >= d) { ++q; r -= d; }
    rem = r;
    return q;
}

template <int BM_, int BN_, int BK_, int WM_, int WN_>
struct Tile {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_;
    static constexpr int WAVES_M = BM / WM, WAVES_N = BN / WN;
    static constexpr int NT = WAVES_M * WAVES_N * 64;
    static constexpr int MB = WM / 32, NB = WN / 32;  // 32x32 MFMA blocks per wave tile
    // Waves per SIMD the SGEMM kernel's register allocation is held to: the eight-block wave tiles need 128
    // accumulator registers and end a handful of registers above the 256 that still let two
    // waves share a SIMD; bounded, the few excess values (epilogue addresses) go to scratch.
    static constexpr int MIN_WAVES = MB * NB >= 8 ? 2 : 1;
    // where SGEMM runs the split stage schedule (gemm_stage): two chunks per stage, two blocks and more
    static constexpr bool SPLIT_STAGE = BK == 16 && MB * NB >= 2;
    static constexpr int LDA = BK + 4;                 // LDS row pitch of the A stage [BM][LDA]
    static constexpr int LDB = BN + 4;                 // LDS row pitch of the B stage [BK][LDB]
    static constexpr int A_STAGE = BM * LDA, B_STAGE = BK * LDB;
    static constexpr int LDS_FLOATS = 2 * (A_STAGE + B_STAGE);
    static_assert(BM % WM == 0 && BN % WN == 0 && WM % 32 == 0 && WN % 32 == 0, "tile shape");
    static_assert(BK % 8 == 0, "a stage is consumed in chunks of 8 reduction elements");
    static_assert(NB == 1 || NB == 2 || NB == 4, "column blocks per wave");
    static_assert(BN % 64 == 0 && NT % BN == 0, "gather loaders: one column per thread");
    static_assert(NT <= 512 && LDS_FLOATS * 4 <= 64 * 1024, "workgroup limits");
};

// ---- A operand: row-major [Mg][lda], reduction index contiguous ------------------------------
// VEC = 4: 128-bit loads (needs lda % 4 == 0 and a 16-byte aligned base); VEC = 1: dword loads.
// The descriptor is rebuilt per stage at A + m0*lda + k0, so offsets stay below BM*lda*4 bytes.
// KTAIL (VEC = 4 only): rows need not be a multiple of four long nor 16-byte aligned -- buffer loads
// of four dwords only need dword alignment -- so a vector may reach past the end of the reduction
// into the next row; in the (one) stage where that can happen those components are zeroed.
template <class T, int VEC, bool KTAIL = false>
struct ALoader {
    static_assert(!KTAIL || VEC == 4, "the tail form is for vector loads");
    static constexpr int UNITS = T::BM * T::BK / VEC;  // load units in one stage
    static constexpr int ITERS = (UNITS + T::NT - 1) / T::NT;
    static constexpr int UPR = T::BK / VEC;            // units per tile row
    static constexpr bool RAGGED = UNITS % T::NT != 0;
    const float *base;   // A + m0*lda
    uint64_t bytes;      // bytes from base to the end of A
    float regs[2][ITERS * VEC];  // two register sets: loads run two stages ahead
    uint32_t off0[ITERS];  // byte offset of the unit at k0 = 0, or kOobOffset if its row is outside
    int kcol[ITERS];       // first reduction index of the unit inside the stage
    int lds_off[ITERS];

    __device__ __forceinline__ void init(const float *A, int tid, int m0, int Mg, int Kg, int lda)
    {
        base = A + (size_t)m0 * lda;
        bytes = ((size_t)(Mg - m0 - 1) * lda + Kg) * 4;
#pragma unroll
        for (int i = 0; i < ITERS; ++i) {
            int u = tid + i * T::NT;
            int row = u / UPR, kc = (u % UPR) * VEC;
            bool ok = (!RAGGED || u < UNITS) && (m0 + row < Mg);
            off0[i] = ok ? ((uint32_t)row * (uint32_t)lda + (uint32_t)kc) * 4u : kOobOffset;
            kcol[i] = kc;
            lds_off[i] = row * T::LDA + kc;
        }
    }
    // loads reduction indices [k0, k0+BK), of which only those below kend exist, into set `set`
    template <int SET>
    __device__ __forceinline__ void load(int k0, int kend)
    {
        // past the end every lane reads out of range: clamp the base so it stays inside A
        const int kb = k0 < kend ? k0 : 0;
        __amdgpu_buffer_rsrc_t rsrc = make_rsrc(base + kb, bytes - (uint64_t)kb * 4);
        int krem = kend - k0;
#pragma unroll
        for (int i = 0; i < ITERS; ++i) {
            uint32_t off = (kcol[i] < krem) ? off0[i] : kOobOffset;
            if constexpr (VEC == 4) {
                v4f v = buf_load4(rsrc, off);
                regs[SET][4 * i] = v.x; regs[SET][4 * i + 1] = v.y; regs[SET][4 * i + 2] = v.z; regs[SET][4 * i + 3] = v.w;
            } else {
                regs[SET][i] = buf_load1(rsrc, off);
            }
        }
        if constexpr (KTAIL) {
            if (krem < T::BK) {   // uniform: the stage the reduction ends in
#pragma unroll
                for (int i = 0; i < ITERS; ++i)
#pragma unroll
                    for (int j = 1; j < 4; ++j)
                        if (kcol[i] + j >= krem) regs[SET][4 * i + j] = 0.f;
            }
        }
    }
    template <int SET>
    __device__ __forceinline__ void store(float *As, int tid) const
    {
#pragma unroll
        for (int i = 0; i < ITERS; ++i) {
            if (RAGGED && tid + i * T::NT >= UNITS) continue;
            if constexpr (VEC == 4) {
                v4f v = {regs[SET][4 * i], regs[SET][4 * i + 1], regs[SET][4 * i + 2], regs[SET][4 * i + 3]};
                *reinterpret_cast<v4f *>(As + lds_off[i]) = v;
            } else {
                As[lds_off[i]] = regs[SET][i];
            }
        }
    }
};

// ---- B operand of a plain GEMM: row-major [Kg][ldb], column index contiguous ------------------
// VEC = 4: 128-bit loads along the columns (needs ldb % 4 == 0, Ng % 4 == 0, aligned base);
// VEC = 1: dword loads.  The descriptor is rebuilt per stage at B + k0*ldb + n0.
template <class T, int VEC>
struct BLoaderRows {
    static constexpr int UNITS = T::BK * T::BN / VEC;
    static constexpr int ITERS = (UNITS + T::NT - 1) / T::NT;
    static constexpr int UPR = T::BN / VEC;
    static constexpr bool RAGGED = UNITS % T::NT != 0;
    const float *base;  // B + n0
    int Kg, ldb, ncols;  // ncols = Ng - n0
    float regs[2][ITERS * VEC];
    uint32_t off0[ITERS];
    int krow[ITERS];
    int lds_off[ITERS];

    __device__ __forceinline__ void init(const float *B, int tid, int n0, int Ng, int Kg_, int ldb_)
    {
        base = B + n0;
        Kg = Kg_;
        ldb = ldb_;
        ncols = Ng - n0;
#pragma unroll
        for (int i = 0; i < ITERS; ++i) {
            int u = tid + i * T::NT;
            int kr = u / UPR, nc = (u % UPR) * VEC;
            bool ok = (!RAGGED || u < UNITS) && (n0 + nc < Ng);
            off0[i] = ok ? ((uint32_t)kr * (uint32_t)ldb + (uint32_t)nc) * 4u : kOobOffset;
            krow[i] = kr;
            lds_off[i] = kr * T::LDB + nc;
        }
    }
    template <int SET>
    __device__ __forceinline__ void load(int k0, int kend)
    {
        const int kb = k0 < kend ? k0 : 0;   // past the end every lane reads out of range anyway
        // valid bytes from the stage's base: up to the last element of the last row of B
        uint64_t bytes = ((uint64_t)(Kg - kb - 1) * ldb + ncols) * 4;
        __amdgpu_buffer_rsrc_t rsrc = make_rsrc(base + (size_t)kb * ldb, bytes);
        int krem = kend - k0;
#pragma unroll
        for (int i = 0; i < ITERS; ++i) {
            uint32_t off = (krow[i] < krem) ? off0[i] : kOobOffset;
            if constexpr (VEC == 4) {
                v4f v = buf_load4(rsrc, off);
                regs[SET][4 * i] = v.x; regs[SET][4 * i + 1] = v.y; regs[SET][4 * i + 2] = v.z; regs[SET][4 * i + 3] = v.w;
            } else {
                regs[SET][i] = buf_load1(rsrc, off);
            }
        }
    }
    template <int SET>
    __device__ __forceinline__ void store(float *Bs, int tid) const
    {
#pragma unroll
        for (int i = 0; i < ITERS; ++i) {
            if (RAGGED && tid + i * T::NT >= UNITS) continue;
            if constexpr (VEC == 4) {
                v4f v = {regs[SET][4 * i], regs[SET][4 * i + 1], regs[SET][4 * i + 2], regs[SET][4 * i + 3]};
                *reinterpret_cast<v4f *>(Bs + lds_off[i]) = v;
            } else {
                Bs[lds_off[i]] = regs[SET][i];
            }
        }
    }
};

// ---- the MFMA stage: consume one LDS stage, WM x WN x BK per wave ----------------------------
// Two schedules.  The plain one: per chunk of eight reduction rows read the fragments, multiply;
// copy the next stage to LDS; barrier.  The split one, see gemm_stage: the stage is multiplied in
// two phases of one chunk each, the fragments of a phase are read from LDS one phase ahead into
// StageFrags.  SGEMM runs the split schedule on wave tiles of two 32x32 blocks and more, where one
// to three waves share a SIMD (measured at 2048^3 and 4096^3: 2-8 % faster on the 128x64, 128x128 and
// larger tiles, no change with 32x32 wave tiles, slower with a single chunk per stage).  The
// convolution kernels keep the plain one: over the suite and 28 further layer shapes the split
// schedule gave the same total (single layers 8 % faster or 6 % slower), because many waves share
// a SIMD there and the gather loaders' address arithmetic mixes less freely with the matrix
// instructions once the scheduling fences are in.
template <class T>
struct StageFrags {
    static constexpr int NC = T::BK / 8;
    v4f a[NC][T::MB];          // rows wm0 + 32*bi + lane%32, reduction 8*kc + 4*(lane/32) + {0..3}
    float b[NC][4][T::NB];     // reduction 8*kc + 4*(lane/32) + t, the lane's NB adjacent columns
};

// fragments of chunk kc: one 128-bit read per row block, one read of NB adjacent columns per rank-2 step
template <class T>
__device__ __forceinline__ void read_chunk(const float *__restrict__ As, const float *__restrict__ Bs,
                                           v4f (&a)[T::MB], float (&b)[4][T::NB], int kc, int wm0, int wn0, int lane)
{
    const int li = lane & 31, lh = lane >> 5;
#pragma unroll
    for (int bi = 0; bi < T::MB; ++bi)
        a[bi] = *reinterpret_cast<const v4f *>(As + (wm0 + 32 * bi + li) * T::LDA + kc * 8 + 4 * lh);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const float *p = Bs + (kc * 8 + 4 * lh + t) * T::LDB + wn0 + T::NB * li;
        if constexpr (T::NB == 4) {
            v4f v = *reinterpret_cast<const v4f *>(p);
            b[t][0] = v.x; b[t][1] = v.y; b[t][2] = v.z; b[t][3] = v.w;
        } else if constexpr (T::NB == 2) {
            v2f v = *reinterpret_cast<const v2f *>(p);
            b[t][0] = v.x; b[t][1] = v.y;
        } else {
            b[t][0] = *p;
        }
    }
}

template <class T>
__device__ __forceinline__ void mma_chunk(const v4f (&a)[T::MB], const float (&b)[4][T::NB], v16f (&acc)[T::MB][T::NB])
{
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int bi = 0; bi < T::MB; ++bi)
#pragma unroll
            for (int bj = 0; bj < T::NB; ++bj)
                acc[bi][bj] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[bi][t], b[t][bj], acc[bi][bj], 0, 0, 0);
}

// The plain schedule's stage.  krem: reduction rows of this stage that exist (the last stage of a
// reduction may be short; its other rows are zeros in A).  A chunk of eight rows that lies wholly
// past the end is skipped (uniform branch): the stem layer's reduction of 147 ends three rows into
// its tenth stage.
template <class T>
__device__ __forceinline__ void mma_stage(const float *__restrict__ As, const float *__restrict__ Bs,
                                          v16f (&acc)[T::MB][T::NB], int wm0, int wn0, int lane, int krem)
{
    const int li = lane & 31, lh = lane >> 5;
#pragma unroll
    for (int kc = 0; kc < T::BK / 8; ++kc) {
        if (kc > 0 && kc * 8 >= krem) break;
        v4f a[T::MB];
#pragma unroll
        for (int bi = 0; bi < T::MB; ++bi)
            a[bi] = *reinterpret_cast<const v4f *>(As + (wm0 + 32 * bi + li) * T::LDA + kc * 8 + 4 * lh);
        float b[4][T::NB];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const float *p = Bs + (kc * 8 + 4 * lh + t) * T::LDB + wn0 + T::NB * li;
            if constexpr (T::NB == 4) {
                v4f v = *reinterpret_cast<const v4f *>(p);
                b[t][0] = v.x; b[t][1] = v.y; b[t][2] = v.z; b[t][3] = v.w;
            } else if constexpr (T::NB == 2) {
                v2f v = *reinterpret_cast<const v2f *>(p);
                b[t][0] = v.x; b[t][1] = v.y;
            } else {
                b[t][0] = *p;
            }
        }
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int bi = 0; bi < T::MB; ++bi)
#pragma unroll
                for (int bj = 0; bj < T::NB; ++bj)
                    acc[bi][bj] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[bi][t], b[t][bj], acc[bi][bj], 0, 0, 0);
    }
}

// Software-pipelined reduction over [kbegin, kend).  Global loads run two stages ahead of the
// matrix cores: while stage t is multiplied out of LDS buffer t&1, the registers of set (t+1)&1
// already hold stage t+1 and the loads of stage t+2 are issued into set t&1.  A load therefore
// has two full stages of MFMA work (several thousand cycles) to come back from HBM before its
// data is copied to LDS during the following stage; one barrier per stage publishes the copy.  A
// loader that runs past kend fills with zeros, so the tail needs no special case.
//
// Split schedule: the barrier sits in the MIDDLE of the stage, between its two chunks.  Before it
// a wave reads the fragments of the second chunk and copies stage t+1 to the other LDS buffer;
// after it the wave still has the whole second chunk to multiply with operands that are already
// in registers, and reads the first chunk of stage t+1 (published by that barrier) underneath.
// So no matrix instruction waits for a barrier and then for an LDS read behind it.  Why the
// buffers do not collide: buffer b is read by stage t only -- first chunk after the barrier of
// stage t-1, second chunk before the barrier of stage t, where every wave waits for its own LDS
// reads before it arrives -- and written (with stage t+2) before the barrier of stage t+1, i.e.
// after every wave has passed the barrier of stage t.  The scheduling fences keep the compiler
// from moving the second chunk's matrix instructions up across the barrier, where nothing but
// memory order holds them, and from sinking the LDS reads down to their first use.
template <class T, int HALF, bool SPLIT, class AL, class BL>
__device__ __forceinline__ void gemm_stage(float *As, float *Bs, AL &al, BL &bl, v16f (&acc)[T::MB][T::NB],
                                           StageFrags<T> &f, int k, int kend, int tid, int wm0, int wn0)
{
    const int lane = tid & 63;
    if constexpr (!SPLIT) {
        // register set HALF is free (its stage is in LDS buffer HALF): fetch stage k + 2*BK into it
        al.template load<HALF>(k + 2 * T::BK, kend);
        bl.template load<HALF>(k + 2 * T::BK, kend);
        mma_stage<T>(As + HALF * T::A_STAGE, Bs + HALF * T::B_STAGE, acc, wm0, wn0, lane, kend - k);
        // stage k + BK sits in the other set: copy it to the other LDS buffer
        al.template store<HALF ^ 1>(As + (HALF ^ 1) * T::A_STAGE, tid);
        bl.template store<HALF ^ 1>(Bs + (HALF ^ 1) * T::B_STAGE, tid);
        __syncthreads();
    } else {
        read_chunk<T>(As + HALF * T::A_STAGE, Bs + HALF * T::B_STAGE, f.a[1], f.b[1], 1, wm0, wn0, lane);
        __builtin_amdgcn_sched_barrier(0);
        al.template load<HALF>(k + 2 * T::BK, kend);
        bl.template load<HALF>(k + 2 * T::BK, kend);
        mma_chunk<T>(f.a[0], f.b[0], acc);
        al.template store<HALF ^ 1>(As + (HALF ^ 1) * T::A_STAGE, tid);
        bl.template store<HALF ^ 1>(Bs + (HALF ^ 1) * T::B_STAGE, tid);
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
        read_chunk<T>(As + (HALF ^ 1) * T::A_STAGE, Bs + (HALF ^ 1) * T::B_STAGE, f.a[0], f.b[0], 0, wm0, wn0, lane);
        __builtin_amdgcn_sched_barrier(0);
        if (kend - k > 8) mma_chunk<T>(f.a[1], f.b[1], acc);   // uniform: a short last stage ends in its first chunk
    }
}

template <class T, bool SPLIT, class AL, class BL>
__device__ __forceinline__ void gemm_mainloop(float *lds, AL &al, BL &bl, v16f (&acc)[T::MB][T::NB],
                                              int kbegin, int kend, int tid, int wm0, int wn0)
{
    float *As = lds;
    float *Bs = lds + 2 * T::A_STAGE;
    StageFrags<T> f;   // used by the split schedule only
    // stage 0 -> LDS buffer 0, stage 1 -> register set 1
    al.template load<0>(kbegin, kend);
    bl.template load<0>(kbegin, kend);
    al.template load<1>(kbegin + T::BK, kend);
    bl.template load<1>(kbegin + T::BK, kend);
    al.template store<0>(As, tid);
    bl.template store<0>(Bs, tid);
    __syncthreads();
    if constexpr (SPLIT) read_chunk<T>(As, Bs, f.a[0], f.b[0], 0, wm0, wn0, tid & 63);
    // Stages go in pairs, both halves unconditionally, and an odd last stage is peeled off: with a
    // conditional second half inside the loop the compiler has to assume at the loop head that the
    // loads of the first half may still be in flight into the registers the head overwrites, and it
    // waits there for loads that were issued only one stage earlier.
    int k0 = kbegin;
    for (; k0 + T::BK < kend; k0 += 2 * T::BK) {
        gemm_stage<T, 0, SPLIT>(As, Bs, al, bl, acc, f, k0, kend, tid, wm0, wn0);
        gemm_stage<T, 1, SPLIT>(As, Bs, al, bl, acc, f, k0 + T::BK, kend, tid, wm0, wn0);
    }
    if (k0 < kend)   // workgroup-uniform
        gemm_stage<T, 0, SPLIT>(As, Bs, al, bl, acc, f, k0, kend, tid, wm0, wn0);
}

// Sum of the `parts` partial accumulator tiles of one output tile, in index order (so the result
// does not depend on which part arrived last).  Tiles lie TILE floats apart, each in register
// order (thread-contiguous).  The loads are device-scope.  (Requesting part i+1 before part i is
// added measured no faster: other workgroups fill the compute unit while the last one of a tile sums.)
template <class T>
__device__ __forceinline__ void sum_partial_tiles(const float *tile0, int parts, size_t TILE, int tid,
                                                  v16f (&acc)[T::MB][T::NB])
{
    constexpr int R = T::MB * T::NB * 16, NT = T::NT;
    auto fetch = [&](float (&dst)[R], int sp) {
        const float *part = tile0 + (size_t)sp * TILE + tid;
#pragma unroll
        for (int i = 0; i < R; ++i) dst[i] = __hip_atomic_load(part + (size_t)i * NT, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    };
    auto add = [&](const float (&src)[R]) {
#pragma unroll
        for (int bi = 0; bi < T::MB; ++bi)
#pragma unroll
            for (int bj = 0; bj < T::NB; ++bj)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[bi][bj][r] += src[(bi * T::NB + bj) * 16 + r];
    };
#pragma unroll
    for (int bi = 0; bi < T::MB; ++bi)
#pragma unroll
        for (int bj = 0; bj < T::NB; ++bj)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[bi][bj][r] = 0.f;
    float a[R];
    for (int sp = 0; sp < parts; ++sp) {
        fetch(a, sp);
        add(a);
    }
}

// Row (inside the workgroup tile) of accumulator register r of row block bi for this lane: a
// 32x32 result keeps column lane%32 in every register and row 8*(r/4) + 4*(lane/32) + r%4 in
// register r.  With the column permutation above the lane's NB blocks are the NB adjacent
// columns starting at NB*(lane%32) of the wave tile.
__device__ __forceinline__ int acc_row(int wm0, int bi, int r, int lane)
{
    return wm0 + 32 * bi + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
}

template <int ACT>
__device__ __forceinline__ float act_of(float v)
{
    if constexpr (ACT != POLYDL_ACT_NONE) v = fmaxf(v, 0.f);
    if constexpr (ACT == POLYDL_ACT_RELU6) v = fminf(v, 6.f);
    return v;
}

// Bias, activation and store of the lane's 16*MB channel rows, NB adjacent pixels each as one
// vector.  `off` is the lane's byte offset of channel row `krow`; row c of the tile lies c*row_bytes
// further, a uniform offset.  FULL: every channel row of the tile exists.
template <class T, int ACT, bool FULL>
__device__ __forceinline__ void store_rows(__amdgpu_buffer_rsrc_t ro, uint32_t off, uint32_t row_bytes,
                                           const v16f (&acc)[T::MB][T::NB], const float (&bias)[T::MB][16], int krow,
                                           int K)
{
#pragma unroll
    for (int bi = 0; bi < T::MB; ++bi)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int c = 32 * bi + 8 * (r >> 2) + (r & 3);
            if (!FULL && krow + c >= K) continue;
            const float b = bias[bi][r];
            if constexpr (T::NB == 4) {
                v4f v = {act_of<ACT>(acc[bi][0][r] + b), act_of<ACT>(acc[bi][1][r] + b), act_of<ACT>(acc[bi][2][r] + b),
                         act_of<ACT>(acc[bi][3][r] + b)};
                buf_store4(ro, off, (uint32_t)c * row_bytes, v);
            } else if constexpr (T::NB == 2) {
                v2f v = {act_of<ACT>(acc[bi][0][r] + b), act_of<ACT>(acc[bi][1][r] + b)};
                buf_store2(ro, off, (uint32_t)c * row_bytes, v);
            } else {
                buf_store1(ro, off, (uint32_t)c * row_bytes, act_of<ACT>(acc[bi][0][r] + b));
            }
        }
}

// The same with the two uniform choices -- which activation, and whether every channel row of
// the tile exists -- made once, outside the run of stores.
template <class T>
__device__ __forceinline__ void store_rows_by(int act, bool full, __amdgpu_buffer_rsrc_t ro, uint32_t off,
                                              uint32_t row_bytes, const v16f (&acc)[T::MB][T::NB],
                                              const float (&bias)[T::MB][16], int krow, int K)
{
    if (full) {
        if (act == POLYDL_ACT_NONE) store_rows<T, POLYDL_ACT_NONE, true>(ro, off, row_bytes, acc, bias, krow, K);
        else if (act == POLYDL_ACT_RELU) store_rows<T, POLYDL_ACT_RELU, true>(ro, off, row_bytes, acc, bias, krow, K);
        else store_rows<T, POLYDL_ACT_RELU6, true>(ro, off, row_bytes, acc, bias, krow, K);
    } else {
        if (act == POLYDL_ACT_NONE) store_rows<T, POLYDL_ACT_NONE, false>(ro, off, row_bytes, acc, bias, krow, K);
        else if (act == POLYDL_ACT_RELU) store_rows<T, POLYDL_ACT_RELU, false>(ro, off, row_bytes, acc, bias, krow, K);
        else store_rows<T, POLYDL_ACT_RELU6, false>(ro, off, row_bytes, acc, bias, krow, K);
    }
}

// Workgroup index -> tile coordinates.  raster 0: tile rows fastest.  raster 1: the hardware
// deals consecutive workgroups round-robin to the 8 XCDs, each with its own L2; give every XCD
// one contiguous chunk of the tile sequence and walk the sequence in bands of 8 tile rows, so
// that tiles resident together share A row panels and B column panels in that L2.
__device__ __forceinline__ void tile_coords(int pid, int raster, int tiles_m, int tiles_n, int &tm, int &tn)
{
    if (raster == 1) {
        const int XCD = 8, GROUP = 8;
        int total = tiles_m * tiles_n;
        int per = total / XCD, rem = total % XCD;
        int x = pid % XCD, local = pid / XCD;
        int seq = x * per + (x < rem ? x : rem) + local;
        int band = GROUP * tiles_n;
        int g = seq / band, first_m = g * GROUP;
        int gsz = tiles_m - first_m < GROUP ? tiles_m - first_m : GROUP;
        int in_band = seq - g * band;
        tm = first_m + in_band % gsz;
        tn = in_band / gsz;
    } else {
        tm = pid % tiles_m;
        tn = pid / tiles_m;
    }
}

}  // namespace polydl
