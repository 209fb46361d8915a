// Host-side declarations shared by the API file and the kernel files (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <tuple>
#include <utility>
#include <vector>
#include "../../include/polydl.h"

namespace polydl {

// Where a split-reduction launch takes its partial tiles and arrival counters from when not from
// the library's own per-stream buffers.
struct ScratchArena {
    float *partials = nullptr;
    size_t partial_bytes = 0;
    unsigned *counters = nullptr;
    int ncounters = 0;
    bool clear_counters = false;   // zero the counters a launch will use (small kernel on its stream) first
};

struct SgemmProblem {
    int M, N, K;
    const float *A, *B;
    float *C;
    float alpha = 1.f, beta = 1.f;   // C = beta*C + alpha*A*B
    const ScratchArena *arena = nullptr;
};

struct ConvProblem {
    int N, C, H, W, K, R, S, stride, pad, P, Q;
    const void *in, *wt;   // float tensors, or tensors of eight-bfloat16 units for the bf16 kernels
    const float *bias;
    float *out;
    int act;
    int pre_act = 0;       // polydl_act applied to every input element as it is read (gather kernel only)
    const ScratchArena *arena = nullptr;   // split reductions: nullptr = the library's per-stream buffers
    // fp32: the caller also holds the filter as [K][R][S][C] (tile layout 2, gather kernel only).  The
    // launchers read wt_tap instead of wt when it is set; the picker only looks at has_tap.
    const float *wt_tap = nullptr;
    bool has_tap = false;
};

// Whether the gather kernel can walk the reduction tap by tap (tile layout 2; bk = stage depth): 2..63 taps,
// whole stages inside one tap, and C * (C*R*S) below 2^32 for its exact division by C.
inline bool gather_tap_major_fits(const ConvProblem &q, int bk)
{
    const int64_t RS = (int64_t)q.R * q.S;
    return RS >= 2 && RS <= 63 && q.C % bk == 0 && RS * q.C * q.C < (1ll << 32);
}

// One compiled variant: its tile parameters and the launchers instantiated for it.
struct Variant {
    int bm, bn, bk, wm, wn;
    int threads;
    int lds_bytes;
    hipError_t (*sgemm)(const SgemmProblem &, int split_k, int raster, hipStream_t);
    hipError_t (*conv)(const ConvProblem &, int split_k, int raster, hipStream_t);
};

// One compiled tile of the row-patch convolution kernel.  dry = true only checks that the
// problem fits the kernel's register, LDS and offset limits with cb channels per stage.
struct PatchVariant {
    int bm, bn, wm, wn;
    int threads;
    hipError_t (*conv)(const ConvProblem &, int cb, int split_k, int raster, hipStream_t, bool dry);
    int (*reg_class)(const ConvProblem &, int cb);   // 2, 1: small-register instantiations, 0 large, -1 none
};

extern const Variant kVariants[];
extern const int kNumVariants;
extern const PatchVariant kPatchVariants[];
extern const PatchVariant kPatchBf16Variants[];
extern const int kNumPatchBf16Variants;
extern const int kNumPatchVariants;

// filled in by the kernel files
#define POLYDL_DECLARE_LAUNCHERS(BM, BN, BK, WM, WN)                                                          \
    hipError_t sgemm_launch_##BM##x##BN##x##BK##_##WM##x##WN(const SgemmProblem &, int, int, hipStream_t);     \
    hipError_t conv_launch_##BM##x##BN##x##BK##_##WM##x##WN(const ConvProblem &, int, int, hipStream_t);

#define POLYDL_DECLARE_PATCH_BF16_LAUNCHER(BM, BN, BK, WM, WN) \
    hipError_t conv_patch_bf16_launch_##BM##x##BN##_##WM##x##WN(const ConvProblem &, int, int, int, hipStream_t, bool);

#define POLYDL_DECLARE_PATCH_LAUNCHER(BM, BN, BK, WM, WN) \
    hipError_t conv_patch_launch_##BM##x##BN##_##WM##x##WN(const ConvProblem &, int, int, int, hipStream_t, bool); \
    int conv_patch_class_##BM##x##BN##_##WM##x##WN(const ConvProblem &, int);

hipError_t launch_nchwc(const void *src, void *dst, int N, int C, int HW, int b, bool to_blocked, int elem_bytes,
                        hipStream_t st);
hipError_t launch_kcrsck(const void *wt, void *dst, int K, int C, int RS, int bc, int bk, int elem_bytes,
                         hipStream_t st);
hipError_t launch_bias_add(float *y, const float *bias, int K, int PQ, size_t total, hipStream_t st);
hipError_t launch_act(float *y, size_t total, int act, hipStream_t st);
hipError_t launch_bnorm_act(const float *x, float *y, const float *gamma, const float *beta, const float *mean,
                            const float *var, float eps, int K, int PQ, size_t total, int act, hipStream_t st);

// scratch.hip: partial-tile buffer (>= partial_bytes) and zeroed arrival counters (>= tiles) for a
// split-reduction launch, from `arena` or (arena == nullptr) from the buffers the library keeps for
// this device and stream.  On failure scratch_refusal() tells this thread why, when the reason is
// not the runtime's: the arena is too small, or the library's buffers would have to grow while the
// stream is being captured.
enum { SCRATCH_OK = 0, SCRATCH_TOO_SMALL = 1, SCRATCH_CAPTURING = 2 };
hipError_t splitk_scratch(hipStream_t stream, const ScratchArena *arena, size_t partial_bytes, int tiles,
                          float **partials, unsigned **counters);
int scratch_refusal();
// the fixed scratch array of the current device (address looked up on the first call per device)
constexpr size_t kStaticCounterBytes = 64 * 1024;            // 16384 tiles
constexpr size_t kStaticPartialBytes = 64 * 1024 * 1024;
hipError_t static_scratch_arena(ScratchArena *arena);
int compute_units();   // of the current device

// Workgroups of one launch are all resident at once or run in rounds; either way a compute unit
// takes a whole number of them, so `tiles % cus` leftover tiles make one more round that most
// compute units sit out.  When those leftovers would occupy at most half of the compute units,
// the gather kernel cuts each of them into `parts` pieces along the reduction (one workgroup
// each, summed through scratch tiles like any split reduction), so that the last round is short
// for everyone.  parts == 1: no tail split.
struct TailSplit { int tiles, parts, stages_per_part; };
inline TailSplit tail_split(int tiles, int stages, int cus)
{
    TailSplit t{0, 1, stages};
    const int rem = tiles % cus;
    if (tiles <= cus || rem == 0 || rem * 2 > cus || stages < 2) return t;
    int want = cus / rem;
    if (want > stages) want = stages;
    if (want < 2) return t;
    t.stages_per_part = (stages + want - 1) / want;
    t.parts = (stages + t.stages_per_part - 1) / t.stages_per_part;
    t.tiles = t.parts > 1 ? rem : 0;
    return t;
}

// Launch with the runtime's verdict as the return value (hipGetLastError() would also report, and
// clear, errors other code of this thread left behind).  Arguments are converted to the kernel's
// parameter types.
template <class... P, size_t... I>
inline hipError_t launch_kernel_impl(void (*kernel)(P...), dim3 grid, dim3 block, size_t lds, hipStream_t st,
                                     std::tuple<P...> &vals, std::index_sequence<I...>)
{
    void *ptrs[] = {static_cast<void *>(&std::get<I>(vals))...};
    return hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, ptrs, lds, st);
}
template <class... P, class... A>
inline hipError_t launch_kernel(void (*kernel)(P...), dim3 grid, dim3 block, size_t lds, hipStream_t st, A... args)
{
    static_assert(sizeof...(P) == sizeof...(A), "argument count");
    std::tuple<P...> vals{static_cast<P>(args)...};
    return launch_kernel_impl(kernel, grid, block, lds, st, vals, std::index_sequence_for<P...>{});
}

// picker.cpp
void reuse_bucket(int n, const double *ws, int nlevels, const double *sizes, double *levels, double *mem);
double reuse_cost(int nlevels, const double *levels, double mem, const double *weights, double mem_weight);
void model_get_levels(double *capacity, double *gbytes_per_s, double *mem_gbytes_per_s);   // 4 levels + memory
void model_set_levels(const double *capacity, const double *gbytes_per_s, double mem_gbytes_per_s);
void model_conv(const ConvProblem &q, const polydl_tile_cfg &cfg, int threads, int reg_class, polydl_model_report *r);
void model_sgemm(const SgemmProblem &q, const polydl_tile_cfg &cfg, int threads, polydl_model_report *r);
double model_conv_bf16(const ConvProblem &q, const polydl_tile_cfg &cfg, int threads);   // predicted microseconds
bool pick_conv(const ConvProblem &q, polydl_tile_cfg *best, polydl_model_report *rep);   // q.pre_act: gather kernel only
bool pick_sgemm(const SgemmProblem &q, polydl_tile_cfg *best, polydl_model_report *rep);
struct ConvCandidate { polydl_tile_cfg cfg; polydl_model_report rep; };
// every (variant, stage depth, split factor, leftover-tile switch) pick_conv ranks, with its model report
void conv_candidates(const ConvProblem &q, std::vector<ConvCandidate> *out);
void sgemm_candidates(const SgemmProblem &q, std::vector<polydl_tile_cfg> *out);

// conv_point.hip: pointwise convolution with the filter resident in LDS (cfg.algo == 2; one variant:
// 32 output channels x 64 pixels per wave and unit, 256 threads)
bool conv_point_fits(const ConvProblem &q);
void conv_point_shape(const ConvProblem &q, int cus, uint32_t *units, uint32_t *workgroups);
hipError_t conv_point_launch(const ConvProblem &q, hipStream_t stream);
void model_conv_point(const ConvProblem &q, polydl_model_report *r);
inline polydl_tile_cfg conv_point_cfg() { return polydl_tile_cfg{32, 64, 0, 32, 64, 1, 0, 0, 2, 0}; }
inline bool is_conv_point_cfg(const polydl_tile_cfg &c)
{
    return c.algo == 2 && c.bm == 32 && c.bn == 64 && c.bk == 0 && c.wm == 32 && c.wn == 64 && c.split_k <= 1 &&
           c.layout == 0 && c.raster == 0 && c.cb == 0;
}

// reuse_analyse.cpp (arguments already validated)
int reuse_analyse(int nloops, const int *extents, const int *parallel, int nrefs, const polydl_loop_ref *refs,
                  int max_deps, polydl_reuse_dep *deps, int *ndeps);

// ranker.cpp
int ranker_num_params();
void ranker_set_params(const double *params);   // ranker_num_params() doubles, copied
bool ranker_ready();
void ranker_stats(const polydl_model_report &r, double *stats);   // POLYDL_RANKER_STATS doubles
// false while no parameters are loaded
bool ranker_play(const double *stats1, const double *stats2, double theta, double *probs, int *winner);
bool ranker_tournament(int n, const double *stats, double theta, int *wins, int *order);

// Exact unsigned division by a runtime constant d for dividends n with n*d < 2^32:
// n / d == (n * magic) >> 32 with magic = floor(2^32 / d) + 1.
inline uint32_t div_magic(uint32_t d) { return d == 1 ? 0u : (uint32_t)((1ull << 32) / d) + 1u; }


// Reciprocal for the device-side div_by(): floor(2^32 / d), saturated for d == 1.
inline uint32_t div_recip(uint32_t d) { return d <= 1 ? 0xFFFFFFFFu : (uint32_t)((1ull << 32) / d); }

}  // namespace polydl
