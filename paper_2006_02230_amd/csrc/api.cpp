// The C ABI: argument checks, variant choice, launch.  No data is touched on the host.
#include <hip/hip_runtime.h>
#include <atomic>
#include <algorithm>
#include <cstring>
#include <array>
#include <map>
#include <mutex>
#include <vector>
#include "internal.hpp"
#include "variants.hpp"

namespace polydl {

POLYDL_TILE_FAMILY(POLYDL_DECLARE_LAUNCHERS)
POLYDL_PATCH_FAMILY(POLYDL_DECLARE_PATCH_LAUNCHER)
POLYDL_PATCH_BF16_FAMILY(POLYDL_DECLARE_PATCH_BF16_LAUNCHER)

#define POLYDL_VARIANT_ROW(BM, BN, BK, WM, WN)                                                     \
    {BM, BN, BK, WM, WN, (BM / WM) * (BN / WN) * 64, 2 * (BM * (BK + 4) + BK * (BN + 4)) * 4,      \
     sgemm_launch_##BM##x##BN##x##BK##_##WM##x##WN, conv_launch_##BM##x##BN##x##BK##_##WM##x##WN},
const Variant kVariants[] = {POLYDL_TILE_FAMILY(POLYDL_VARIANT_ROW)};
const int kNumVariants = (int)(sizeof(kVariants) / sizeof(kVariants[0]));

#define POLYDL_PATCH_ROW(BM, BN, BK, WM, WN) \
    {BM, BN, WM, WN, (BM / WM) * (BN / WN) * 64, conv_patch_launch_##BM##x##BN##_##WM##x##WN,   \
     conv_patch_class_##BM##x##BN##_##WM##x##WN},
const PatchVariant kPatchVariants[] = {POLYDL_PATCH_FAMILY(POLYDL_PATCH_ROW)};
const int kNumPatchVariants = (int)(sizeof(kPatchVariants) / sizeof(kPatchVariants[0]));

#define POLYDL_PATCH_BF16_ROW(BM, BN, BK, WM, WN) \
    {BM, BN, WM, WN, (BM / WM) * (BN / WN) * 64, conv_patch_bf16_launch_##BM##x##BN##_##WM##x##WN, nullptr},
const PatchVariant kPatchBf16Variants[] = {POLYDL_PATCH_BF16_FAMILY(POLYDL_PATCH_BF16_ROW)};
const int kNumPatchBf16Variants = (int)(sizeof(kPatchBf16Variants) / sizeof(kPatchBf16Variants[0]));

static std::mutex g_mu;
static std::atomic<int> g_last_hip_error{0};
static int launch_failed(hipError_t e)
{
    // a launch that needed scratch memory it may not have: not the runtime's refusal
    const int why = scratch_refusal();
    if (e == hipErrorOutOfMemory && why == SCRATCH_TOO_SMALL) return POLYDL_ERR_SCRATCH_LIMIT;
    if (e == hipErrorStreamCaptureUnsupported && why == SCRATCH_CAPTURING) return POLYDL_ERR_UNSUPPORTED;
    g_last_hip_error = (int)e;
    return POLYDL_ERR_LAUNCH;
}
static int launched(hipError_t e) { return e == hipSuccess ? POLYDL_OK : launch_failed(e); }

// The kernels are gfx950 code: any other current device (or none) is refused.  Asked once per device.
static bool on_gfx950()
{
    static std::mutex mu;
    static std::map<int, bool> known;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    std::lock_guard<std::mutex> lk(mu);
    auto it = known.find(dev);
    if (it != known.end()) return it->second;
    hipDeviceProp_t prop;
    bool ok = false;
    if (hipGetDeviceProperties(&prop, dev) == hipSuccess) ok = std::strncmp(prop.gcnArchName, "gfx950", 6) == 0;
    else (void)hipGetLastError();
    known[dev] = ok;
    return ok;
}
static bool g_have_override = false;
static polydl_tile_cfg g_override;
static polydl_tile_cfg g_last = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
// picks already made, keyed by the problem's dimensions (the ranking depends on nothing else)
static std::map<std::array<int, 10>, polydl_tile_cfg> g_conv_plans;   // shape, and whether the input is activated on the way in
static std::map<std::array<int, 3>, polydl_tile_cfg> g_sgemm_plans;
static std::map<std::array<int, 9>, polydl_tile_cfg> g_bf16_plans;

static const Variant *find_variant(const polydl_tile_cfg &c)
{
    for (int i = 0; i < kNumVariants; ++i) {
        const Variant &v = kVariants[i];
        if (v.bm == c.bm && v.bn == c.bn && v.bk == c.bk && v.wm == c.wm && v.wn == c.wn) return &v;
    }
    return nullptr;
}

static const PatchVariant *find_patch_bf16_variant(const polydl_tile_cfg &c)
{
    for (int i = 0; i < kNumPatchBf16Variants; ++i) {
        const PatchVariant &v = kPatchBf16Variants[i];
        if (v.bm == c.bm && v.bn == c.bn && v.wm == c.wm && v.wn == c.wn) return &v;
    }
    return nullptr;
}

static const PatchVariant *find_patch_variant(const polydl_tile_cfg &c)
{
    for (int i = 0; i < kNumPatchVariants; ++i) {
        const PatchVariant &v = kPatchVariants[i];
        if (v.bm == c.bm && v.bn == c.bn && v.wm == c.wm && v.wn == c.wn) return &v;
    }
    return nullptr;
}

static void cfg_of(const Variant &v, int split_k, int layout, int raster, polydl_tile_cfg *c)
{
    c->bm = v.bm; c->bn = v.bn; c->bk = v.bk; c->wm = v.wm; c->wn = v.wn;
    c->split_k = split_k; c->layout = layout; c->raster = raster;
    c->algo = 0; c->cb = 0;
}

static void cfg_of_patch(const PatchVariant &v, int cb, int raster, polydl_tile_cfg *c)
{
    c->bm = v.bm; c->bn = v.bn; c->bk = 0; c->wm = v.wm; c->wn = v.wn;
    c->split_k = 1; c->layout = 0; c->raster = raster;
    c->algo = 1; c->cb = cb;
}

// Largest even channel count per stage the patch kernel can hold for this problem and tile,
// preferring stages of at most 72 reduction elements; 0 if none fits.  Used when an override
// names a patch tile but leaves cb = 0.
static int choose_cb(const PatchVariant &v, const ConvProblem &q)
{
    int cpad = (q.C + 1) & ~1;
    int best = 0;
    for (int cb = 2; cb <= cpad && cb <= 64; cb += 2) {
        if (cpad % cb != 0 && cb != cpad) continue;
        if (cb * q.R * q.S > 72 && best != 0) break;
        if (v.conv(q, cb, 1, 0, nullptr, true) == hipSuccess) best = cb;
    }
    return best;
}

static bool conv_dims(int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int64_t *P, int64_t *Q)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0) return false;
    if (H + 2 * (int64_t)pad < R || W + 2 * (int64_t)pad < S) return false;
    *P = (H + 2 * (int64_t)pad - R) / stride + 1;
    *Q = (W + 2 * (int64_t)pad - S) / stride + 1;
    return *P > 0 && *Q > 0;
}

// index ranges of the kernels: filter taps as bit masks, 32-bit pixel counts and offsets, exact
// magic division of reduction indices
static bool conv_in_range(int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int64_t P, int64_t Q)
{
    const int64_t Kg = (int64_t)C * R * S, Ng = (int64_t)N * P * Q;
    if (R > 32 || S > 32 || pad > 0x3FFFFF || stride > 0x3FFFFF) return false;
    if (Ng >= 0x7FFF0000ll || Kg >= (1ll << 22) || Kg * R * S >= (1ll << 32)) return false;
    if ((int64_t)N * C * H * W >= (1ll << 40) || (int64_t)N * K * P * Q >= (1ll << 40)) return false;
    return true;
}

static int sgemm_impl(int M, int N, int K, float alpha, const float *A, const float *B, float beta, float *C,
                      void *stream)
{
    if (M <= 0 || N <= 0 || K < 0) return POLYDL_ERR_BAD_DIMENSION;
    if (!C || (K > 0 && (!A || !B))) return POLYDL_ERR_NULL_POINTER;
    if (K == 0 && beta == 1.f) return POLYDL_OK;
    if (!on_gfx950()) return POLYDL_ERR_NO_DEVICE;
    polydl_tile_cfg cfg;
    if (K == 0) {
        // an empty product: only C = beta*C is left, any variant's epilogue does it
        cfg_of(kVariants[0], 1, 0, 0, &cfg);
    } else {
        std::lock_guard<std::mutex> lk(g_mu);
        cfg = g_override;
        if (!g_have_override) {
            const std::array<int, 3> key = {M, N, K};
            auto it = g_sgemm_plans.find(key);
            if (it != g_sgemm_plans.end()) {
                cfg = it->second;
            } else {
                polydl_model_report rep;
                SgemmProblem pq{M, N, K, A, B, C};
                if (!pick_sgemm(pq, &cfg, &rep)) return POLYDL_ERR_UNSUPPORTED;
                g_sgemm_plans[key] = cfg;
            }
        }
    }
    const Variant *v = find_variant(cfg);
    if (!v) return POLYDL_ERR_UNSUPPORTED;
    // 32-bit byte offsets inside one workgroup's slice of A (bm rows) and of B (bk rows)
    if ((uint64_t)v->bm * (uint64_t)K * 4 >= 0x7FFFFFF0ull) return POLYDL_ERR_UNSUPPORTED;
    if ((uint64_t)v->bk * (uint64_t)N * 4 >= 0x7FFFFFF0ull) return POLYDL_ERR_UNSUPPORTED;
    if ((uint64_t)v->bm * (uint64_t)N * 4 >= 0x7FFFFFF0ull) return POLYDL_ERR_UNSUPPORTED;   // and of C (bm rows)
    uint64_t tiles = (uint64_t)((M + v->bm - 1) / v->bm) * (uint64_t)((N + v->bn - 1) / v->bn);
    if (tiles >= 0x7FFFFFFFull || cfg.split_k > 65535 || cfg.raster >= 2) return POLYDL_ERR_UNSUPPORTED;
    SgemmProblem q{M, N, K, A, B, C, alpha, beta};
    hipError_t e = v->sgemm(q, cfg.split_k < 1 ? 1 : cfg.split_k, cfg.raster, (hipStream_t)stream);
    if (e != hipSuccess) return launch_failed(e);
    std::lock_guard<std::mutex> lk(g_mu);
    g_last = cfg;
    return POLYDL_OK;
}

static int conv_impl(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                     const float *in, const float *wt, const float *bias, float *out, int pre_act, int act,
                     void *stream, const ScratchArena *arena = nullptr, const float *wt_tap = nullptr)
{
    if (pre_act != POLYDL_ACT_NONE && pre_act != POLYDL_ACT_RELU && pre_act != POLYDL_ACT_RELU6)
        return POLYDL_ERR_UNSUPPORTED;
    int64_t P, Q;
    if (!conv_dims(N, C, H, W, K, R, S, stride, pad, &P, &Q)) return POLYDL_ERR_BAD_DIMENSION;
    if (!in || !wt || !out) return POLYDL_ERR_NULL_POINTER;
    if (act != POLYDL_ACT_NONE && act != POLYDL_ACT_RELU && act != POLYDL_ACT_RELU6)
        return POLYDL_ERR_UNSUPPORTED;
    if (!conv_in_range(N, C, H, W, K, R, S, stride, pad, P, Q)) return POLYDL_ERR_UNSUPPORTED;
    if (!on_gfx950()) return POLYDL_ERR_NO_DEVICE;
    const int64_t Kg = (int64_t)C * R * S, CHW = (int64_t)C * H * W;
    ConvProblem q{N, C, H, W, K, R, S, stride, pad, (int)P, (int)Q, in, wt, bias, out, act, pre_act, arena};
    // a filter copy aligned to less than 16 bytes is ignored: every kernel then reads wt
    q.has_tap = wt_tap && !((uintptr_t)wt_tap & 15);
    polydl_tile_cfg cfg;
    bool forced;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        forced = g_have_override;
        cfg = g_override;
    }
    if (!forced) {
        const std::array<int, 10> key = {N, C, H, W, K, R, S, stride, pad,
                                         (pre_act != POLYDL_ACT_NONE ? 1 : 0) | (q.has_tap ? 2 : 0)};
        std::lock_guard<std::mutex> lk(g_mu);
        auto it = g_conv_plans.find(key);
        if (it != g_conv_plans.end()) {
            cfg = it->second;
        } else {
            polydl_model_report rep;
            if (!pick_conv(q, &cfg, &rep)) return POLYDL_ERR_UNSUPPORTED;
            g_conv_plans[key] = cfg;
        }
    }
    const bool point_aligned = !(((uintptr_t)in | (uintptr_t)out) & 7) && !((uintptr_t)wt & 15) && !((uintptr_t)bias & 15);
    if (!forced && cfg.algo == 2 && !point_aligned) {
        // the pointwise kernel moves pixel pairs as 8-byte words and filter and bias as 16-byte
        // words: for tensors aligned to less take the best of the other candidates (not cached:
        // the plan is about shapes)
        std::vector<ConvCandidate> cands;
        conv_candidates(q, &cands);
        const ConvCandidate *b = nullptr;
        for (const ConvCandidate &c : cands)
            if (c.cfg.algo != 2 && (!b || c.rep.predicted_us < b->rep.predicted_us)) b = &c;
        if (!b) return POLYDL_ERR_UNSUPPORTED;
        cfg = b->cfg;
    }
    if (cfg.layout != 0 && !(cfg.layout == 2 && cfg.algo == 0)) return POLYDL_ERR_UNSUPPORTED;
    if (cfg.algo == 2) {
        if (!is_conv_point_cfg(cfg) || !conv_point_fits(q) || !point_aligned) return POLYDL_ERR_UNSUPPORTED;
        hipError_t pe = conv_point_launch(q, (hipStream_t)stream);
        if (pe != hipSuccess) return launch_failed(pe);
        std::lock_guard<std::mutex> lk(g_mu);
        g_last = cfg;
        return POLYDL_OK;
    }
    if (cfg.algo == 1) {
        if (pre_act != POLYDL_ACT_NONE) return POLYDL_ERR_UNSUPPORTED;   // a forced patch-kernel variant
        const PatchVariant *pv = find_patch_variant(cfg);
        if (!pv) return POLYDL_ERR_UNSUPPORTED;
        if (cfg.cb == 0) cfg.cb = choose_cb(*pv, q);
        if (cfg.cb < 2 || (cfg.cb & 1)) return POLYDL_ERR_UNSUPPORTED;
        const int sk = cfg.split_k < 1 ? 1 : cfg.split_k;
        if (pv->conv(q, cfg.cb, sk, cfg.raster, nullptr, true) != hipSuccess) return POLYDL_ERR_UNSUPPORTED;
        hipError_t pe = pv->conv(q, cfg.cb, sk, cfg.raster, (hipStream_t)stream, false);
        if (pe != hipSuccess) return launch_failed(pe);
        std::lock_guard<std::mutex> lk(g_mu);
        g_last = cfg;
        return POLYDL_OK;
    }
    const Variant *v = find_variant(cfg);
    if (!v) return POLYDL_ERR_UNSUPPORTED;
    // a tile of bn pixels spans at most bn/PQ + 2 images; their offsets must fit 31 bits
    const int64_t span = (v->bn / (P * Q) + 2) * CHW * 4;
    const int64_t span_out = (v->bn / (P * Q) + 2) * (int64_t)K * P * Q * 4;
    if (span >= 0x7FFFFFF0ll || span_out >= 0x7FFFFFF0ll || (int64_t)v->bm * Kg * 4 >= 0x7FFFFFF0ll)
        return POLYDL_ERR_UNSUPPORTED;
    if (cfg.layout == 2) {
        if (!q.has_tap || !gather_tap_major_fits(q, v->bk)) return POLYDL_ERR_UNSUPPORTED;
        q.wt_tap = wt_tap;
    }
    hipError_t e = v->conv(q, cfg.split_k < 1 ? 1 : cfg.split_k, cfg.raster, (hipStream_t)stream);
    if (e != hipSuccess) return launch_failed(e);
    std::lock_guard<std::mutex> lk(g_mu);
    g_last = cfg;
    return POLYDL_OK;
}

}  // namespace polydl

using namespace polydl;

extern "C" {

int polydl_conv2d_fwd(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                      const float *in, const float *wt, const float *bias, float *out,
                      int fuse_relu, void *stream)
{
    return conv_impl(N, C, H, W, K, R, S, stride, pad, in, wt, bias, out, POLYDL_ACT_NONE,
                     fuse_relu ? POLYDL_ACT_RELU : POLYDL_ACT_NONE, stream);
}

int polydl_conv2d_fwd_act(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                          const float *in, const float *wt, const float *bias, float *out, int act,
                          void *stream)
{
    return conv_impl(N, C, H, W, K, R, S, stride, pad, in, wt, bias, out, POLYDL_ACT_NONE, act, stream);
}

int polydl_conv2d_fwd_pre_act(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                              const float *in, const float *wt, const float *bias, float *out, int pre_act,
                              int act, void *stream)
{
    return conv_impl(N, C, H, W, K, R, S, stride, pad, in, wt, bias, out, pre_act, act, stream);
}

int polydl_conv2d_fwd_noalloc(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                              const float *in, const float *wt, const float *bias, float *out, int act,
                              void *stream)
{
    ScratchArena arena;
    const hipError_t e = static_scratch_arena(&arena);
    if (e != hipSuccess) {
        g_last_hip_error = (int)e;
        return POLYDL_ERR_LAUNCH;
    }
    return conv_impl(N, C, H, W, K, R, S, stride, pad, in, wt, bias, out, POLYDL_ACT_NONE, act, stream, &arena);
}

int polydl_conv2d_fwd_tap(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                          const float *in, const float *wt, const float *wt_tap, const float *bias, float *out,
                          int act, void *stream)
{
    return conv_impl(N, C, H, W, K, R, S, stride, pad, in, wt, bias, out, POLYDL_ACT_NONE, act, stream, nullptr,
                     wt_tap);
}

int polydl_sgemm(int M, int N, int K, const float *A, const float *B, float *C, void *stream)
{
    return sgemm_impl(M, N, K, 1.f, A, B, 1.f, C, stream);
}

int polydl_sgemm_ex(int M, int N, int K, float alpha, const float *A, const float *B, float beta, float *C,
                    void *stream)
{
    return sgemm_impl(M, N, K, alpha, A, B, beta, C, stream);
}

int polydl_nchw_to_nchwc(int N, int C, int H, int W, int b, const float *in, float *out, void *stream)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || b <= 0) return POLYDL_ERR_BAD_DIMENSION;
    if (!in || !out) return POLYDL_ERR_NULL_POINTER;
    if (b > 32 || N > 65535 || (C + b - 1) / b > 65535 || (int64_t)H * W >= (1ll << 31)) return POLYDL_ERR_UNSUPPORTED;
    if (!on_gfx950()) return POLYDL_ERR_NO_DEVICE;
    return launched(launch_nchwc(in, out, N, C, H * W, b, true, 4, (hipStream_t)stream));
}

int polydl_nchwc_to_nchw(int N, int C, int H, int W, int b, const float *in, float *out, void *stream)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || b <= 0) return POLYDL_ERR_BAD_DIMENSION;
    if (!in || !out) return POLYDL_ERR_NULL_POINTER;
    if (b > 32 || N > 65535 || (C + b - 1) / b > 65535 || (int64_t)H * W >= (1ll << 31)) return POLYDL_ERR_UNSUPPORTED;
    if (!on_gfx950()) return POLYDL_ERR_NO_DEVICE;
    return launched(launch_nchwc(in, out, N, C, H * W, b, false, 4, (hipStream_t)stream));
}

int polydl_kcrs_to_kcrsck(int K, int C, int R, int S, int bc, int bk, const float *wt, float *out, void *stream)
{
    if (K <= 0 || C <= 0 || R <= 0 || S <= 0 || bc <= 0 || bk <= 0) return POLYDL_ERR_BAD_DIMENSION;
    if (!wt || !out) return POLYDL_ERR_NULL_POINTER;
    const int64_t total = (int64_t)((K + bk - 1) / bk) * bk * ((C + bc - 1) / bc) * bc * R * S;
    if (total >= (1ll << 39) || (int64_t)R * S >= (1ll << 31)) return POLYDL_ERR_UNSUPPORTED;
    if (!on_gfx950()) return POLYDL_ERR_NO_DEVICE;
    return launched(launch_kcrsck(wt, out, K, C, R * S, bc, bk, 4, (hipStream_t)stream));
}

int polydl_nchw_to_nchwc_bf16(int N, int C, int H, int W, int b, const uint16_t *in, uint16_t *out, void *stream)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || b <= 0) return POLYDL_ERR_BAD_DIMENSION;
    if (!in || !out) return POLYDL_ERR_NULL_POINTER;
    if (b > 32 || N > 65535 || (C + b - 1) / b > 65535 || (int64_t)H * W >= (1ll << 31)) return POLYDL_ERR_UNSUPPORTED;
    if (!on_gfx950()) return POLYDL_ERR_NO_DEVICE;
    return launched(launch_nchwc(in, out, N, C, H * W, b, true, 2, (hipStream_t)stream));
}

int polydl_kcrs_to_kcrsck_bf16(int K, int C, int R, int S, int bc, int bk, const uint16_t *wt, uint16_t *out,
                               void *stream)
{
    if (K <= 0 || C <= 0 || R <= 0 || S <= 0 || bc <= 0 || bk <= 0) return POLYDL_ERR_BAD_DIMENSION;
    if (!wt || !out) return POLYDL_ERR_NULL_POINTER;
    const int64_t total = (int64_t)((K + bk - 1) / bk) * bk * ((C + bc - 1) / bc) * bc * R * S;
    if (total >= (1ll << 39) || (int64_t)R * S >= (1ll << 31)) return POLYDL_ERR_UNSUPPORTED;
    if (!on_gfx950()) return POLYDL_ERR_NO_DEVICE;
    return launched(launch_kcrsck(wt, out, K, C, R * S, bc, bk, 2, (hipStream_t)stream));
}

// Every (tile, stage depth in eight-channel units, split factor) the bfloat16 picker ranks; qb.C counts units.
static const int kBf16Depths[] = {32, 24, 16, 12, 8, 6, 4, 2};
static void bf16_candidates(const ConvProblem &qb, std::vector<polydl_tile_cfg> *out)
{
    out->clear();
    const int cunits = qb.C;
    const int rows_per_stage = qb.R >= 5 ? 1 : qb.R;
    for (int i = 0; i < kNumPatchBf16Variants; ++i) {
        const PatchVariant &v = kPatchBf16Variants[i];
        // deepest stages first: on equal predictions fewer, longer stages win (fewer barriers)
        for (int cb : kBf16Depths) {
            if (cb > ((cunits + 1) & ~1)) continue;
            if (v.conv(qb, cb, 1, 0, nullptr, true) != hipSuccess) continue;
            const int nstages = (cunits + cb - 1) / cb * (qb.R / rows_per_stage);
            const int splits[] = {1, 2, 3, 4, 6, 8, 12, 16};
            for (int sk : splits) {
                if (sk > nstages) break;
                // raster 1: the workgroups of one XCD take neighbouring tiles, so the tiles that share a
                // pixel run (all filter row blocks of it) fetch it into one L2 instead of eight; on
                // the suite at batch 64 the 64 -> 256 pointwise layer gains 14 %, the others 0-6 %
                out->push_back(polydl_tile_cfg{v.bm, v.bn, 0, v.wm, v.wn, sk, 1, 1, 1, cb});
            }
        }
    }
}

static int bf16_threads(const polydl_tile_cfg &c) { return (c.bm / c.wm) * (c.bn / c.wn) * 64; }

// bf16 candidates are ranked with the round-by-round time model at the bf16 instruction's rate
static bool pick_bf16(const ConvProblem &qb, polydl_tile_cfg *out)
{
    std::vector<polydl_tile_cfg> cands;
    bf16_candidates(qb, &cands);
    bool have = false;
    double best = 0;
    for (const polydl_tile_cfg &c : cands) {
        const double t = model_conv_bf16(qb, c, bf16_threads(c));
        if (!have || t < best * 0.999) { best = t; *out = c; have = true; }
    }
    return have;
}

int polydl_conv2d_fwd_bf16_blocked(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                                   const uint16_t *in8c, const uint16_t *wt8c, const float *bias, float *out,
                                   int act, void *stream)
{
    int64_t P, Q;
    if (!conv_dims(N, C, H, W, K, R, S, stride, pad, &P, &Q)) return POLYDL_ERR_BAD_DIMENSION;
    if (!in8c || !wt8c || !out) return POLYDL_ERR_NULL_POINTER;
    if (act != POLYDL_ACT_NONE && act != POLYDL_ACT_RELU && act != POLYDL_ACT_RELU6) return POLYDL_ERR_UNSUPPORTED;
    if (!conv_in_range(N, C, H, W, K, R, S, stride, pad, P, Q)) return POLYDL_ERR_UNSUPPORTED;
    if (((uintptr_t)in8c & 15) || ((uintptr_t)wt8c & 15)) return POLYDL_ERR_UNSUPPORTED;   // 16-byte units
    if (!on_gfx950()) return POLYDL_ERR_NO_DEVICE;
    const int cunits = (C + 7) / 8;
    ConvProblem q{N, cunits, H, W, K, R, S, stride, pad, (int)P, (int)Q, in8c, wt8c, bias, out, act};
    polydl_tile_cfg cfg;
    bool forced;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        forced = g_have_override;
        cfg = g_override;
    }
    if (forced) {
        if (cfg.algo != 1) return POLYDL_ERR_UNSUPPORTED;
    } else {
        // the pick depends on the shape alone: made once per shape
        const std::array<int, 9> key = {N, cunits, H, W, K, R, S, stride, pad};
        std::lock_guard<std::mutex> lk(g_mu);
        auto it = g_bf16_plans.find(key);
        if (it != g_bf16_plans.end()) {
            cfg = it->second;
        } else {
            if (!pick_bf16(q, &cfg)) return POLYDL_ERR_UNSUPPORTED;
            g_bf16_plans[key] = cfg;
        }
    }
    const PatchVariant *pv = find_patch_bf16_variant(cfg);
    if (!pv) return POLYDL_ERR_UNSUPPORTED;
    if (cfg.cb == 0) {
        for (int cb = 2; cb <= ((cunits + 1) & ~1) && cb <= 32; cb += 2)
            if (pv->conv(q, cb, 1, 0, nullptr, true) == hipSuccess) cfg.cb = cb;
    }
    if (cfg.cb < 2 || (cfg.cb & 1)) return POLYDL_ERR_UNSUPPORTED;
    const int sk = cfg.split_k < 1 ? 1 : cfg.split_k;
    if (pv->conv(q, cfg.cb, sk, cfg.raster, nullptr, true) != hipSuccess) return POLYDL_ERR_UNSUPPORTED;
    hipError_t e = pv->conv(q, cfg.cb, sk, cfg.raster, (hipStream_t)stream, false);
    if (e != hipSuccess) return launch_failed(e);
    cfg.layout = 1;
    std::lock_guard<std::mutex> lk(g_mu);
    g_last = cfg;
    return POLYDL_OK;
}

size_t polydl_conv2d_bf16_workspace_bytes(int N, int C, int H, int W, int K, int R, int S)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0 || R <= 0 || S <= 0) return 0;
    const size_t cu = ((size_t)C + 7) / 8;
    const size_t in_b = ((size_t)N * cu * H * W * 16 + 255) / 256 * 256;
    return in_b + (size_t)K * cu * R * S * 16;
}

int polydl_conv2d_fwd_bf16(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                           const uint16_t *in, const uint16_t *wt, const float *bias, float *out, int act,
                           void *workspace, size_t workspace_bytes, void *stream)
{
    int64_t P, Q;
    if (!conv_dims(N, C, H, W, K, R, S, stride, pad, &P, &Q)) return POLYDL_ERR_BAD_DIMENSION;
    if (!in || !wt || !out || !workspace) return POLYDL_ERR_NULL_POINTER;
    if (workspace_bytes < polydl_conv2d_bf16_workspace_bytes(N, C, H, W, K, R, S) || ((uintptr_t)workspace & 255))
        return POLYDL_ERR_UNSUPPORTED;
    const size_t cu = ((size_t)C + 7) / 8;
    uint16_t *in8c = static_cast<uint16_t *>(workspace);
    uint16_t *wt8c = reinterpret_cast<uint16_t *>(static_cast<char *>(workspace) +
                                                  ((size_t)N * cu * H * W * 16 + 255) / 256 * 256);
    int st = polydl_nchw_to_nchwc_bf16(N, C, H, W, 8, in, in8c, stream);
    if (st != POLYDL_OK) return st;
    st = polydl_kcrs_to_kcrsck_bf16(K, C, R, S, 8, 1, wt, wt8c, stream);
    if (st != POLYDL_OK) return st;
    return polydl_conv2d_fwd_bf16_blocked(N, C, H, W, K, R, S, stride, pad, in8c, wt8c, bias, out, act, stream);
}

int polydl_bias_add(int N, int K, int P, int Q, float *y, const float *bias, void *stream)
{
    if (N <= 0 || K <= 0 || P <= 0 || Q <= 0) return POLYDL_ERR_BAD_DIMENSION;
    if (!y || !bias) return POLYDL_ERR_NULL_POINTER;
    if ((int64_t)P * Q >= (1ll << 31)) return POLYDL_ERR_UNSUPPORTED;
    if (!on_gfx950()) return POLYDL_ERR_NO_DEVICE;
    return launched(launch_bias_add(y, bias, K, P * Q, (size_t)N * K * P * Q, (hipStream_t)stream));
}

int polydl_bnorm_fwd(int N, int K, int P, int Q, const float *x, const float *gamma, const float *beta,
                     const float *mean, const float *var, float eps, float *y, int act, void *stream)
{
    if (N <= 0 || K <= 0 || P <= 0 || Q <= 0) return POLYDL_ERR_BAD_DIMENSION;
    if (!x || !y || !gamma || !beta || !mean || !var) return POLYDL_ERR_NULL_POINTER;
    if (act < POLYDL_ACT_NONE || act > POLYDL_ACT_RELU6 || !(eps >= 0.f)) return POLYDL_ERR_UNSUPPORTED;
    // element indices are 31-bit in the kernel
    if ((int64_t)N * K * P * Q >= (1ll << 31)) return POLYDL_ERR_UNSUPPORTED;
    if (!on_gfx950()) return POLYDL_ERR_NO_DEVICE;
    return launched(launch_bnorm_act(x, y, gamma, beta, mean, var, eps, K, P * Q, (size_t)N * K * P * Q, act,
                                     (hipStream_t)stream));
}

int polydl_activation(int64_t count, float *y, int act, void *stream)
{
    if (count <= 0) return POLYDL_ERR_BAD_DIMENSION;
    if (!y) return POLYDL_ERR_NULL_POINTER;
    if (act != POLYDL_ACT_RELU && act != POLYDL_ACT_RELU6) return POLYDL_ERR_UNSUPPORTED;
    if (!on_gfx950()) return POLYDL_ERR_NO_DEVICE;
    return launched(launch_act(y, (size_t)count, act, (hipStream_t)stream));
}

int polydl_reuse_analyse(int nloops, const int *extents, const int *parallel, int nrefs, const polydl_loop_ref *refs,
                         int max_deps, polydl_reuse_dep *deps, int *ndeps)
{
    if (!extents || !refs || !ndeps || (max_deps > 0 && !deps)) return POLYDL_ERR_NULL_POINTER;
    if (nloops < 1 || nloops > POLYDL_REUSE_MAX_LOOPS || nrefs < 1 || nrefs > 16 || max_deps < 0)
        return POLYDL_ERR_BAD_DIMENSION;
    int64_t count = 1;
    for (int l = 0; l < nloops; ++l) {
        if (extents[l] < 1) return POLYDL_ERR_BAD_DIMENSION;
        count *= extents[l];
        if (count > POLYDL_REUSE_MAX_ITERATIONS) return POLYDL_ERR_BAD_DIMENSION;
    }
    for (int r = 0; r < nrefs; ++r) {
        if (refs[r].rank < 1 || refs[r].rank > 4) return POLYDL_ERR_BAD_DIMENSION;
        for (int d = 0; d < refs[r].rank; ++d) {
            // subscripts must stay well inside int
            int64_t reach = refs[r].offset[d] < 0 ? -(int64_t)refs[r].offset[d] : refs[r].offset[d];
            for (int l = 0; l < nloops; ++l) {
                const int64_t c = refs[r].coef[d][l] < 0 ? -(int64_t)refs[r].coef[d][l] : refs[r].coef[d][l];
                reach += c * extents[l];
            }
            if (reach > 0x3FFFFFFF) return POLYDL_ERR_BAD_DIMENSION;
        }
    }
    return reuse_analyse(nloops, extents, parallel, nrefs, refs, max_deps, deps, ndeps);
}

int polydl_reuse_bucket(int n, const double *ws, int nlevels, const double *sizes, double *levels, double *mem)
{
    if (n < 0 || nlevels < 0) return POLYDL_ERR_BAD_DIMENSION;
    if ((n > 0 && !ws) || (nlevels > 0 && (!sizes || !levels)) || !mem) return POLYDL_ERR_NULL_POINTER;
    reuse_bucket(n, ws, nlevels, sizes, levels, mem);
    return POLYDL_OK;
}

double polydl_reuse_cost(int nlevels, const double *levels, double mem, const double *weights, double mem_weight)
{
    if (nlevels < 0 || (nlevels > 0 && (!levels || !weights))) return -1.0;
    return reuse_cost(nlevels, levels, mem, weights, mem_weight);
}

static int threads_of(const polydl_tile_cfg &c)
{
    if (c.wm <= 0 || c.wn <= 0 || c.bm % c.wm || c.bn % c.wn) return 0;
    return (c.bm / c.wm) * (c.bn / c.wn) * 64;
}

int polydl_model_get_levels(double *capacity_bytes, double *gbytes_per_s, double *mem_gbytes_per_s)
{
    if (!capacity_bytes || !gbytes_per_s || !mem_gbytes_per_s) return POLYDL_ERR_NULL_POINTER;
    model_get_levels(capacity_bytes, gbytes_per_s, mem_gbytes_per_s);
    return POLYDL_OK;
}

int polydl_model_set_levels(const double *capacity_bytes, const double *gbytes_per_s, double mem_gbytes_per_s)
{
    if (!capacity_bytes || !gbytes_per_s) return POLYDL_ERR_NULL_POINTER;
    if (!(mem_gbytes_per_s > 0)) return POLYDL_ERR_BAD_DIMENSION;
    for (int i = 0; i < 4; ++i)
        if (!(capacity_bytes[i] > 0) || !(gbytes_per_s[i] > 0) || (i > 0 && !(capacity_bytes[i] >= capacity_bytes[i - 1])))
            return POLYDL_ERR_BAD_DIMENSION;
    std::lock_guard<std::mutex> lk(g_mu);
    model_set_levels(capacity_bytes, gbytes_per_s, mem_gbytes_per_s);
    g_conv_plans.clear();      // picks made with the old table
    g_sgemm_plans.clear();
    g_bf16_plans.clear();
    return POLYDL_OK;
}

int polydl_model_conv2d(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                        const polydl_tile_cfg *cfg, polydl_model_report *report)
{
    int64_t P, Q;
    if (!conv_dims(N, C, H, W, K, R, S, stride, pad, &P, &Q)) return POLYDL_ERR_BAD_DIMENSION;
    if (!cfg || !report) return POLYDL_ERR_NULL_POINTER;
    const bool known = cfg->algo == 2 ? is_conv_point_cfg(*cfg)
                                      : (cfg->algo == 1 ? find_patch_variant(*cfg) != nullptr
                                                        : (cfg->algo == 0 && find_variant(*cfg) != nullptr));
    if (!known || !conv_in_range(N, C, H, W, K, R, S, stride, pad, P, Q)) return POLYDL_ERR_UNSUPPORTED;
    ConvProblem q{N, C, H, W, K, R, S, stride, pad, (int)P, (int)Q, nullptr, nullptr, nullptr, nullptr, 0};
    if (cfg->algo == 2) {
        if (!conv_point_fits(q)) return POLYDL_ERR_UNSUPPORTED;
        model_conv_point(q, report);
        return POLYDL_OK;
    }
    int rc = 0;
    if (cfg->algo == 1) rc = find_patch_variant(*cfg)->reg_class(q, cfg->cb < 2 ? 2 : cfg->cb);
    if (rc < 0) return POLYDL_ERR_UNSUPPORTED;   // a stage of this depth does not fit the kernel's LDS or registers
    model_conv(q, *cfg, threads_of(*cfg), rc, report);
    return POLYDL_OK;
}

int polydl_model_sgemm(int M, int N, int K, const polydl_tile_cfg *cfg, polydl_model_report *report)
{
    if (M <= 0 || N <= 0 || K <= 0) return POLYDL_ERR_BAD_DIMENSION;
    if (!cfg || !report) return POLYDL_ERR_NULL_POINTER;
    if (!find_variant(*cfg)) return POLYDL_ERR_UNSUPPORTED;
    SgemmProblem q{M, N, K, nullptr, nullptr, nullptr};
    model_sgemm(q, *cfg, threads_of(*cfg), report);
    return POLYDL_OK;
}

int polydl_pick_conv2d(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                       polydl_tile_cfg *cfg, polydl_model_report *report)
{
    int64_t P, Q;
    if (!conv_dims(N, C, H, W, K, R, S, stride, pad, &P, &Q)) return POLYDL_ERR_BAD_DIMENSION;
    if (!cfg) return POLYDL_ERR_NULL_POINTER;
    if (!conv_in_range(N, C, H, W, K, R, S, stride, pad, P, Q)) return POLYDL_ERR_UNSUPPORTED;
    ConvProblem q{N, C, H, W, K, R, S, stride, pad, (int)P, (int)Q, nullptr, nullptr, nullptr, nullptr, 0};
    polydl_model_report rep;
    if (!pick_conv(q, cfg, &rep)) return POLYDL_ERR_UNSUPPORTED;
    if (report) *report = rep;
    return POLYDL_OK;
}

int polydl_ranker_num_params(void) { return ranker_num_params(); }

int polydl_ranker_set_params(const double *params, int count)
{
    if (!params) return POLYDL_ERR_NULL_POINTER;
    if (count != ranker_num_params()) return POLYDL_ERR_BAD_DIMENSION;
    for (int i = 0; i < count; ++i)
        if (!(params[i] == params[i]) || params[i] > 1e300 || params[i] < -1e300) return POLYDL_ERR_BAD_DIMENSION;
    ranker_set_params(params);
    return POLYDL_OK;
}

int polydl_ranker_stats_conv2d(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                               const polydl_tile_cfg *cfg, double *stats)
{
    if (!stats) return POLYDL_ERR_NULL_POINTER;
    polydl_model_report rep;
    const int rc = polydl_model_conv2d(N, C, H, W, K, R, S, stride, pad, cfg, &rep);
    if (rc != POLYDL_OK) return rc;
    ranker_stats(rep, stats);
    return POLYDL_OK;
}

static bool stats_ok(const double *stats, int64_t count)
{
    for (int64_t i = 0; i < count; ++i)
        if (!(stats[i] >= 0) || stats[i] > 1e300) return false;   // also rejects NaN
    return true;
}

int polydl_ranker_play(const double *stats1, const double *stats2, double theta, double *probs, int *winner)
{
    if (!stats1 || !stats2) return POLYDL_ERR_NULL_POINTER;
    if (!stats_ok(stats1, POLYDL_RANKER_STATS) || !stats_ok(stats2, POLYDL_RANKER_STATS) || !(theta >= 0 && theta <= 1))
        return POLYDL_ERR_BAD_DIMENSION;
    return ranker_play(stats1, stats2, theta, probs, winner) ? POLYDL_OK : POLYDL_ERR_UNSUPPORTED;
}

int polydl_ranker_tournament(int n, const double *stats, double theta, int *wins, int *order)
{
    if (n < 0 || n > 1024) return POLYDL_ERR_BAD_DIMENSION;   // n*(n-1) games of about 4000 multiply-adds each
    if (n > 0 && !stats) return POLYDL_ERR_NULL_POINTER;
    if (!stats_ok(stats, (int64_t)n * POLYDL_RANKER_STATS) || !(theta >= 0 && theta <= 1)) return POLYDL_ERR_BAD_DIMENSION;
    return ranker_tournament(n, stats, theta, wins, order) ? POLYDL_OK : POLYDL_ERR_UNSUPPORTED;
}

int polydl_pick_conv2d_learned(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                               double theta, polydl_tile_cfg *cfg, polydl_model_report *report, int *wins,
                               int *games)
{
    int64_t P, Q;
    if (!conv_dims(N, C, H, W, K, R, S, stride, pad, &P, &Q)) return POLYDL_ERR_BAD_DIMENSION;
    if (!cfg) return POLYDL_ERR_NULL_POINTER;
    if (!(theta >= 0 && theta <= 1)) return POLYDL_ERR_BAD_DIMENSION;
    if (!conv_in_range(N, C, H, W, K, R, S, stride, pad, P, Q) || !ranker_ready()) return POLYDL_ERR_UNSUPPORTED;
    ConvProblem q{N, C, H, W, K, R, S, stride, pad, (int)P, (int)Q, nullptr, nullptr, nullptr, nullptr, 0};
    std::vector<ConvCandidate> cands;
    conv_candidates(q, &cands);
    if (cands.empty()) return POLYDL_ERR_UNSUPPORTED;
    const int n = (int)cands.size();
    std::vector<double> stats((size_t)n * POLYDL_RANKER_STATS);
    for (int i = 0; i < n; ++i) ranker_stats(cands[i].rep, &stats[(size_t)i * POLYDL_RANKER_STATS]);
    std::vector<int> w(n), order(n);
    if (!ranker_tournament(n, stats.data(), theta, w.data(), order.data())) return POLYDL_ERR_UNSUPPORTED;
    *cfg = cands[order[0]].cfg;
    if (report) *report = cands[order[0]].rep;
    if (wins) *wins = w[order[0]];
    if (games) *games = 2 * (n - 1);
    return POLYDL_OK;
}

// C is the channel count of the bfloat16 tensors; the kernels see blocks of eight channels.
static bool bf16_problem(int N, int C, int H, int W, int K, int R, int S, int stride, int pad, ConvProblem *q, int *status)
{
    int64_t P, Q;
    if (!conv_dims(N, C, H, W, K, R, S, stride, pad, &P, &Q)) { *status = POLYDL_ERR_BAD_DIMENSION; return false; }
    if (!conv_in_range(N, C, H, W, K, R, S, stride, pad, P, Q)) { *status = POLYDL_ERR_UNSUPPORTED; return false; }
    *q = ConvProblem{N, (C + 7) / 8, H, W, K, R, S, stride, pad, (int)P, (int)Q, nullptr, nullptr, nullptr, nullptr, 0};
    return true;
}

int polydl_model_conv2d_bf16(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                             const polydl_tile_cfg *cfg, double *predicted_us)
{
    ConvProblem q;
    int st = POLYDL_OK;
    if (!bf16_problem(N, C, H, W, K, R, S, stride, pad, &q, &st)) return st;
    if (!cfg || !predicted_us) return POLYDL_ERR_NULL_POINTER;
    for (int i = 0; i < kNumPatchBf16Variants; ++i) {
        const PatchVariant &v = kPatchBf16Variants[i];
        if (v.bm != cfg->bm || v.bn != cfg->bn || v.wm != cfg->wm || v.wn != cfg->wn) continue;
        if (cfg->cb < 2 || (cfg->cb & 1) || cfg->split_k < 1) return POLYDL_ERR_UNSUPPORTED;
        if (v.conv(q, cfg->cb, cfg->split_k, 0, nullptr, true) != hipSuccess) return POLYDL_ERR_UNSUPPORTED;
        *predicted_us = model_conv_bf16(q, *cfg, v.threads);
        return POLYDL_OK;
    }
    return POLYDL_ERR_UNSUPPORTED;
}

int polydl_pick_conv2d_bf16(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                            polydl_tile_cfg *cfg, double *predicted_us)
{
    ConvProblem q;
    int st = POLYDL_OK;
    if (!bf16_problem(N, C, H, W, K, R, S, stride, pad, &q, &st)) return st;
    if (!cfg) return POLYDL_ERR_NULL_POINTER;
    if (!pick_bf16(q, cfg)) return POLYDL_ERR_UNSUPPORTED;
    if (predicted_us) {
        for (int i = 0; i < kNumPatchBf16Variants; ++i) {
            const PatchVariant &v = kPatchBf16Variants[i];
            if (v.bm == cfg->bm && v.bn == cfg->bn && v.wm == cfg->wm && v.wn == cfg->wn)
                *predicted_us = model_conv_bf16(q, *cfg, v.threads);
        }
    }
    return POLYDL_OK;
}

int polydl_pick_sgemm(int M, int N, int K, polydl_tile_cfg *cfg, polydl_model_report *report)
{
    if (M <= 0 || N <= 0 || K <= 0) return POLYDL_ERR_BAD_DIMENSION;
    if (!cfg) return POLYDL_ERR_NULL_POINTER;
    SgemmProblem q{M, N, K, nullptr, nullptr, nullptr};
    polydl_model_report rep;
    if (!pick_sgemm(q, cfg, &rep)) return POLYDL_ERR_UNSUPPORTED;
    if (report) *report = rep;
    return POLYDL_OK;
}

int polydl_conv2d_candidates(int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int kind,
                             int max_cfgs, polydl_tile_cfg *cfgs, int *count)
{
    if (!count || (max_cfgs > 0 && !cfgs)) return POLYDL_ERR_NULL_POINTER;
    if (max_cfgs < 0) return POLYDL_ERR_BAD_DIMENSION;
    std::vector<polydl_tile_cfg> list;
    if (kind == 0 || kind == 3) {
        int64_t P, Q;
        if (!conv_dims(N, C, H, W, K, R, S, stride, pad, &P, &Q)) return POLYDL_ERR_BAD_DIMENSION;
        if (!conv_in_range(N, C, H, W, K, R, S, stride, pad, P, Q)) return POLYDL_ERR_UNSUPPORTED;
        ConvProblem q{N, C, H, W, K, R, S, stride, pad, (int)P, (int)Q, nullptr, nullptr, nullptr, nullptr, 0};
        q.has_tap = kind == 3;
        std::vector<ConvCandidate> cands;
        conv_candidates(q, &cands);
        for (const ConvCandidate &c : cands) list.push_back(c.cfg);
    } else if (kind == 2) {
        ConvProblem q;
        int st = POLYDL_OK;
        if (!bf16_problem(N, C, H, W, K, R, S, stride, pad, &q, &st)) return st;
        bf16_candidates(q, &list);
    } else {
        return POLYDL_ERR_UNSUPPORTED;
    }
    *count = (int)list.size();
    for (int i = 0; i < *count && i < max_cfgs; ++i) cfgs[i] = list[i];
    return POLYDL_OK;
}

int polydl_sgemm_candidates(int M, int N, int K, int max_cfgs, polydl_tile_cfg *cfgs, int *count)
{
    if (!count || (max_cfgs > 0 && !cfgs)) return POLYDL_ERR_NULL_POINTER;
    if (M <= 0 || N <= 0 || K <= 0 || max_cfgs < 0) return POLYDL_ERR_BAD_DIMENSION;
    std::vector<polydl_tile_cfg> list;
    sgemm_candidates(SgemmProblem{M, N, K, nullptr, nullptr, nullptr}, &list);
    *count = (int)list.size();
    for (int i = 0; i < *count && i < max_cfgs; ++i) cfgs[i] = list[i];
    return POLYDL_OK;
}

int polydl_set_tile_override(const polydl_tile_cfg *cfg)
{
    std::lock_guard<std::mutex> lk(g_mu);
    if (!cfg) {
        g_have_override = false;
        return POLYDL_OK;
    }
    const bool known = cfg->algo == 2 ? is_conv_point_cfg(*cfg)
                                      : (cfg->algo == 1 ? (find_patch_variant(*cfg) != nullptr ||
                                                           find_patch_bf16_variant(*cfg) != nullptr)
                                                        : (cfg->algo == 0 && find_variant(*cfg) != nullptr));
    if (!known || cfg->split_k < 1 || cfg->layout < 0 || cfg->layout > 2 || (cfg->layout == 2 && cfg->algo != 0) ||
        cfg->raster < 0 ||
        cfg->raster > 3 || (cfg->raster >= 2 && cfg->algo != 0) || cfg->cb < 0 || (cfg->cb & 1))
        return POLYDL_ERR_UNSUPPORTED;
    g_override = *cfg;
    g_have_override = true;
    return POLYDL_OK;
}

int polydl_get_last_tile(polydl_tile_cfg *cfg)
{
    if (!cfg) return POLYDL_ERR_NULL_POINTER;
    std::lock_guard<std::mutex> lk(g_mu);
    *cfg = g_last;
    return POLYDL_OK;
}

int polydl_num_variants(int kind)
{
    if (kind == 0) return kNumVariants + kNumPatchVariants + 1;   // the last one is the pointwise kernel
    if (kind == 2) return kNumPatchBf16Variants;
    return kind == 1 ? kNumVariants : POLYDL_ERR_UNSUPPORTED;
}

int polydl_get_variant(int kind, int index, polydl_tile_cfg *cfg)
{
    if (!cfg) return POLYDL_ERR_NULL_POINTER;
    if (kind < 0 || kind > 2 || index < 0 || index >= polydl_num_variants(kind)) return POLYDL_ERR_UNSUPPORTED;
    if (kind == 2) {
        cfg_of_patch(kPatchBf16Variants[index], 0, 0, cfg);
        cfg->layout = 1;
    } else if (index < kNumVariants) cfg_of(kVariants[index], 1, 0, 0, cfg);
    else if (index < kNumVariants + kNumPatchVariants) cfg_of_patch(kPatchVariants[index - kNumVariants], 0, 0, cfg);
    else *cfg = conv_point_cfg();
    return POLYDL_OK;
}

int polydl_last_hip_error(void) { return g_last_hip_error.load(); }

const char *polydl_status_string(int status)
{
    switch (status) {
    case POLYDL_OK: return "ok";
    case POLYDL_ERR_NULL_POINTER: return "null pointer";
    case POLYDL_ERR_BAD_DIMENSION: return "bad dimension";
    case POLYDL_ERR_UNSUPPORTED: return "unsupported configuration";
    case POLYDL_ERR_LAUNCH: return "HIP launch failed";
    case POLYDL_ERR_NO_DEVICE: return "the current device is not a gfx950 GPU";
    case POLYDL_ERR_SCRATCH_LIMIT: return "needs more scratch memory than the fixed array holds";
    default: return "unknown status";
    }
}

}  // extern "C"
