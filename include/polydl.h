/*
 * polydl.h -- C ABI of the MI355X (gfx950) convolution / matrix-product library.
 *
 * The library computes the two loop nests PolyDL (arXiv 2006.02230) optimises: the forward 2-D
 * convolution of a CNN layer (figure "The 2-D Convolution code", section "Convolutions") and
 * the matrix multiplication at its core (figure "Matrix multiplication code", section
 * "Notation"; C = beta*C + alpha*A*B in section "GEMM").  Argument names follow the paper's
 * loop bounds: N = nImg, C = nIfm, K = nOfm, H/W = input height/width, R/S = kh/kw,
 * P/Q = ofh/ofw.
 *
 * Conventions common to every entry point
 *   - every data pointer is a DEVICE pointer (HBM), owned by the caller; the library neither
 *     frees nor keeps it after the work it enqueued has run, except where a handle says so;
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream); all work is
 *     enqueued on it and the call returns without synchronising;
 *   - the return value is POLYDL_OK (0) or a negative polydl_status; on an argument error
 *     nothing is enqueued and no output byte is written;
 *   - tensors are dense, contiguous float32 unless stated; input and output must not overlap;
 *   - memory of its own: a convolution or matrix product whose reduction is split over
 *     several workgroups (split_k > 1, or the leftover tiles of rasters 2 and 3) keeps partial tiles
 *     and arrival counters in a device buffer the library allocates with hipMalloc on first
 *     need, one per (device, stream), and keeps until the process ends.  When a later problem
 *     needs more, a larger buffer is allocated (this waits for the device) and the smaller one is
 *     kept, not freed, so launches recorded earlier stay valid.  Calls on ONE stream share the
 *     buffer safely (they run in order); calls on different streams use different buffers.  An
 *     allocation failure is reported as POLYDL_ERR_LAUNCH;
 *   - HIP graphs: every entry point may be captured.  Three rules follow from the scratch memory
 *     above.  (1) A call that would have to allocate or grow it while its stream is being
 *     captured returns POLYDL_ERR_UNSUPPORTED and records nothing: run the same call once on
 *     that stream before capturing (or use polydl_conv2d_fwd_noalloc).  (2) A graph keeps the
 *     scratch addresses of its capture stream; they stay valid for the life of the process.
 *     (3) Replaying the graph, on any stream, uses the scratch memory of the stream it was
 *     CAPTURED on: do not let a replay overlap in time with other split-reduction work of this
 *     library enqueued on that capture stream (or with another replay of the same graph); their
 *     partial tiles and counters would mix.
 */
#ifndef POLYDL_H
#define POLYDL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum polydl_status {
    POLYDL_OK = 0,
    POLYDL_ERR_NULL_POINTER = -1,   /* a required pointer is NULL */
    POLYDL_ERR_BAD_DIMENSION = -2,  /* a size <= 0, stride <= 0, pad < 0, or no output (P or Q <= 0) */
    POLYDL_ERR_UNSUPPORTED = -3,    /* valid problem outside the kernels' index range, bad override */
    POLYDL_ERR_LAUNCH = -4,         /* the HIP runtime refused the launch or an allocation */
    POLYDL_ERR_NO_DEVICE = -5,      /* the current device is not a gfx950 GPU (or there is none) */
    POLYDL_ERR_SCRATCH_LIMIT = -6   /* polydl_conv2d_fwd_noalloc: the problem's variant needs more scratch
                                       memory than the fixed array holds; nothing was enqueued */
} polydl_status;

/* Element-wise operator applied to every output after the reduction (section "Operator
 * Fusion": the operator is placed in the peeled last iteration of the reduction loops, which
 * on this hardware is the kernel's epilogue).  ReLU y = max(x,0); ReLU6 y = min(max(x,0),6)
 * (section "Evaluation of Operator Fusion"). */
typedef enum polydl_act { POLYDL_ACT_NONE = 0, POLYDL_ACT_RELU = 1, POLYDL_ACT_RELU6 = 2 } polydl_act;

/* A point of the variant space (section "Compile Time Selection of Top performing code
 * version": variants differ in tile sizes and loop order; figure "A code version generated for
 * PolyDL": two tiling levels around the microkernel).  Here level 2 is the workgroup tile of
 * the implicit GEMM, level 1 the tile one 64-lane wave keeps in accumulator registers.
 * For convolution the GEMM is out[K][N*P*Q] = wt[K][C*R*S] * im2col[C*R*S][N*P*Q], so
 * bm tiles output channels and bn tiles output pixels; for SGEMM bm tiles M and bn tiles N. */
typedef struct polydl_tile_cfg {
    int bm, bn, bk;   /* workgroup tile: bm x bn outputs, bk reduction elements per stage      */
    int wm, wn;       /* wave tile (multiples of 32); the workgroup has (bm/wm)*(bn/wn) waves  */
    int split_k;      /* >= 1: the reduction is cut into this many parts (one workgroup each);  */
    int layout;       /* 0: read NCHW / KCRS directly; 1: via blocked NCHWc / KCRSck copies;
                         2: gather kernel reading the filter's [K][R][S][C] copy, reduction walked
                         tap by tap (polydl_conv2d_fwd_tap)                                      */
    int raster;       /* 0: workgroups walk M fastest; 1: chunked per XCD, grouped for L2 reuse;
                         2 (convolution, algo 0, split_k 1): order 0, and when the tile count
                         leaves a last round of workgroups that at most half of the compute units
                         take part in, each tile of that round is cut into parts along the
                         reduction (summed through scratch tiles in a fixed order);
                         3: the same cut with the tiles in order 1 (what the picker ranks)   */
    int algo;         /* convolution only.  0: im2col columns gathered element by element from
                         HBM (any shape); 1: input rows staged once per workgroup in LDS and the
                         taps formed on the LDS read (bk is ignored, the stage is cb channels);
                         2: pointwise kernel for R = S = 1, stride 1, pad 0, C in {16, 32, 64},
                         K a multiple of 64 with 128 <= K and K*C <= 16384, H*W even, tensors
                         below 2 GiB, in/out 8-byte and wt/bias 16-byte aligned: the filter
                         stays in LDS, a wave loads 64 pixels straight into registers and forms
                         the output channels 32 at a time.  One variant (bm = wm = 32, bn = wn = 64,
                         bk = 0, split_k = 1, raster = 0, cb = 0); forced on any other problem the
                         call returns POLYDL_ERR_UNSUPPORTED */
    int cb;           /* algo 1: input channels per stage, even, >= 2; 0 lets the library choose */
} polydl_tile_cfg;

/* ---- forward convolution ------------------------------------------------------------------
 * out[n][k][p][q] = act( bias[k] + sum_{c,r,s} in[n][c][p*stride+r-pad][q*stride+s-pad] * wt[k][c][r][s] )
 * with taps outside the image contributing zero (the paper's listing has no padding; logical
 * zero padding is this library's reading), no filter flip, the same stride and pad on both
 * axes, P = floor((H+2*pad-R)/stride)+1 and Q likewise from W and S.
 *   in   N*C*H*W floats, NCHW.      wt  K*C*R*S floats, KCRS.
 *   bias K floats or NULL (= none). out N*K*P*Q floats, NKPQ, overwritten.
 *   fuse_relu: 0 = no activation, 1 = ReLU.  (polydl_conv2d_fwd_act takes any polydl_act.)
 * Accumulation is float32 on the matrix cores; the summation order is unspecified but fixed for
 * a given tile configuration, so repeated calls agree bit for bit. */
int polydl_conv2d_fwd(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                      const float *in, const float *wt, const float *bias, float *out,
                      int fuse_relu, void *stream);

int polydl_conv2d_fwd_act(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                          const float *in, const float *wt, const float *bias, float *out,
                          int act /* polydl_act */, void *stream);

/* The same with an element-wise operator BEFORE the convolution fused in as well (the symmetric
 * case of section "Operator Fusion": an element-wise operator fused with the heavy operator that
 * follows it): out = act(conv(pre_act(in)) + bias), where pre_act (a polydl_act) is applied to
 * every input element as it is read, so the activated input is never written to memory.  Padding
 * contributes zeros (ReLU and ReLU6 of zero).  Served by the gather kernel (algo 0) only: with a
 * forced algo 1 or algo 2 variant and pre_act != POLYDL_ACT_NONE the call returns POLYDL_ERR_UNSUPPORTED. */
int polydl_conv2d_fwd_pre_act(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                              const float *in, const float *wt, const float *bias, float *out,
                              int pre_act /* polydl_act */, int act /* polydl_act */, void *stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): polydl_conv2d_fwd_act with the scratch memory of split
 * reductions taken from a fixed array inside the library's code object instead of from
 * hipMalloc.  Same arguments, same variant choice and bit for bit the same result as
 * polydl_conv2d_fwd_act.  The call makes no hipMalloc / hipFree and no call into an allocating
 * library.  The array holds 64 MiB of partial tiles and 16384 arrival counters per device (each
 * device the library runs on keeps its copy until the process ends); a problem whose chosen variant
 * needs more returns POLYDL_ERR_SCRATCH_LIMIT with nothing enqueued (an unsplit variant, forced
 * through polydl_set_tile_override, needs none).  Every call on a device shares that device's
 * array, whatever its stream: the counters a call uses are cleared by a small kernel on its stream
 * first, and two calls that overlap in time on one device race on it -- keep them on one stream or
 * order them with events. */
int polydl_conv2d_fwd_noalloc(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                              const float *in, const float *wt, const float *bias, float *out,
                              int act /* polydl_act */, void *stream);

/* Convolution with the filter also given in a blocked layout (figure "The 2-D Convolution code":
 * the listing's filter is blocked; section "Microkernel Specification": the order of the reduction
 * is free).  wt_tap is the same filter as [K][R][S][C], that is KCRSck with bc = C and bk = 1,
 * written by polydl_kcrs_to_kcrsck(K, C, R, S, C, 1, wt, wt_tap, stream): K*C*R*S floats of device
 * memory owned by the caller, 16-byte aligned, prepared once per filter and reused while wt does
 * not change (the library keeps no copy and cannot tell a stale one).  With it, the gather kernel
 * can walk the reduction tap by tap (all channels of a tap, then the next tap), so that a whole
 * stage of the reduction shares one tap: the padding test and the address distance are then found
 * once per stage instead of once per element.  Used when R*S is 2..63 and C is a multiple of the
 * stage depth (16); otherwise, or with wt_tap NULL or aligned to less, the call is
 * polydl_conv2d_fwd_act.  The picker chooses among the same variants, the gather ones priced for
 * the cheaper addressing (tile layout 2); the other kernels read wt.  Result: the same sum in
 * another order, the same tolerance.  Arguments, ownership and errors otherwise as
 * polydl_conv2d_fwd_act. */
int polydl_conv2d_fwd_tap(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                          const float *in, const float *wt, const float *wt_tap, const float *bias, float *out,
                          int act /* polydl_act */, void *stream);

/* ---- matrix product ------------------------------------------------------------------------
 * C[i][j] += sum_k A[i][k] * B[k][j]   (alpha = beta = 1, the reading taken of section "GEMM").
 * Row-major, A is M x K, B is K x N, C is M x N and is read and accumulated into.  K = 0 is
 * allowed (C is left as it is). */
int polydl_sgemm(int M, int N, int K, const float *A, const float *B, float *C, void *stream);

/* The general form the text of section "GEMM" states, C = beta*C + alpha*A*B, with both scalars
 * applied once per element of C (the baseline listing of that section applies beta inside the
 * reduction loop, which agrees only for beta = 1).  Same operands, layout and errors as
 * polydl_sgemm; alpha = beta = 1 gives bit for bit the result of polydl_sgemm.  beta = 0 writes C
 * without reading it (what C held, NaN included, does not reach the result).  K = 0 scales C. */
int polydl_sgemm_ex(int M, int N, int K, float alpha, const float *A, const float *B, float beta, float *C,
                    void *stream);

/* ---- blocked layouts (figure "The 2-D Convolution code": the listing indexes
 * input[img][ifm_tile][h][w][ifm] and filter[ofm_tile][ifm_tile][kj][ki][ifm][ofm]) --------------
 * polydl_nchw_to_nchwc:  out[n][c/b][h][w][c%b] = in[n][c][h][w]; out has N*ceil(C/b)*H*W*b floats,
 *   channels beyond C are written as zeros.  1 <= b <= 32.  polydl_nchwc_to_nchw is the inverse
 *   (reads the blocked tensor, writes N*C*H*W floats).
 * polydl_kcrs_to_kcrsck: out[k/bk][c/bc][r][s][c%bc][k%bk] = wt[k][c][r][s]; out has
 *   ceil(K/bk)*ceil(C/bc)*R*S*bc*bk floats, entries beyond K or C are zeros.
 * The paper runs only layers whose channel counts are multiples of the block; zero filling a
 * partial last block is this library's reading.  Pure permutations: results are bit exact. */
int polydl_nchw_to_nchwc(int N, int C, int H, int W, int b, const float *in, float *out, void *stream);
int polydl_nchwc_to_nchw(int N, int C, int H, int W, int b, const float *in, float *out, void *stream);
int polydl_kcrs_to_kcrsck(int K, int C, int R, int S, int bc, int bk, const float *wt, float *out, void *stream);

/* ---- bfloat16 inputs, float32 accumulation and output -------------------------------------------
 * The same convolution with `in` and `wt` given as bfloat16 bit patterns (uint16_t; the paper is
 * fp32 only, this is the reduced-precision configuration of the workload list).  Products of two
 * bfloat16 values are exact in float32, sums are float32 on the matrix cores
 * (v_mfma_f32_32x32x16_bf16), bias and out are float32.
 *
 * The kernel consumes the blocked layouts with a channel block of eight (16 bytes = one matrix-
 * core operand): in8c = [N][ceil(C/8)][H][W][8], wt8c = [K][ceil(C/8)][R][S][8] (that is KCRSck with
 * bc = 8, bk = 1), channels beyond C zero.  polydl_nchw_to_nchwc_bf16 / polydl_kcrs_to_kcrsck_bf16
 * produce them (bit-exact permutations).  polydl_conv2d_fwd_bf16_blocked takes blocked tensors
 * (16-byte aligned); polydl_conv2d_fwd_bf16 takes NCHW / KCRS bfloat16 and blocks them into a
 * caller-provided workspace of at least polydl_conv2d_bf16_workspace_bytes() bytes (256-byte
 * aligned device memory, contents undefined afterwards) before running the same kernel. */
int polydl_nchw_to_nchwc_bf16(int N, int C, int H, int W, int b, const uint16_t *in, uint16_t *out, void *stream);
int polydl_kcrs_to_kcrsck_bf16(int K, int C, int R, int S, int bc, int bk, const uint16_t *wt, uint16_t *out,
                               void *stream);
int polydl_conv2d_fwd_bf16_blocked(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                                   const uint16_t *in8c, const uint16_t *wt8c, const float *bias, float *out,
                                   int act /* polydl_act */, void *stream);
size_t polydl_conv2d_bf16_workspace_bytes(int N, int C, int H, int W, int K, int R, int S);
int polydl_conv2d_fwd_bf16(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                           const uint16_t *in, const uint16_t *wt, const float *bias, float *out, int act,
                           void *workspace, size_t workspace_bytes, void *stream);

/* ---- the element-wise operators as separate kernels (section "Operator Fusion": what the fused
 * epilogue of polydl_conv2d_fwd replaces; kept for the fused-versus-unfused comparison) ---------
 * polydl_bias_add:   y[n][k][p][q] += bias[k], in place on an NKPQ tensor.
 * polydl_activation: y = max(y,0) (POLYDL_ACT_RELU) or min(max(y,0),6) (POLYDL_ACT_RELU6), in
 *   place on `count` floats. */
int polydl_bias_add(int N, int K, int P, int Q, float *y, const float *bias, void *stream);

/* ---- batch normalisation followed by an activation, one pass (section "Experimental Evaluation",
 * operator-fusion experiments: the bnorm + ReLU sequence fused by the fusion algorithm) ----------
 * Inference form on an NKPQ fp32 tensor in device memory, per channel k:
 *   y = act(gamma[k] * (x - mean[k]) / sqrt(var[k] + eps) + beta[k])
 * gamma, beta, mean, var: K floats each (device); eps >= 0; y may be x (in place) or a disjoint
 * tensor of the same shape; act as in polydl_act (POLYDL_ACT_NONE gives the unfused first half,
 * polydl_activation the second).  Nothing is retained.  N*K*P*Q must be below 2^31.
 * Errors: BAD_DIMENSION, NULL_POINTER, UNSUPPORTED (act, eps, size), LAUNCH. */
int polydl_bnorm_fwd(int N, int K, int P, int Q, const float *x, const float *gamma, const float *beta,
                     const float *mean, const float *var, float eps, float *y, int act /* polydl_act */,
                     void *stream);
int polydl_activation(int64_t count, float *y, int act, void *stream);

/* ---- the reuse model (sections "Working set size computation" and "Poly-ranking algorithm") ------
 * polydl_reuse_analyse (declared below, before polydl_reuse_bucket): the working sets of a small loop nest.
 * polydl_reuse_bucket: algorithm "Compute working set sizes w.r.t cache sizes": the n working set
 *   sizes ws[] are sorted ascending and each is added to the first of the nlevels levels (fastest
 *   first, capacities sizes[]) where it still fits beside what is already there; the rest is
 *   summed into *mem.  levels[] receives the per-level sums.  Host pointers.
 * polydl_reuse_cost: equation (1) with lat/bw given as one weight per level:
 *   sum_i levels[i]*weights[i] + mem*mem_weight.  Lower is better.
 * polydl_model_conv2d / polydl_model_sgemm: the model's report for one variant of one problem.
 * polydl_pick_conv2d / polydl_pick_sgemm: the variant with the lowest predicted time over the
 *   compiled family (what polydl_conv2d_fwd / polydl_sgemm use when no override is set).
 * The report holds the working sets of the variant's reuses in bytes (accumulator tile, LDS stage,
 * one column-tile step, the workgroups resident on one XCD, the whole problem), the level each was
 * placed in by algorithm "Compute working set sizes w.r.t cache sizes" over (accumulator registers,
 * LDS, L2, Infinity Cache) + memory, the per-level sums, equation (1) over them, the bytes each
 * reuse moves, and the predicted time split into its matrix-core, data and fixed parts.  The data
 * part charges every reuse's bytes at the rate of the level its working set was placed in. */
typedef struct polydl_model_report {
    double predicted_us, mfma_us, mem_us, fixed_us;
    double ws[8];
    int n_ws;
    double level_bytes[4];
    double mem_bytes;
    double eq1_cost;
    int workgroups;
    double simd_load;   /* waves the busiest SIMD has to run one after another */
    int ws_level[8];    /* per working set: the level algorithm 2 placed it in (0 .. 3, 4 = memory) */
    double ws_traffic[8]; /* per working set: bytes that move because of that reuse over the whole launch */
} polydl_model_report;

/* The memory hierarchy the model places working sets in: four levels, fastest first (accumulator
 * registers of a wave, LDS share of a workgroup, one XCD's L2, Infinity Cache), each with a capacity
 * in bytes and the rate in GB/s the whole chip sustains from it (1 / rate is the level's weight in
 * equation (1)), then memory's rate.  polydl_model_get_levels reads the table; polydl_model_set_levels
 * replaces it for every later model and pick of the process (capacities > 0 and ascending, rates > 0;
 * POLYDL_ERR_BAD_DIMENSION otherwise) and drops the picks cached so far.  Host pointers, 4 doubles each. */
int polydl_model_get_levels(double *capacity_bytes, double *gbytes_per_s, double *mem_gbytes_per_s);
int polydl_model_set_levels(const double *capacity_bytes, const double *gbytes_per_s, double mem_gbytes_per_s);

/* polydl_reuse_analyse: algorithm "Compute working set sizes" (section "Working set size
 * computation") on a small perfect loop nest, by enumerating its iterations (no polyhedral
 * library): at most POLYDL_REUSE_MAX_LOOPS loops with extents >= 1 and at most
 * POLYDL_REUSE_MAX_ITERATIONS iterations in all, outermost loop first, executed in that order;
 * parallel[l] != 0 marks loop l parallel (parallel may be NULL = none).  refs are nrefs (1 .. 16)
 * array references with affine subscripts: subscript d of a reference is
 * offset[d] + sum_l coef[d][l] * iterator[l].  A dependence is a pair of references to the same
 * array with all pairs of iterations (I before I') in which they touch the same element; reads
 * and writes are not distinguished, and reference pairs with identical iteration pairs are
 * reported once (n_pairs of them; src_ref/tgt_ref name the first).  Sequential dependence:
 * source = its lexicographically first source iteration, min_target/max_target = that source's
 * first and last target, ws[0] = WS_min and, if the targets differ, ws[1] = WS_max: distinct
 * array elements touched from the source up to and including the target.  A dependence that
 * spans iterations of a parallel loop (parallel = 1): ws[0] = WS_par, the elements touched by the
 * whole nest with the iterators outside the outermost such loop held at the source's values.
 * Sizes are in elements.  All pointers are host pointers.  *ndeps receives the number of
 * dependences found; the first min(*ndeps, max_deps) are written.  POLYDL_ERR_BAD_DIMENSION for
 * sizes outside the limits above, POLYDL_ERR_UNSUPPORTED if a dependence has more than 2^20
 * iteration pairs or all dependences together more than 2^24. */
#define POLYDL_REUSE_MAX_LOOPS 8
#define POLYDL_REUSE_MAX_ITERATIONS 65536
typedef struct polydl_loop_ref {
    int array;                                  /* which array (any integer id) */
    int rank;                                   /* number of subscripts, 1 .. 4 */
    int coef[4][POLYDL_REUSE_MAX_LOOPS];
    int offset[4];
} polydl_loop_ref;
typedef struct polydl_reuse_dep {
    int src_ref, tgt_ref, n_pairs, parallel;
    int n_ws;
    double ws[2];
    int source[POLYDL_REUSE_MAX_LOOPS], min_target[POLYDL_REUSE_MAX_LOOPS], max_target[POLYDL_REUSE_MAX_LOOPS];
} polydl_reuse_dep;
int polydl_reuse_analyse(int nloops, const int *extents, const int *parallel, int nrefs, const polydl_loop_ref *refs,
                         int max_deps, polydl_reuse_dep *deps, int *ndeps);
int polydl_reuse_bucket(int n, const double *ws, int nlevels, const double *sizes, double *levels, double *mem);
double polydl_reuse_cost(int nlevels, const double *levels, double mem, const double *weights, double mem_weight);
int polydl_model_conv2d(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                        const polydl_tile_cfg *cfg, polydl_model_report *report);
int polydl_model_sgemm(int M, int N, int K, const polydl_tile_cfg *cfg, polydl_model_report *report);
int polydl_pick_conv2d(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                       polydl_tile_cfg *cfg, polydl_model_report *report);
int polydl_pick_sgemm(int M, int N, int K, polydl_tile_cfg *cfg, polydl_model_report *report);
/* The same two for the bfloat16 convolution (C counts channels; cfg is an algo 1 variant with its
 * cb and split_k set): the predicted time in microseconds of one variant, and the variant
 * polydl_conv2d_fwd_bf16_blocked uses when no override is set.  predicted_us may be NULL in the
 * pick.  POLYDL_ERR_UNSUPPORTED for a variant that is not compiled or cannot hold the problem. */
int polydl_model_conv2d_bf16(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                             const polydl_tile_cfg *cfg, double *predicted_us);
int polydl_pick_conv2d_bf16(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                            polydl_tile_cfg *cfg, double *predicted_us);

/* ---- learned ranking (section "DNN-based ranking algorithm") ---------------------------------
 * A feed-forward network compares two variants from their statistics; every variant plays every
 * other one and the variants are ranked by games won.  All pointers are host pointers; all
 * arithmetic is double precision on the host.
 *
 * Network (that section and its architecture figure): 2*POLYDL_RANKER_STATS inputs, hidden
 * layers of 64, 32, 16 and 8 units with relu, relu, softsign and relu, two outputs under a
 * softmax.  An output above theta (the paper uses 0.6) counts as 1: the first output means the
 * first variant wins, the second output the second variant, neither a draw.
 *
 * Statistics of a variant, POLYDL_RANKER_STATS doubles, all >= 0: the four level_bytes and the
 * mem_bytes of its model report (the result of algorithm "Compute working set sizes w.r.t cache
 * sizes", which is all the paper feeds its network), then mfma_us, mem_us and fixed_us of the same
 * report, which carry what the split factor and the grid's fit to the chip change.  Before they
 * enter the network the byte counts of both variants are divided by the sum of the byte counts
 * of both, and the times by the sum of the times of both (the paper's normalisation, once per
 * unit of measurement; a sum of 0 leaves zeros).  Network input: variant 1's eight, variant 2's eight.
 *
 * polydl_ranker_num_params: length of the parameter vector.
 * polydl_ranker_set_params: copies the parameters (per layer: weights W[out][in] row-major, then
 *   biases b[out]); count must equal polydl_ranker_num_params(), every value finite.  Until it
 *   has succeeded once the calls below return POLYDL_ERR_UNSUPPORTED.  Process-wide.
 * polydl_ranker_stats_conv2d: the statistics of one fp32 convolution variant (errors as
 *   polydl_model_conv2d).
 * polydl_ranker_play: one game; probs[2] (may be NULL) receives the two outputs, *winner (may be
 *   NULL) 1, 2 or 0 for a draw.
 * polydl_ranker_tournament: stats holds n * POLYDL_RANKER_STATS doubles, 0 <= n <= 1024 (a full tournament of 1024 takes a few seconds).  Every
 *   ordered pair (i first, j second), i != j, plays once: n*(n-1) games.  wins[n] (may be NULL)
 *   receives the games each variant won, order[n] (may be NULL) the variants from most to fewest
 *   wins, equal wins in the order given.
 * polydl_pick_conv2d_learned: the tournament over the same candidates polydl_pick_conv2d ranks;
 *   *cfg receives the winner, *report (may be NULL) its model report, *wins (may be NULL) its
 *   games won out of *games (may be NULL) = 2 * (candidates - 1) played.  polydl_conv2d_fwd does
 *   not use it: it is reported next to the model's pick and the sweep.
 * POLYDL_ERR_BAD_DIMENSION for a wrong count, a negative or non-finite statistic or a theta
 * outside [0, 1]. */
#define POLYDL_RANKER_STATS 8
int polydl_ranker_num_params(void);
int polydl_ranker_set_params(const double *params, int count);
int polydl_ranker_stats_conv2d(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                               const polydl_tile_cfg *cfg, double *stats);
int polydl_ranker_play(const double *stats1, const double *stats2, double theta, double *probs, int *winner);
int polydl_ranker_tournament(int n, const double *stats, double theta, int *wins, int *order);
int polydl_pick_conv2d_learned(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                               double theta, polydl_tile_cfg *cfg, polydl_model_report *report, int *wins,
                               int *games);

/* ---- variant control (the sweep forces a variant; reports read back the one used) -----------
 * polydl_set_tile_override: cfg != NULL forces that variant for every later call of the
 * calling process (POLYDL_ERR_UNSUPPORTED if it is not a compiled variant; a later problem it
 * cannot serve returns POLYDL_ERR_UNSUPPORTED); cfg == NULL returns to the reuse-model pick.
 * polydl_get_last_tile: the variant the most recent successful conv/sgemm call launched.
 * polydl_num_variants / polydl_get_variant: enumerate the compiled family
 * (kind 0 = convolution, 1 = sgemm, 2 = bfloat16 convolution). */
int polydl_set_tile_override(const polydl_tile_cfg *cfg);
int polydl_get_last_tile(polydl_tile_cfg *cfg);
/* The candidate lists the pickers rank, for an exhaustive sweep over exactly the same space
 * (section "Experimental Evaluation": the picked variant against the best of all variants).
 * polydl_conv2d_candidates: kind 0 = what polydl_pick_conv2d ranks (fp32: kernel, tile, stage depth,
 *   split factor, leftover-tile switch), kind 3 = the same when polydl_conv2d_fwd_tap is given
 *   the filter copy (gather variants in tile layout 2 where it applies), kind 2 = what
 *   polydl_pick_conv2d_bf16 ranks (C counts channels).  polydl_sgemm_candidates: what polydl_pick_sgemm ranks.
 * *count receives the number of candidates; the first min(*count, max_cfgs) are written to cfgs
 * (host memory; cfgs may be NULL when max_cfgs is 0).  Errors as the matching pick function. */
int polydl_conv2d_candidates(int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int kind,
                             int max_cfgs, polydl_tile_cfg *cfgs, int *count);
int polydl_sgemm_candidates(int M, int N, int K, int max_cfgs, polydl_tile_cfg *cfgs, int *count);
int polydl_num_variants(int kind);
int polydl_get_variant(int kind, int index, polydl_tile_cfg *cfg);

const char *polydl_status_string(int status);
/* hipError_t of the most recent launch the runtime refused (POLYDL_ERR_LAUNCH), 0 if none. */
int polydl_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* POLYDL_H */
