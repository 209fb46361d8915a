// Tile-configuration picker: the paper's reuse analysis re-derived for the CDNA4 memory hierarchy.
//
// PolyDL ranks loop-nest variants without running them (section "Compile Time Selection of Top
// performing code version"): algorithm "Compute working set sizes" lists, per data reuse, how much
// data is touched between the source and the target of the reuse; algorithm "Compute working set
// sizes w.r.t cache sizes" places every working set in the fastest level it fits; equation (1)
// charges each level's working sets with that level's cost per byte.  Here the variants are the
// compiled tile family, the loop nest is fixed (workgroup tile around a register-resident wave
// tile), so the working sets have closed forms, and the levels are accumulator registers, LDS,
// the XCD's L2 and the Infinity Cache, with HBM as memory.
//
// Two additions the GPU needs, both stated by the paper as requirements of a good schedule
// (section "Introduction": load-balanced parallel loops; section "The GEMM microkernel": the
// microkernel must keep the vector/matrix unit busy):
//   * a matrix-core term: the MFMA cycles of the busiest SIMD after the workgroups are dealt to
//     256 compute units, divided by an issue efficiency that depends on the wave tile and the
//     stage depth;
//   * the data term weights each reuse by the bytes that actually travel (the operand panel times
//     the number of times it is fetched) instead of by the working-set size alone.
// The predicted time is max(matrix-core term, data term) + fixed costs; the lowest wins, as in
// the paper's ranking (lower cost = higher rank).
#include <algorithm>
#include <cmath>
#include <cstring>
#include <vector>
#include "internal.hpp"

namespace polydl {

// ---- hardware table (MI355X; capacities are public figures, rates are measured or assumed) -----
struct Level {
    const char *name;
    double capacity;      // bytes available to one reuse scope at this level
    double gbytes_per_s;  // aggregate rate the whole chip sustains from this level
};
static Level kLevels[4] = {
    {"acc", 64.0 * 1024, 1e9},              // accumulator registers of one wave (256 regs x 64 lanes)
    {"lds", 80.0 * 1024, 60000.0},          // half of a CU's 160 KB: two workgroups share a CU
    {"l2", 4.0 * 1024 * 1024, 16000.0},     // one XCD's L2
    {"mall", 256.0 * 1024 * 1024, 8000.0},  // Infinity Cache
};
static double kHbmGBs = 4500.0;             // sustained mixed read/write HBM rate

void model_get_levels(double *capacity, double *gbytes_per_s, double *mem_gbytes_per_s)
{
    for (int i = 0; i < 4; ++i) { capacity[i] = kLevels[i].capacity; gbytes_per_s[i] = kLevels[i].gbytes_per_s; }
    *mem_gbytes_per_s = kHbmGBs;
}
void model_set_levels(const double *capacity, const double *gbytes_per_s, double mem_gbytes_per_s)
{
    for (int i = 0; i < 4; ++i) { kLevels[i].capacity = capacity[i]; kLevels[i].gbytes_per_s = gbytes_per_s[i]; }
    kHbmGBs = mem_gbytes_per_s;
}
static const double kClockHz = 2.4e9;
// Gather cost per element with the filter copy of tile layout 2, relative to layout 0 (fitted to a
// sweep of the 3x3 layers of the ResNet-50-shaped suite).
static const double kTapMajorGather = 0.5, kTapMajorGather11 = 0.3, kTapMajorGather21 = 0.6;
static const int kSimdsPerCU = 4, kXcds = 8;
// compute units of the current device (256 on an MI355X; also the answer when no device is visible)
#define kCUs (compute_units())

// Algorithm "Compute working set sizes w.r.t cache sizes".  placed (may be null) receives, per
// working set in the caller's order, the level it went to (nlevels = memory).
static void bucket_placed(int n, const double *ws, int nlevels, const double *sizes, double *levels, double *mem,
                          int *placed)
{
    std::vector<int> order(n);
    for (int i = 0; i < n; ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return ws[a] < ws[b]; });
    for (int i = 0; i < nlevels; ++i) levels[i] = 0;
    *mem = 0;
    for (int idx : order) {
        int at = nlevels;
        for (int i = 0; i < nlevels && at == nlevels; ++i)
            if (ws[idx] + levels[i] <= sizes[i]) at = i;
        if (at < nlevels) levels[at] += ws[idx];
        else *mem += ws[idx];
        if (placed) placed[idx] = at;
    }
}

void reuse_bucket(int n, const double *ws, int nlevels, const double *sizes, double *levels, double *mem)
{
    bucket_placed(n, ws, nlevels, sizes, levels, mem, nullptr);
}

double reuse_cost(int nlevels, const double *levels, double mem, const double *weights, double mem_weight)
{
    double c = mem * mem_weight;
    for (int i = 0; i < nlevels; ++i) c += levels[i] * weights[i];
    return c;
}

static double rate_of(int level) { return level < 4 ? kLevels[level].gbytes_per_s : kHbmGBs; }

struct Shape {   // the GEMM a candidate works on
    double Mg, Ng, Kg;           // output rows, output columns, reduction length (padded as executed)
    double a_bytes, b_bytes, d_bytes;   // operand and result tensors
    double b_tile_bytes;         // B-side bytes one workgroup fetches for its whole reduction
};

struct Cand {
    int bm, bn, wm, wn, threads;
    int split_k;
    double steps_per_stage;      // MFMA k-steps between two barriers
    double lds_bytes;
    double loop_eff;             // matrix-core share of the reduction loop's time, large wave tile, deep stage
    double wg_overhead_cycles;   // cycles a wave spends outside the reduction loop (setup, first loads, stores)
    double kernel_fixed_us;      // launch, first-stage latency and the store tail that nothing overlaps
    int max_waves_per_simd;
    // Convolution kernels are timed round by round (see model()): workgroups that are resident
    // together start, load and store in step, so each round pays its own latency.
    bool rounds = false;
    int regs = 128;              // vector registers the compiler reports for the instantiation
    double eff_sat = 0.65;       // matrix-core share of a stage once enough workgroups share a SIMD
    double t_lat_us = 0.8;       // a stage is never shorter than one global-to-LDS round trip
    double t_round_us = 8.0;     // per round: setup, first loads, epilogue of the last workgroup
    double gather_elems = 0;     // B elements a thread gathers per stage (im2col addressing in the ALUs)
    double gather_cycles = 0;    // cycles of that addressing per element
    double split_c0 = 0, split_c1 = 0;   // split reduction: microseconds, and microseconds per MB of parts
    bool tail_split = false;     // the kernel cuts the leftover tiles of an unsplit grid (tail_split())
};

// Constants below were fitted to an exhaustive sweep of the compiled family on the ResNet-50-shaped
// suite (time against reduction length, workgroup count and wave tile).
static void model(const Shape &s, const Cand &c, polydl_model_report *r)
{
    std::memset(r, 0, sizeof(*r));
    const double tiles_m = std::ceil(s.Mg / c.bm), tiles_n = std::ceil(s.Ng / c.bn);
    const double wgs = tiles_m * tiles_n * c.split_k;
    const double waves_per_wg = c.threads / 64.0;
    const double mb = c.wm / 32.0, nb = c.wn / 32.0;
    // ---- matrix-core term -----------------------------------------------------------------
    // Workgroups are dealt to the 256 CUs; a SIMD runs the waves it is given one after another
    // (two at a time share its matrix core), so the busiest SIMD sets the time: this is the
    // load-balance requirement on the parallel loops.
    const double steps = std::ceil(s.Kg / 2.0 / c.split_k);               // rank-2 updates per wave
    const double wgs_on_busiest_cu = std::ceil(wgs / kCUs);
    const double waves_on_busiest_simd = std::ceil(wgs_on_busiest_cu * waves_per_wg / kSimdsPerCU);
    double resident = std::min<double>(c.max_waves_per_simd, std::floor(2.0 * kLevels[1].capacity / c.lds_bytes) *
                                                                 waves_per_wg / kSimdsPerCU);
    resident = std::max(1.0, std::min(resident, waves_on_busiest_simd));
    // issue efficiency: small wave tiles spend more issue slots per MFMA on operand reads and
    // address updates; every stage pays a barrier and an LDS round trip; a SIMD holding a single
    // wave cannot hide either
    double eff = c.loop_eff * (1.0 - 0.16 / (mb * nb));
    eff *= c.steps_per_stage / (c.steps_per_stage + 1.0 / (mb * nb));
    if (resident < 2) eff *= 0.72;
    else if (resident * mb * nb < 4) eff *= 0.85;   // two small waves leave gaps a third would fill
    // setup plus an epilogue that grows with the accumulators a lane has to store
    const double overhead = c.wg_overhead_cycles * (0.3 + 0.7 * mb * nb / 2.0);
    const double wave_cycles = steps * mb * nb * 64.0 / eff + overhead;
    double mfma_us = waves_on_busiest_simd * wave_cycles / kClockHz * 1e6;
    if (c.rounds) {
        // Resident workgroups per CU, from registers (512 per SIMD lane, at most 8 waves per SIMD)
        // and LDS (160 KB).  The grid runs in rounds of that many workgroups per CU; within a
        // round the workgroups of a CU share its matrix cores stage by stage, and a round ends
        // with the epilogue of its workgroups before the next one's first loads are issued.
        const int waves_per_simd = std::min(8, 512 / ((c.regs + 7) / 8 * 8));
        const double by_regs = std::floor(waves_per_simd * kSimdsPerCU / waves_per_wg);
        const double by_lds = std::floor(160.0 * 1024 / c.lds_bytes);
        const double occ = std::max(1.0, std::min(by_regs, by_lds));
        double per_cu = wgs / kCUs;
        const double stages_all = std::ceil(steps / c.steps_per_stage);
        // leftover tiles cut into pieces: whole tiles are dealt evenly, the pieces make a short tail
        double tail_us = 0;
        if (c.tail_split && c.split_k == 1 && wgs < 2e9) {
            const TailSplit ts = tail_split((int)wgs, (int)stages_all, kCUs);
            if (ts.parts > 1) {
                per_cu = (wgs - ts.tiles) / kCUs;
                const double pieces = std::ceil((double)ts.tiles * ts.parts / kCUs);
                const double simd_share0 = std::ceil(waves_per_wg / kSimdsPerCU);
                tail_us = 4.0 + pieces * ts.stages_per_part *
                                    (c.steps_per_stage * mb * nb * 64.0 * simd_share0 / kClockHz * 1e6 / c.eff_sat +
                                     c.gather_elems * c.gather_cycles / kClockHz * 1e6);
            }
        }
        const double full_rounds = std::floor(per_cu / occ);
        const double rest = per_cu - full_rounds * occ;
        const double stages = std::ceil(steps / c.steps_per_stage);
        const double simd_share = std::ceil(waves_per_wg / kSimdsPerCU);
        const double t_stage = c.steps_per_stage * mb * nb * 64.0 * simd_share / kClockHz * 1e6 / c.eff_sat +
                               c.gather_elems * c.gather_cycles / kClockHz * 1e6;
        auto round_us = [&](double n) { return c.t_round_us + stages * std::max(n * t_stage, c.t_lat_us); };
        mfma_us = full_rounds * round_us(occ) + (rest > 1e-9 ? round_us(std::ceil(rest - 1e-9)) : 0.0) + tail_us;
    }
    // ---- the reuses of the nest: working set (bytes) and the bytes that travel because of it ----
    // Algorithm 2 places the working sets, smallest first, each in the fastest level that still
    // has room beside those already there; a reuse whose working set was placed in level L is
    // served from L, so its traffic is charged at L's rate: equation (1) with each level's term
    // weighted by the bytes that actually move instead of by the working-set size alone.
    enum { R_ACC = 0, R_STAGE, R_COL_STEP, R_PAR, R_ALL, N_REUSE };
    const double a_panel = c.bm * s.Kg * 4;                                // A row panel between two column tiles
    // reuse across workgroups that run together on one XCD (the dependence spans the parallel
    // loop): the footprint of everything resident there
    const double res_wgs = std::min(wgs, (double)kCUs / kXcds * std::max(1.0, resident * kSimdsPerCU / waves_per_wg));
    const double dm = std::min(tiles_m, res_wgs), dn = std::max(1.0, std::ceil(res_wgs / tiles_m));
    double ws[N_REUSE], traffic[N_REUSE];
    ws[R_ACC] = (double)c.wm * c.wn * 4;                                   // accumulators over the reduction
    ws[R_STAGE] = c.lds_bytes;                                             // staged operands, shared by the waves
    ws[R_COL_STEP] = a_panel + s.b_tile_bytes + (double)c.bm * c.bn * 4;   // one column-tile step: A panel reused by the next
    ws[R_PAR] = dm * a_panel + dn * s.b_tile_bytes;                        // B tile (and A panels) shared by concurrent tiles
    ws[R_ALL] = s.a_bytes + s.b_bytes + s.d_bytes;                         // the tensors themselves
    // A is fetched once per column tile, B once per row tile; the accumulators never leave the
    // registers; every staged element is read from LDS once per wave that multiplies it
    const double a_traffic = tiles_n * s.a_bytes, b_traffic = tiles_m * tiles_n * s.b_tile_bytes;
    traffic[R_ACC] = 0;
    traffic[R_STAGE] = tiles_m * tiles_n * s.Kg * ((double)c.bm * (c.bn / c.wn) + (double)c.bn * (c.bm / c.wm)) * 4;
    traffic[R_COL_STEP] = a_traffic - s.a_bytes;
    traffic[R_PAR] = b_traffic > s.b_bytes ? b_traffic - s.b_bytes : 0;
    traffic[R_ALL] = s.a_bytes + s.b_bytes + s.d_bytes;
    double sizes[4], weights[4];
    for (int i = 0; i < 4; ++i) { sizes[i] = kLevels[i].capacity; weights[i] = 1.0 / kLevels[i].gbytes_per_s; }
    int placed[N_REUSE];
    bucket_placed(N_REUSE, ws, 4, sizes, r->level_bytes, &r->mem_bytes, placed);
    r->eq1_cost = reuse_cost(4, r->level_bytes, r->mem_bytes, weights, 1.0 / kHbmGBs);
    r->n_ws = N_REUSE;
    for (int i = 0; i < N_REUSE; ++i) { r->ws[i] = ws[i]; r->ws_level[i] = placed[i]; r->ws_traffic[i] = traffic[i]; }
    // ---- data term ------------------------------------------------------------------------------
    // Nothing faster than L2 is shared between workgroups, and nothing faster than the Infinity
    // Cache holds a tensor from one launch to the next: reuses across workgroups are served from
    // their placed level or L2, whichever is slower; the tensors from theirs or the Infinity Cache.
    const int a_level = std::max(2, placed[R_COL_STEP]), b_level = std::max(2, placed[R_PAR]);
    const int all_level = std::max(3, placed[R_ALL]);
    const double refetch_us = traffic[R_COL_STEP] / rate_of(a_level) * 1e-3 + traffic[R_PAR] / rate_of(b_level) * 1e-3;
    const double lds_us = traffic[R_STAGE] / rate_of(std::max(1, placed[R_STAGE])) * 1e-3;
    double mem_us = traffic[R_ALL] / rate_of(all_level) * 1e-3;            // compulsory
    if (c.rounds) mem_us = std::max(mem_us, refetch_us);                   // caches and memory work side by side
    else mem_us += refetch_us;
    mem_us = std::max(mem_us, lds_us);
    double fixed = c.kernel_fixed_us;
    if (c.rounds) {
        // nothing streams the tensors faster than this, with the first and last touches exposed
        mem_us = std::max(mem_us, (s.a_bytes + s.b_bytes + s.d_bytes) / 5500.0 * 1e-3 + 2.0);
        // a layer that mostly writes is slower than that: measured on the pointwise layers of the
        // suite (batch 16 .. 128, either kernel), the output leaves at about 3.15 TB/s
        mem_us = std::max(mem_us, (s.a_bytes + s.b_bytes) / 20000.0 * 1e-3 + s.d_bytes / 3150.0 * 1e-3 + 2.0);
        if (c.split_k > 1) fixed += c.split_c0 + c.split_c1 * c.split_k * s.d_bytes * 1e-6;
    } else if (c.split_k > 1) {
        // every part writes its accumulator tile once, coalesced; the last part of each tile reads
        // them all back and runs the epilogue: no other launch, no pass over the output
        fixed += 2.0 * c.split_k * s.d_bytes / kHbmGBs * 1e-3;
    }
    r->mfma_us = mfma_us;
    r->mem_us = mem_us;
    r->fixed_us = fixed;
    r->predicted_us = std::max(mfma_us, mem_us) + fixed;
    r->workgroups = (int)std::min(wgs, 2e9);
    r->simd_load = waves_on_busiest_simd;
}

// ---- convolution ---------------------------------------------------------------------------------
// filters of five rows or more are staged one filter row at a time by the patch kernel
static int patch_rows_per_stage(const ConvProblem &q) { return q.R >= 5 ? 1 : q.R; }

static double conv_patch_rows(const ConvProblem &q, int bn)
{
    const double Rp = patch_rows_per_stage(q);
    const double PQ = (double)q.P * q.Q, Ng = q.N * PQ;
    const double run = std::min<double>(bn, Ng);
    const double rows_out = std::min<double>(std::ceil((run - 1) / q.Q) + 1, (double)q.N * q.P);
    const double imgs = std::min<double>(std::ceil((run - 1) / PQ) + 1, q.N);
    const double prs = Rp == 1 ? 1 : q.stride;
    return rows_out * prs + imgs * std::max(0.0, Rp - prs);
}

static Shape conv_shape(const ConvProblem &q, int algo, int bn, int cb)
{
    Shape s;
    const double RS = (double)q.R * q.S;
    s.Mg = q.K;
    s.Ng = (double)q.N * q.P * q.Q;
    const double cexec = algo == 1 ? std::ceil((double)q.C / cb) * cb : q.C;
    s.Kg = cexec * RS;
    s.a_bytes = (double)q.K * q.C * RS * 4;
    s.b_bytes = (double)q.N * q.C * q.H * q.W * 4;
    s.d_bytes = (double)q.N * q.K * q.P * q.Q * 4;
    if (algo == 1) {
        const double wp = q.S == 1 ? q.Q : q.W + 2 * q.pad;
        // rows staged once per channel (once per channel and filter row when staged row by row)
        s.b_tile_bytes = q.C * conv_patch_rows(q, bn) * wp * 4 * (q.R / patch_rows_per_stage(q));
    } else {
        s.b_tile_bytes = (double)bn * q.C * RS * 4;                        // every tap gathered again
    }
    return s;
}

void model_conv(const ConvProblem &q, const polydl_tile_cfg &cfg, int threads, int reg_class, polydl_model_report *r)
{
    Cand c;
    c.bm = cfg.bm; c.bn = cfg.bn; c.wm = cfg.wm; c.wn = cfg.wn; c.threads = threads;
    c.split_k = std::max(1, cfg.split_k);
    if (cfg.algo == 1) {
        const int cb = std::max(2, cfg.cb);
        const double wp = q.S == 1 ? q.Q : q.W + 2 * q.pad;
        const double RSp = (double)patch_rows_per_stage(q) * q.S;     // taps of a channel in one stage
        c.steps_per_stage = cb / 2.0 * RSp;
        // two stage buffers, one when a workgroup's share of the reduction is a single stage
        const int nstages = (q.C + cb - 1) / cb * (q.R / patch_rows_per_stage(q));
        const int per_split = (nstages + c.split_k - 1) / c.split_k;
        c.lds_bytes = (per_split > 1 ? 2.0 : 1.0) * (cfg.bm * (cb * RSp + 1) + cb * conv_patch_rows(q, cfg.bn) * wp) * 4;
        c.loop_eff = 0.74;
        c.wg_overhead_cycles = 9000;
        c.kernel_fixed_us = 14.0;
        // the small-register instantiation holds 5 waves per SIMD with a 32x32 wave tile, 3 with
        // 64x32 in the 128x64 tile; everything else 2
        c.max_waves_per_simd = 2;
        if (reg_class >= 1 && cfg.wm * cfg.wn == 32 * 32) {
            c.max_waves_per_simd = 5;      // enough waves to cover each other's loads and stores
            c.loop_eff = 0.92;
            c.wg_overhead_cycles = 4000;
        }
        else if (reg_class >= 1 && cfg.bm == 128 && cfg.bn == 64) c.max_waves_per_simd = 3;
        // fitted on the sweep, by wave tile
        const int mbn = (cfg.wm / 32) * 10 + cfg.wn / 32;
        const int rc = reg_class < 0 ? 0 : reg_class;
        c.rounds = true;
        c.kernel_fixed_us = 5.0;
        if (mbn == 11)      { static const int R[3] = {192, 80, 60};   c.regs = R[rc]; c.eff_sat = 0.65; c.t_lat_us = 0.8; c.t_round_us = 6; }
        else if (mbn == 21) { static const int R[3] = {215, 110, 89};  c.regs = R[rc]; c.eff_sat = 0.60; c.t_lat_us = 0.6; c.t_round_us = 6; }
        else                { static const int R[3] = {247, 156, 121}; c.regs = R[rc]; c.eff_sat = 0.75; c.t_lat_us = 0.6; c.t_round_us = 6; c.split_c0 = 4; }
        c.split_c1 = 0.1;
    } else {
        c.steps_per_stage = cfg.bk / 2.0;
        c.lds_bytes = 2.0 * (cfg.bm * (cfg.bk + 4) + cfg.bk * (cfg.bn + 4)) * 4;
        c.loop_eff = 0.84;
        c.wg_overhead_cycles = 5000;
        c.kernel_fixed_us = 10.0;
        c.max_waves_per_simd = (cfg.wm * cfg.wn > 64 * 64) ? 1 : ((cfg.wm * cfg.wn == 64 * 64) ? 2 : 4);
        const int mbn = (cfg.wm / 32) * 10 + cfg.wn / 32;
        const bool point = q.R == 1 && q.S == 1 && q.pad == 0;   // loads without per-lane arithmetic
        c.rounds = true;
        c.kernel_fixed_us = 5.0;
        c.gather_elems = (double)cfg.bk * cfg.bn / threads;
        switch (mbn) {
        case 11: c.regs = 62;  c.eff_sat = 0.85; c.t_lat_us = 0.6; c.t_round_us = 2; c.gather_cycles = 32; c.split_c0 = 1; break;
        case 12: c.regs = 90;  c.eff_sat = 0.80; c.t_lat_us = 1.0; c.t_round_us = 4; c.gather_cycles = 20; c.split_c0 = 2; break;
        case 21: c.regs = 88;  c.eff_sat = 0.90; c.t_lat_us = 0.8; c.t_round_us = 4; c.gather_cycles = 40; c.split_c0 = 1; break;
        case 22: c.regs = cfg.bk == 16 ? 136 : 104; c.eff_sat = 0.80; c.t_lat_us = 0.8; c.t_round_us = 2; c.gather_cycles = 40;
                 c.split_c0 = 8; c.split_c1 = 0.2; break;
        case 24: c.regs = 212; c.eff_sat = 0.70; c.t_lat_us = 0.4; c.t_round_us = 2; c.gather_cycles = 20; c.split_c0 = 15; c.split_c1 = 0.6; break;
        default: c.regs = 228; c.eff_sat = 0.80; c.t_lat_us = 0.4; c.t_round_us = 4; c.gather_cycles = 20; c.split_c0 = 15; c.split_c1 = 1.0; break;
        }
        c.tail_split = cfg.raster >= 2;
        // 1x1 filters without padding: the channel rides in the instruction's uniform offset and the
        // lanes read a contiguous run of pixels (stride 1); with a stride the lanes' addresses are
        // spread over several times the cache lines and the loads cost what gathered ones do
        if (point && q.stride == 1) c.gather_cycles *= 0.1;
        // tap by tap over the [K][R][S][C] filter copy: one tap per stage, so the validity bit and
        // the distance are worked out per stage and not per element
        // (with a stride the lanes' addresses spread over twice the cache lines and the cost of
        // the load is in the memory pipeline, which the cheaper addressing does not touch)
        if (cfg.layout == 2 && q.stride == 1)
            c.gather_cycles *= mbn == 11 ? kTapMajorGather11 : (mbn == 21 ? kTapMajorGather21 : kTapMajorGather);
        if (c.split_c1 == 0) c.split_c1 = 0.1;   // scratch tiles, as in the patch kernel
    }
    Shape s = conv_shape(q, cfg.algo, cfg.bn, std::max(2, cfg.cb));
    model(s, c, r);
}

// bfloat16 patch kernel; q.C counts units of eight channels.  Same round-by-round timing as the
// fp32 kernels with the bf16 instruction's rate (a 32x32x16 step takes 32 cycles).  The stage
// efficiency is low because every step needs two 16-byte operand reads per lane from LDS, which
// the LDS cannot deliver at the matrix cores' pace; constants fitted to a sweep of the family on
// the ResNet-50-shaped suite at batch 64.
double model_conv_bf16(const ConvProblem &q, const polydl_tile_cfg &cfg, int threads)
{
    const double RS = (double)q.R * q.S;
    const int cb = q.C == 1 ? 1 : std::max(2, cfg.cb);
    const double mb = cfg.wm / 32.0, nb = cfg.wn / 32.0, waves_per_wg = threads / 64.0;
    const double Ng = (double)q.N * q.P * q.Q;
    const double tiles = std::ceil((double)q.K / cfg.bm) * std::ceil(Ng / cfg.bn);
    const double RSp = (double)patch_rows_per_stage(q) * q.S;
    const double nstages = std::ceil((double)q.C / cb) * (q.R / patch_rows_per_stage(q));
    const double per_split = std::ceil(nstages / std::max(1, cfg.split_k));
    const double parts = std::ceil(nstages / per_split);
    const double wp = q.S == 1 ? q.Q : q.W + 2 * q.pad;
    // the kernel's stage buffers: filter rows of odd pitch, both operands rounded up to whole
    // passes of the workgroup
    const double lda = (double)(((int)(cb * RSp) + 1) | 1);
    const double stage_units = std::ceil(cfg.bm * lda / threads) * threads +
                               std::ceil(cb * conv_patch_rows(q, cfg.bn) * wp / threads) * threads;
    const double lds_bytes = ((per_split > 1 ? 2.0 : 1.0) * stage_units + 64) * 16;
    const int waves_per_simd = mb * nb == 4 ? 3 : 4;   // from the kernels' register counts
    const double occ = std::max(1.0, std::min(std::floor(waves_per_simd * kSimdsPerCU / waves_per_wg),
                                              std::floor(160.0 * 1024 / lds_bytes)));
    // per wave tile: stage efficiency, per-round latency, stage latency floor, bytes per microsecond a
    // CU stages into LDS, split cost per MB of parts
    double eff = 0.25, t_round = 3.0, t_lat = 0.8, rate = 60000.0, c1 = 0.1;
    if (mb * nb == 2) { eff = 0.4; t_round = 4.0; c1 = 0.2; }
    else if (mb * nb == 4) { eff = 0.4; t_round = 4.0; t_lat = 0.4; rate = 31000.0; c1 = 0.4; }
    // matrix instructions of a stage per accumulator block: one per tap and pair of units; a
    // reduction of a single unit takes two taps per instruction instead
    const double steps = q.C == 1 ? std::ceil(RSp / 2.0) : std::ceil(cb / 2.0) * RSp;
    const double t_stage = std::max(steps * mb * nb * 32.0 * std::ceil(waves_per_wg / kSimdsPerCU) /
                                        kClockHz * 1e6 / eff,
                                    (cfg.bm * cb * RSp + cb * conv_patch_rows(q, cfg.bn) * wp) * 16.0 / rate);
    const double per_cu = tiles * parts / kCUs;
    const double full_rounds = std::floor(per_cu / occ), rest = per_cu - full_rounds * occ;
    auto round_us = [&](double n) { return t_round + per_split * std::max(n * t_stage, t_lat); };
    double t = full_rounds * round_us(occ) + (rest > 1e-9 ? round_us(std::ceil(rest - 1e-9)) : 0.0);
    const double d_bytes = (double)q.N * q.K * q.P * q.Q * 4;
    const double mem_bytes = (double)q.N * q.C * 8 * q.H * q.W * 2 + (double)q.K * q.C * 8 * RS * 2 + d_bytes;
    t = 5.0 + std::max(t, mem_bytes / 6000.0 * 1e-3 + 2.0);
    if (parts > 1) t += c1 * parts * d_bytes * 1e-6;
    return t;
}

void model_sgemm(const SgemmProblem &q, const polydl_tile_cfg &cfg, int threads, polydl_model_report *r)
{
    Shape s;
    s.Mg = q.M; s.Ng = q.N; s.Kg = std::ceil((double)q.K / cfg.bk) * cfg.bk;
    s.a_bytes = (double)q.M * q.K * 4;
    s.b_bytes = (double)q.K * q.N * 4;
    s.d_bytes = 2.0 * q.M * q.N * 4;                                       // C is read and written
    s.b_tile_bytes = (double)cfg.bn * q.K * 4;
    Cand c;
    c.bm = cfg.bm; c.bn = cfg.bn; c.wm = cfg.wm; c.wn = cfg.wn; c.threads = threads;
    c.split_k = std::max(1, cfg.split_k);
    c.steps_per_stage = cfg.bk / 2.0;
    c.lds_bytes = 2.0 * (cfg.bm * (cfg.bk + 4) + cfg.bk * (cfg.bn + 4)) * 4;
    c.loop_eff = 0.84;
    c.wg_overhead_cycles = 3000;
    c.kernel_fixed_us = 6.0;
    // from the kernels' register counts (the eight-block wave tiles are held to 256 registers)
    c.max_waves_per_simd = (cfg.wm * cfg.wn > 64 * 64) ? 2 : ((cfg.wm * cfg.wn == 64 * 64) ? 3 : 4);
    model(s, c, r);
    if (cfg.split_k > 1) {   // every part writes its tile to scratch once, the last one reads them all back
        // plus the hand-over itself (store, count, read back), which no amount of bandwidth shortens
        r->fixed_us = c.kernel_fixed_us + 2.0 * cfg.split_k * (double)q.M * q.N * 4 / kHbmGBs * 1e-3 +
                      0.4 * (cfg.split_k - 1);
        r->predicted_us = std::max(r->mfma_us, r->mem_us) + r->fixed_us;
    }
}

static const int kSplits[] = {1, 2, 3, 4, 6, 8, 12, 16};

// Pointwise kernel (filter resident in LDS, pixels loaded straight into registers): a unit is
// 64 pixels x 32 output channels, C/2 * 2 matrix instructions; units are dealt to the waves in
// equal runs, so the busiest SIMD runs ceil(units / SIMDs) of them one after another.  The tensors
// are streamed once.
void model_conv_point(const ConvProblem &q, polydl_model_report *r)
{
    std::memset(r, 0, sizeof(*r));
    uint32_t units, wgs;
    conv_point_shape(q, kCUs, &units, &wgs);
    const double pixels = (double)q.N * q.H * q.W;
    const double in_bytes = pixels * q.C * 4, out_bytes = pixels * q.K * 4, wt_bytes = (double)q.K * q.C * 4;
    const double unit_us = (q.C / 2.0) * 2.0 * 64.0 / kClockHz * 1e6;
    const double per_simd = std::ceil((double)units / (kCUs * kSimdsPerCU));
    r->mfma_us = per_simd * unit_us / 0.85;
    // measured over batch sizes 16 .. 128 on 64 -> 64 and 64 -> 256 channels at 56 x 56 (back-to-back
    // launches on the same buffers): the time follows the bytes written, at 3.3 TB/s; the input,
    // re-read from the last-level cache, hardly shows
    r->mem_us = (in_bytes + wt_bytes) / 20000.0 * 1e-3 + out_bytes / 3300.0 * 1e-3;
    r->fixed_us = 7.0;                               // launch, filling LDS with the filter, first loads, last stores
    r->predicted_us = std::max(r->mfma_us, r->mem_us) + r->fixed_us;
    r->workgroups = (int)wgs;
    r->simd_load = per_simd;
    // reuses: accumulators of a unit (registers); the pixel registers reused by the channel groups;
    // the filter in LDS reused by every unit (read once per unit); the tensors themselves
    const double ws[4] = {32.0 * 64 * 4, 64.0 * q.C * 4, wt_bytes, in_bytes + out_bytes + wt_bytes};
    const double moved[4] = {0, 0, (double)units * 32.0 * q.C * 4, in_bytes + out_bytes + wt_bytes};
    double sizes[4], weights[4];
    for (int i = 0; i < 4; ++i) { sizes[i] = kLevels[i].capacity; weights[i] = 1.0 / kLevels[i].gbytes_per_s; }
    int placed[4];
    bucket_placed(4, ws, 4, sizes, r->level_bytes, &r->mem_bytes, placed);
    r->eq1_cost = reuse_cost(4, r->level_bytes, r->mem_bytes, weights, 1.0 / kHbmGBs);
    r->n_ws = 4;
    for (int i = 0; i < 4; ++i) { r->ws[i] = ws[i]; r->ws_level[i] = placed[i]; r->ws_traffic[i] = moved[i]; }
}

void conv_candidates(const ConvProblem &q, std::vector<ConvCandidate> *out)
{
    out->clear();
    ConvCandidate cand;
    if (conv_point_fits(q)) {
        cand.cfg = conv_point_cfg();
        model_conv_point(q, &cand.rep);
        out->push_back(cand);
    }
    const int cpad = (q.C + 1) & ~1;
    // the patch kernel copies input rows straight into LDS and cannot touch them on the way
    for (int i = 0; i < (q.pre_act ? 0 : kNumPatchVariants); ++i) {
        const PatchVariant &v = kPatchVariants[i];
        for (int cb = 2; cb <= cpad && cb <= 64; cb += 2) {
            if (cpad % cb != 0) continue;
            const int rc = v.reg_class(q, cb);
            if (rc < 0) continue;
            const int nstages = (q.C + cb - 1) / cb;
            for (int sk : kSplits) {
                if (sk > nstages) break;
                cand.cfg = {v.bm, v.bn, 0, v.wm, v.wn, sk, 0, 0, 1, cb};
                model_conv(q, cand.cfg, v.threads, rc, &cand.rep);
                out->push_back(cand);
            }
        }
    }
    const long Kg = (long)q.C * q.R * q.S;
    for (int i = 0; i < kNumVariants; ++i) {
        const Variant &v = kVariants[i];
        const long stages = (Kg + v.bk - 1) / v.bk;
        for (int sk : kSplits) {
            if (sk > stages) break;
            // raster 1: each XCD's workgroups take neighbouring tiles, so filter rows and the input rows
            // that neighbouring pixel tiles share are fetched into one L2 instead of eight (time
            // within 1 % of raster 0 on every layer measured, a third less traffic from the fabric)
            cand.cfg = {v.bm, v.bn, v.bk, v.wm, v.wn, sk, 0, 1, 0, 0};
            if (q.has_tap && gather_tap_major_fits(q, v.bk)) cand.cfg.layout = 2;   // never slower than layout 0
            model_conv(q, cand.cfg, v.threads, 0, &cand.rep);
            out->push_back(cand);
            // the same with the leftover tiles of the last round split (wave tiles up to 64x32:
            // with larger ones the pieces measured slower than the round they save)
            if (sk == 1 && v.wm * v.wn <= 64 * 32) {
                cand.cfg.raster = 3;
                model_conv(q, cand.cfg, v.threads, 0, &cand.rep);
                out->push_back(cand);
            }
        }
    }
}

bool pick_conv(const ConvProblem &q, polydl_tile_cfg *best, polydl_model_report *best_rep)
{
    std::vector<ConvCandidate> cands;
    conv_candidates(q, &cands);
    // Equal predictions are candidates held by the same data floor: of those the smaller workgroup
    // tile goes first (more workgroups, so more independent loads in flight and a shorter last round).
    auto before = [](const ConvCandidate &c, const ConvCandidate &b) {
        const double tie = 1e-6 * b.rep.predicted_us;
        if (c.rep.predicted_us < b.rep.predicted_us - tie) return true;
        if (c.rep.predicted_us > b.rep.predicted_us + tie) return false;
        return c.cfg.bm * c.cfg.bn < b.cfg.bm * b.cfg.bn;
    };
    const ConvCandidate *b = nullptr;
    for (const ConvCandidate &c : cands)
        if (!b || before(c, *b)) b = &c;
    if (!b) return false;
    *best = b->cfg;
    *best_rep = b->rep;
    return true;
}

// every (variant, split factor, workgroup order) pick_sgemm ranks
void sgemm_candidates(const SgemmProblem &q, std::vector<polydl_tile_cfg> *out)
{
    out->clear();
    for (int i = 0; i < kNumVariants; ++i) {
        const Variant &v = kVariants[i];
        const long stages = ((long)q.K + v.bk - 1) / v.bk;
        // long, skinny reductions (few output tiles) want many parts
        static const int kSgemmSplits[] = {1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64, 96, 128};
        for (int sk : kSgemmSplits) {
            if (sk > stages) break;
            for (int raster = 0; raster < 2; ++raster)
                out->push_back(polydl_tile_cfg{v.bm, v.bn, v.bk, v.wm, v.wn, sk, 0, raster, 0, 0});
        }
    }
}

bool pick_sgemm(const SgemmProblem &q, polydl_tile_cfg *best, polydl_model_report *best_rep)
{
    bool have = false;
    polydl_model_report rep;
    std::vector<polydl_tile_cfg> cands;
    sgemm_candidates(q, &cands);
    for (const polydl_tile_cfg &c : cands) {
        model_sgemm(q, c, (c.bm / c.wm) * (c.bn / c.wn) * 64, &rep);
        if (c.raster == 1) rep.predicted_us *= 0.999;   // ties go to the XCD-aware order
        if (!have || rep.predicted_us < best_rep->predicted_us) { *best = c; *best_rep = rep; have = true; }
    }
    return have;
}

}  // namespace polydl
