// Learned ranking of code variants (section "DNN-based ranking algorithm"): a small feed-forward
// network compares the statistics of two variants, a tournament over all ordered pairs ranks them
// by games won.  Host code, double precision.
//
// Network of that section's architecture figure: 2 * POLYDL_RANKER_STATS inputs, hidden layers of
// 64 (relu), 32 (relu), 16 (softsign) and 8 (relu) units, 2 outputs under a softmax.  An output
// above the threshold counts as 1; first output 1 = first variant wins, second output 1 = second
// variant wins, neither = draw.
//
// Inputs: the statistics of both variants divided by their sum over the two variants together
// (so the network sees which variant has the larger working sets), once for the five byte
// counts of algorithm "Compute working set sizes w.r.t cache sizes" and once for the three
// times that stand for occupancy here.
#include <algorithm>
#include <cmath>
#include <mutex>
#include <numeric>
#include <vector>
#include "internal.hpp"

namespace polydl {

namespace {

constexpr int S = POLYDL_RANKER_STATS;
constexpr int kSizes = 5;   // leading statistics measured in bytes; the rest are microseconds
constexpr int kLayers = 5;
constexpr int kWidth[kLayers + 1] = {2 * S, 64, 32, 16, 8, 2};
enum Act { RELU, SOFTSIGN, SOFTMAX };
constexpr Act kAct[kLayers] = {RELU, RELU, SOFTSIGN, RELU, SOFTMAX};

constexpr int num_params()
{
    int n = 0;
    for (int l = 0; l < kLayers; ++l) n += kWidth[l] * kWidth[l + 1] + kWidth[l + 1];
    return n;
}

std::mutex g_mu;
std::vector<double> g_params;   // empty until ranker_set_params()

void inputs_of(const double *a, const double *b, double *x)
{
    double bytes = 0, us = 0;
    for (int k = 0; k < S; ++k) (k < kSizes ? bytes : us) += a[k] + b[k];
    for (int k = 0; k < S; ++k) {
        const double total = k < kSizes ? bytes : us;
        x[k] = total > 0 ? a[k] / total : 0.0;
        x[S + k] = total > 0 ? b[k] / total : 0.0;
    }
}

void forward(const double *p, const double *x, double *out)
{
    double h[64], z[64];
    std::copy(x, x + kWidth[0], h);
    for (int l = 0; l < kLayers; ++l) {
        const int n_in = kWidth[l], n_out = kWidth[l + 1];
        const double *W = p, *b = p + n_in * n_out;
        p = b + n_out;
        for (int o = 0; o < n_out; ++o) {
            double acc = 0;
            for (int i = 0; i < n_in; ++i) acc += W[o * n_in + i] * h[i];
            z[o] = acc + b[o];
        }
        if (kAct[l] == RELU) {
            for (int o = 0; o < n_out; ++o) h[o] = z[o] > 0 ? z[o] : 0.0;
        } else if (kAct[l] == SOFTSIGN) {
            for (int o = 0; o < n_out; ++o) h[o] = z[o] / (1.0 + std::fabs(z[o]));
        } else {
            const double m = std::max(z[0], z[1]);
            const double e0 = std::exp(z[0] - m), e1 = std::exp(z[1] - m);
            h[0] = e0 / (e0 + e1);
            h[1] = e1 / (e0 + e1);
        }
    }
    out[0] = h[0];
    out[1] = h[1];
}

int winner_of(const double *probs, double theta) { return probs[0] > theta ? 1 : (probs[1] > theta ? 2 : 0); }

}  // namespace

int ranker_num_params() { return num_params(); }

void ranker_set_params(const double *params)
{
    std::lock_guard<std::mutex> lock(g_mu);
    g_params.assign(params, params + num_params());
}

bool ranker_ready()
{
    std::lock_guard<std::mutex> lock(g_mu);
    return !g_params.empty();
}

bool ranker_play(const double *stats1, const double *stats2, double theta, double *probs, int *winner)
{
    std::vector<double> p;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        p = g_params;
    }
    if (p.empty()) return false;
    double x[2 * S], out[2];
    inputs_of(stats1, stats2, x);
    forward(p.data(), x, out);
    if (probs) { probs[0] = out[0]; probs[1] = out[1]; }
    if (winner) *winner = winner_of(out, theta);
    return true;
}

bool ranker_tournament(int n, const double *stats, double theta, int *wins, int *order)
{
    std::vector<double> p;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        p = g_params;
    }
    if (p.empty()) return false;
    std::vector<int> w(n, 0);
    double x[2 * S], out[2];
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j) {
            if (i == j) continue;
            inputs_of(stats + (size_t)i * S, stats + (size_t)j * S, x);
            forward(p.data(), x, out);
            const int won = winner_of(out, theta);
            if (won == 1) ++w[i];
            else if (won == 2) ++w[j];
        }
    if (wins) std::copy(w.begin(), w.end(), wins);
    if (order) {
        std::iota(order, order + n, 0);
        std::stable_sort(order, order + n, [&](int a, int b) { return w[a] > w[b]; });
    }
    return true;
}

void ranker_stats(const polydl_model_report &r, double *stats)
{
    for (int k = 0; k < 4; ++k) stats[k] = r.level_bytes[k];
    stats[4] = r.mem_bytes;
    stats[5] = r.mfma_us;
    stats[6] = r.mem_us;
    stats[7] = r.fixed_us;
}

}  // namespace polydl
