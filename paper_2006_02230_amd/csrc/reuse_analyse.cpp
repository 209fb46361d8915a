// Working set sizes of a small loop nest by enumeration: algorithm "Compute working set sizes"
// (section "Working set size computation") with every iteration written out instead of
// polyhedral sets, so it serves nests of a few thousand iterations -- enough to check the closed
// forms the picker uses, and to reproduce the paper's matmul example (WS_min = 2K+3,
// WS_max = N*K+N+1 for the reuse of A).  Host code.
//
// A dependence is a pair of references to one array together with all pairs of iterations
// (I before I') in which they touch the same element; reads and writes are not told apart (the
// paper takes the union of the four kinds), and reference pairs with identical iteration pairs
// are one dependence.  For a dependence carried by sequential loops: its lexicographically first
// source iteration, that source's first and last target, and the number of distinct elements
// touched from the source up to and including each of the two targets.  For a dependence that
// spans iterations of a parallel loop: the elements touched by the whole nest with the iterators
// outside the outermost such loop fixed at the first source's values.
#include <algorithm>
#include <map>
#include <vector>
#include "internal.hpp"

namespace polydl {

namespace {

struct Nest {
    int nloops;
    std::vector<int> extent;
    std::vector<long> stride;      // iteration number = sum iter[l] * stride[l]
    long count;
    void tuple(long it, int *out) const
    {
        for (int l = 0; l < nloops; ++l) { out[l] = (int)(it / stride[l]); it -= (long)out[l] * stride[l]; }
    }
};

}  // namespace

int reuse_analyse(int nloops, const int *extents, const int *parallel, int nrefs, const polydl_loop_ref *refs,
                  int max_deps, polydl_reuse_dep *deps, int *ndeps)
{
    Nest nest;
    nest.nloops = nloops;
    nest.extent.assign(extents, extents + nloops);
    nest.stride.assign(nloops, 1);
    for (int l = nloops - 2; l >= 0; --l) nest.stride[l] = nest.stride[l + 1] * extents[l + 1];
    nest.count = nest.stride[0] * extents[0];

    // element touched by reference r in iteration it, as a dense id over (array, subscripts)
    std::map<std::vector<int>, int> ids;
    std::vector<std::vector<int>> elem(nrefs, std::vector<int>(nest.count));
    std::vector<int> iter(nloops), key;
    for (long it = 0; it < nest.count; ++it) {
        nest.tuple(it, iter.data());
        for (int r = 0; r < nrefs; ++r) {
            key.assign(1, refs[r].array);
            for (int d = 0; d < refs[r].rank; ++d) {
                long v = refs[r].offset[d];
                for (int l = 0; l < nloops; ++l) v += (long)refs[r].coef[d][l] * iter[l];
                key.push_back((int)v);
            }
            auto ins = ids.insert({key, (int)ids.size()});
            elem[r][it] = ins.first->second;
        }
    }
    const int nelems = (int)ids.size();
    std::vector<int> stamp(nelems, -1);
    int stamp_now = 0;
    auto footprint = [&](long first, long last) {     // distinct elements touched by iterations first .. last
        ++stamp_now;
        int n = 0;
        for (long it = first; it <= last; ++it)
            for (int r = 0; r < nrefs; ++r)
                if (stamp[elem[r][it]] != stamp_now) { stamp[elem[r][it]] = stamp_now; ++n; }
        return n;
    };

    // dependences: iteration pairs per (source reference, target reference), merged when equal
    typedef std::vector<std::pair<int, int>> Pairs;
    std::map<Pairs, int> index;
    std::vector<const Pairs *> order;
    std::vector<std::vector<std::pair<int, int>>> members;
    std::vector<std::vector<int>> where(nelems);
    const size_t kMaxPairs = 1u << 20, kMaxStored = 16u << 20;   // per dependence, and over all of them
    size_t stored = 0;
    for (int s = 0; s < nrefs; ++s)
        for (int t = 0; t < nrefs; ++t) {
            if (refs[s].array != refs[t].array) continue;
            for (auto &w : where) w.clear();
            for (long it = 0; it < nest.count; ++it) where[elem[t][it]].push_back((int)it);
            Pairs pairs;
            for (long it = 0; it < nest.count; ++it) {
                const std::vector<int> &later = where[elem[s][it]];
                for (auto p = std::upper_bound(later.begin(), later.end(), (int)it); p != later.end(); ++p) {
                    pairs.push_back({(int)it, *p});
                    if (pairs.size() > kMaxPairs) return POLYDL_ERR_UNSUPPORTED;
                }
            }
            if (pairs.empty()) continue;
            const size_t added = pairs.size();
            auto ins = index.insert({std::move(pairs), (int)members.size()});
            if (ins.second && (stored += added) > kMaxStored) return POLYDL_ERR_UNSUPPORTED;
            if (ins.second) { order.push_back(&ins.first->first); members.emplace_back(); }
            members[ins.first->second].push_back({s, t});
        }

    *ndeps = (int)members.size();
    std::vector<int> a(nloops), b(nloops);
    for (int d = 0; d < (int)members.size() && d < max_deps; ++d) {
        const Pairs &pairs = *order[d];
        polydl_reuse_dep &o = deps[d];
        o = polydl_reuse_dep{};
        o.src_ref = members[d][0].first;
        o.tgt_ref = members[d][0].second;
        o.n_pairs = (int)members[d].size();
        int outer_par = nloops;   // outermost parallel loop in which a source and its target differ
        if (parallel)
            for (const auto &p : pairs) {
                nest.tuple(p.first, a.data());
                nest.tuple(p.second, b.data());
                for (int l = 0; l < outer_par; ++l)
                    if (parallel[l] && a[l] != b[l]) { outer_par = l; break; }
            }
        const long src = pairs.front().first;    // pairs are sorted by source, then target
        nest.tuple(src, o.source);
        if (outer_par < nloops) {
            o.parallel = 1;
            const long span = outer_par == 0 ? nest.count : nest.stride[outer_par - 1];
            const long first = src / span * span;
            o.n_ws = 1;
            o.ws[0] = footprint(first, first + span - 1);
        } else {
            long tmin = -1, tmax = -1;
            for (const auto &p : pairs) {
                if (p.first != src) break;
                if (tmin < 0) tmin = p.second;
                tmax = p.second;
            }
            nest.tuple(tmin, o.min_target);
            nest.tuple(tmax, o.max_target);
            o.ws[0] = footprint(src, tmin);
            o.n_ws = 1;
            if (tmax != tmin) { o.ws[1] = footprint(src, tmax); o.n_ws = 2; }
        }
    }
    return POLYDL_OK;
}

}  // namespace polydl
