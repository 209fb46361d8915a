"""Reuse analysis of the paper, by brute force.  TEST INFRASTRUCTURE ONLY.

working_sets()  follows algorithm "Compute working set sizes" (section "Working set size
computation") on a small loop nest given explicitly: instead of polyhedral sets it enumerates
every iteration, so it only serves tiny bounds.  For a dependence carried by sequential loops it
takes the lexicographically first source iteration, its first and last target iterations, and
counts the distinct array elements touched by all iterations from the source up to and including
that target (WS_min, WS_max).  For a dependence that spans iterations of a parallel loop it counts
the elements touched by the whole nest with the iterators outside the outermost parallel loop
held fixed (WS_par).

A dependence here is a pair of array references (source reference, target reference) to the same
array together with all pairs of iterations (I, I'), I before I', in which they touch the same
element.  Read/write kinds are not distinguished: the paper takes the union of RAR, RAW, WAR and
WAW dependences, and pairs of references with identical iteration pairs are merged, which gives
the three relations d1, d2, d3 the paper lists for matrix multiplication.

bucket_working_sets()  is algorithm "Compute working set sizes w.r.t cache sizes"; cost()  is
equation (1), with lat/bw taken as one weight per level.

Pinned by tests/test_oracle_reuse.py against the closed forms the paper prints for dependence d2
of the three-loop matrix multiplication (WS_min = 2K+3, WS_max = N*K+N+1).
"""
import itertools


def _iterations(extents):
    return list(itertools.product(*[range(e) for e in extents]))


def working_sets(loops, refs, parallel=()):
    """loops: [(name, extent)] outermost first (the schedule is the loop order);
    refs: [(array, fn)] with fn(iteration tuple) -> index tuple;  parallel: names of parallel loops.

    Returns a list of dicts, one per merged dependence:
      {"refs": [(src_ref, tgt_ref), ...], "parallel": bool, "ws": [sizes added to WS_all],
       "source": iteration, "min_target": iteration, "max_target": iteration}
    """
    names = [n for n, _ in loops]
    extents = [e for _, e in loops]
    its = _iterations(extents)                     # lexicographic = execution order
    order = {it: k for k, it in enumerate(its)}
    touched = {it: frozenset((a, f(it)) for a, f in refs) for it in its}

    def footprint(iter_subset):
        s = set()
        for it in iter_subset:
            s |= touched[it]
        return len(s)

    merged = {}
    for si, (sa, sf) in enumerate(refs):
        for ti, (ta, tf) in enumerate(refs):
            if sa != ta:
                continue
            by_elem = {}
            for it in its:
                by_elem.setdefault(tf(it), []).append(it)
            pairs = []
            for it in its:
                for it2 in by_elem.get(sf(it), ()):
                    if order[it2] > order[it]:
                        pairs.append((it, it2))
            if pairs:
                merged.setdefault(frozenset(pairs), []).append((si, ti))

    out = []
    par_idx = [names.index(p) for p in parallel]
    for pairs, rr in merged.items():
        spans_par = any(s[i] != t[i] for s, t in pairs for i in par_idx)
        if spans_par:
            ip = min(i for i in par_idx if any(s[i] != t[i] for s, t in pairs))
            src = min(s for s, _ in pairs)
            fixed = src[:ip]
            ws = footprint(it for it in its if it[:ip] == fixed)
            out.append({"refs": rr, "parallel": True, "ws": [ws], "source": src,
                        "min_target": None, "max_target": None})
        else:
            src = min(s for s, _ in pairs)
            targets = sorted(t for s, t in pairs if s == src)
            tmin, tmax = targets[0], targets[-1]
            lo = order[src]
            ws_min = footprint(its[lo:order[tmin] + 1])
            ws_max = footprint(its[lo:order[tmax] + 1])
            ws = [ws_min] if tmin == tmax else [ws_min, ws_max]
            out.append({"refs": rr, "parallel": False, "ws": ws, "source": src,
                        "min_target": tmin, "max_target": tmax})
    return out


def ws_all(deps):
    """The multiset WS_all: every size added by every dependence."""
    return sorted(w for d in deps for w in d["ws"])


def bucket_working_sets(ws, sizes):
    """Working set sizes per level and the memory working set size.  ws and sizes in the same
    unit.  Sorted ascending, each working set goes to the first (fastest) level where it still
    fits beside what was placed there before; what fits nowhere is added to memory."""
    levels = [0] * len(sizes)
    mem = 0
    for w in sorted(ws):
        for i, cap in enumerate(sizes):
            if w + levels[i] <= cap:
                levels[i] += w
                break
        else:
            mem += w
    return levels, mem


def cost(levels, mem, weights, mem_weight):
    """Equation (1): sum over levels of WS^Li * lat^Li/bw^Li plus WS^mem * lat^mem/bw^mem, the
    ratio lat/bw given as one weight per level.  Lower is better."""
    return sum(w * c for w, c in zip(levels, weights)) + mem * mem_weight


def matmul_nest(M, N, K):
    """The paper's running example: for i, j, k: C[i][j] += A[i][k] * B[k][j]."""
    loops = [("i", M), ("j", N), ("k", K)]
    refs = [("C", lambda it: (it[0], it[1])), ("A", lambda it: (it[0], it[2])),
            ("B", lambda it: (it[2], it[1]))]
    return loops, refs
