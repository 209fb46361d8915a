"""Pairwise network and tournament of the paper's learned ranking.  TEST INFRASTRUCTURE ONLY.

Section "DNN-based ranking algorithm": a feed-forward network looks at the statistics of two code
variants and says which of the two runs faster; every variant plays every other one and the
variants are ranked by the number of games won.

Network (that section and its architecture figure): four hidden layers of 64, 32, 16 and 8 units
with relu, relu, softsign and relu, then two output units under a softmax.  An output above the
threshold theta (0.6 in the paper) counts as 1: the first unit firing means the first variant
wins, the second unit the second variant; neither firing is a draw.

Input (same section): the statistics of the two variants divided by their sum over BOTH variants,
so that the network sees which of the two has the larger working sets.  Readings taken here,
where the paper leaves room:
  * a variant carries STATS = 8 statistics: the five numbers of algorithm "Compute working set
    sizes w.r.t cache sizes" (bytes reused from each of four levels, bytes reused from memory),
    then three times in microseconds (matrix-unit time, memory time, fixed cost).  The paper has
    the first kind only.  Each kind is divided by the sum of that kind over both variants, i.e.
    the paper's rule applied once per unit of measurement; a kind whose sum is 0 stays 0;
  * the input vector is [variant 1: 5 sizes, 3 times; variant 2: 5 sizes, 3 times];
  * "plays every other variant" is taken as every ORDERED pair (i first, j second), i != j, since
    the network need not be symmetric in its two halves: n*(n-1) games;
  * equal numbers of wins keep the order the variants were given in.

Parameters are one flat float64 vector: for each of the five layers the weight matrix W[out][in],
row-major, then the bias b[out].

Everything is float64 and written as plain loops over units.  Pinned by
tests/test_oracle_ranker.py: all-zero parameters (a draw everywhere), a network built by hand whose
outputs have closed forms worked out on paper, and tournaments whose ranking is known.
"""
import math

STATS = 8
N_SIZES = 5
LAYERS = [(2 * STATS, 64, "relu"), (64, 32, "relu"), (32, 16, "softsign"), (16, 8, "relu"),
          (8, 2, "softmax")]
NUM_PARAMS = sum(i * o + o for i, o, _ in LAYERS)


def normalise(s1, s2):
    """The 16 network inputs from the statistics of the first and of the second variant."""
    if len(s1) != STATS or len(s2) != STATS:
        raise ValueError("a variant has %d statistics" % STATS)
    size_sum = sum(s1[:N_SIZES]) + sum(s2[:N_SIZES])
    time_sum = sum(s1[N_SIZES:]) + sum(s2[N_SIZES:])
    x = []
    for s in (s1, s2):
        for k in range(STATS):
            total = size_sum if k < N_SIZES else time_sum
            x.append(s[k] / total if total > 0 else 0.0)
    return x


def forward(params, x):
    """The two softmax outputs for one input vector."""
    if len(params) != NUM_PARAMS:
        raise ValueError("expected %d parameters" % NUM_PARAMS)
    h = [float(v) for v in x]
    at = 0
    for n_in, n_out, act in LAYERS:
        if len(h) != n_in:
            raise ValueError("layer input size")
        z = []
        for o in range(n_out):
            acc = 0.0
            for i in range(n_in):
                acc += float(params[at + o * n_in + i]) * h[i]
            z.append(acc)
        at += n_in * n_out
        for o in range(n_out):
            z[o] += float(params[at + o])
        at += n_out
        if act == "relu":
            h = [v if v > 0 else 0.0 for v in z]
        elif act == "softsign":
            h = [v / (1.0 + abs(v)) for v in z]
        else:
            m = max(z)
            e = [math.exp(v - m) for v in z]
            h = [v / sum(e) for v in e]
    return h


def play(params, s1, s2, theta=0.6):
    """One game.  Returns (winner, probs): winner 1 or 2, or 0 for a draw."""
    p = forward(params, normalise(s1, s2))
    if p[0] > theta:
        return 1, p
    if p[1] > theta:
        return 2, p
    return 0, p


def tournament(params, stats, theta=0.6):
    """Every ordered pair plays once.  Returns (wins, order): games won per variant, and the
    variants' indices from most to fewest wins (equal wins: lower index first)."""
    n = len(stats)
    wins = [0] * n
    for i in range(n):
        for j in range(n):
            if i == j:
                continue
            w, _ = play(params, stats[i], stats[j], theta)
            if w == 1:
                wins[i] += 1
            elif w == 2:
                wins[j] += 1
    order = sorted(range(n), key=lambda i: (-wins[i], i))
    return wins, order
