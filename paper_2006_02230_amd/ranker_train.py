"""Train the pairwise network of the learned ranking (section "DNN-based ranking algorithm") on
measured sweeps of this library's own convolution variants, and report how its picks compare.

    python bench.py --batch 32 --sweep --sweep-out n32.json ...          (on the GPU: times every variant)
    python -m paper_2006_02230_amd.ranker_train --import-sweeps n16.json n32.json n64.json n128.json
    python -m paper_2006_02230_amd.ranker_train --train --report report.md

--import-sweeps  packs sweep files into ranker_data/conv_fp32_sweeps.json (shape, variant, microseconds).
--train          fits the network and writes ranker_params.txt, the file ranker_load() reads.
--report FILE    evaluates the parameters on disk and writes a markdown summary.
--sizes-only     the paper's own inputs: the three times are withheld (set to 0) from training and
                 evaluation; nothing is written, the figures are printed (with --train).

Following the experimental set-up section of the paper, 70 % of the code versions (drawn at random,
seeded) form the training set and one network serves all problems.  A training example is an
ordered pair of variants of the same problem, its label which of the two ran faster; pairs
closer than --margin (relative) are left out of training.  Statistics and their normalisation are
those of polydl_ranker_stats_conv2d / polydl_ranker_play; tournaments are played by the library.
The forward and backward pass used for fitting are written out here with numpy.
"""
import argparse
import glob
import json
import os
import time

import numpy as np

from . import binding as P

HERE = os.path.dirname(os.path.abspath(__file__))
DATA = os.path.join(HERE, "ranker_data", "conv_fp32_sweeps.json")
CFG_FIELDS = ["bm", "bn", "bk", "wm", "wn", "split_k", "layout", "raster", "algo", "cb"]
WIDTHS = [2 * P.RANKER_STATS, 64, 32, 16, 8, 2]
ACTS = ["relu", "relu", "softsign", "relu", "softmax"]
N_SIZES = 5


def import_sweeps(paths, out_path=DATA):
    problems = []
    for path in paths:
        for layer in json.load(open(path)):
            rows = [[c["cfg"][f] for f in CFG_FIELDS] + [c["us"]] for c in layer["candidates"]]
            problems.append({"shape": layer["shape"], "rows": rows})
    os.makedirs(os.path.dirname(out_path), exist_ok=True)
    with open(out_path, "w") as f:
        f.write('{"fields": %s,\n "problems": [\n' % json.dumps(CFG_FIELDS + ["us"]))
        f.write(",\n".join("  " + json.dumps(p, separators=(",", ":")) for p in problems))
        f.write("\n ]}\n")
    return len(problems), sum(len(p["rows"]) for p in problems)


def load_table(path=DATA, sizes_only=False):
    """Arrays over all measured variants: problem index, microseconds, model prediction, statistics."""
    data = json.load(open(path))
    assert data["fields"] == CFG_FIELDS + ["us"]
    group, us, pred, stats, cfgs, shapes = [], [], [], [], [], []
    for g, prob in enumerate(data["problems"]):
        shape = tuple(prob["shape"])
        shapes.append(shape)
        for row in prob["rows"]:
            cfg = P.TileCfg(*row[:len(CFG_FIELDS)])
            try:
                rep = P.model_conv2d(shape, cfg)
            except P.PolydlError:
                continue          # a variant the library no longer ranks for this problem
            group.append(g)
            us.append(row[-1])
            pred.append(rep.predicted_us)
            stats.append(P.ranker_stats_conv2d(shape, cfg))
            cfgs.append(cfg)
    stats = np.array(stats, dtype=np.float64)
    if sizes_only:
        stats[:, N_SIZES:] = 0.0
    return np.array(group), np.array(us, dtype=np.float64), np.array(pred), stats, cfgs, shapes


def split_mask(n, seed):
    """True = training variant (70 %)."""
    return np.random.default_rng(seed).random(n) < 0.7


def ordered_pairs(group, select):
    I, J = [], []
    for g in np.unique(group):
        idx = np.where((group == g) & select)[0]
        a, b = np.meshgrid(idx, idx, indexing="ij")
        keep = a != b
        I.append(a[keep])
        J.append(b[keep])
    return np.concatenate(I), np.concatenate(J)


def network_inputs(stats, I, J):
    a, b = stats[I], stats[J]
    size = a[:, :N_SIZES].sum(1) + b[:, :N_SIZES].sum(1)
    tim = a[:, N_SIZES:].sum(1) + b[:, N_SIZES:].sum(1)
    size[size == 0] = 1.0
    tim[tim == 0] = 1.0
    return np.concatenate([a[:, :N_SIZES] / size[:, None], a[:, N_SIZES:] / tim[:, None],
                           b[:, :N_SIZES] / size[:, None], b[:, N_SIZES:] / tim[:, None]], axis=1)


def forward(layers, X, keep=False):
    h, cache = X, []
    for (W, b), act in zip(layers, ACTS):
        z = h @ W.T + b
        cache.append((h, z))
        if act == "relu":
            h = np.maximum(z, 0)
        elif act == "softsign":
            h = z / (1 + np.abs(z))
        else:
            e = np.exp(z - z.max(1, keepdims=True))
            h = e / e.sum(1, keepdims=True)
    return (h, cache) if keep else h


def loss_and_gradients(layers, X, Y):
    p, cache = forward(layers, X, keep=True)
    d = (p - Y) / len(X)                      # softmax with cross-entropy
    grads = [None] * len(layers)
    for k in range(len(layers) - 1, -1, -1):
        h, z = cache[k]
        if ACTS[k] == "relu":
            d = d * (z > 0)
        elif ACTS[k] == "softsign":
            d = d / (1 + np.abs(z)) ** 2
        grads[k] = (d.T @ h, d.sum(0))
        d = d @ layers[k][0]
    return -np.mean(np.sum(Y * np.log(p + 1e-300), axis=1)), grads


def flatten(layers):
    return np.concatenate([np.concatenate([W.ravel(), b]) for W, b in layers])


def unflatten(flat):
    layers, at = [], 0
    for n_in, n_out in zip(WIDTHS[:-1], WIDTHS[1:]):
        W = np.array(flat[at:at + n_in * n_out]).reshape(n_out, n_in)
        b = np.array(flat[at + n_in * n_out:at + n_in * n_out + n_out])
        layers.append((W, b))
        at += n_in * n_out + n_out
    return layers


def train(table, seed=0, epochs=30, batch=4096, margin=0.01, log=print):
    group, us, _, stats, _, _ = table
    rng = np.random.default_rng(seed + 1)
    I, J = ordered_pairs(group, split_mask(len(us), seed))
    apart = np.abs(np.log(us[I] / us[J])) > margin
    I, J = I[apart], J[apart]
    X = network_inputs(stats, I, J)
    Y = np.stack([us[I] < us[J], us[I] >= us[J]], axis=1).astype(np.float64)
    log("training pairs: %d" % len(X))
    layers = [(rng.normal(0, np.sqrt(2.0 / i), (o, i)), np.zeros(o)) for i, o in zip(WIDTHS[:-1], WIDTHS[1:])]
    m = [[np.zeros_like(W), np.zeros_like(b)] for W, b in layers]
    v = [[np.zeros_like(W), np.zeros_like(b)] for W, b in layers]
    step, t0 = 0, time.time()
    for ep in range(epochs):
        lr = 1e-3 if ep < 0.6 * epochs else (3e-4 if ep < 0.85 * epochs else 1e-4)
        perm = rng.permutation(len(X))
        total, count = 0.0, 0
        for s in range(0, len(X), batch):
            sel = perm[s:s + batch]
            loss, grads = loss_and_gradients(layers, X[sel], Y[sel])
            total, count, step = total + loss, count + 1, step + 1
            for k in range(len(layers)):
                new = []
                for q in range(2):          # Adam
                    m[k][q] = 0.9 * m[k][q] + 0.1 * grads[k][q]
                    v[k][q] = 0.999 * v[k][q] + 0.001 * grads[k][q] ** 2
                    mh, vh = m[k][q] / (1 - 0.9 ** step), v[k][q] / (1 - 0.999 ** step)
                    new.append(layers[k][q] - lr * mh / (np.sqrt(vh) + 1e-8))
                layers[k] = tuple(new)
        log("epoch %d: loss %.4f (%.0f s)" % (ep + 1, total / count, time.time() - t0))
    return flatten(layers)


def write_params(flat, path, note):
    with open(path, "w") as f:
        f.write("# Parameters of the pairwise ranking network: per layer W[out][in] row-major, then b[out];\n")
        f.write("# layers %s.  Written by paper_2006_02230_amd/ranker_train.py.\n" % "-".join(str(w) for w in WIDTHS))
        for line in note:
            f.write("# %s\n" % line)
        for x in flat:
            f.write("%.17g\n" % x)


def read_params(path):
    with open(path) as f:
        return [float(l) for l in f if l.strip() and not l.startswith("#")]


def evaluate(table, flat, seed=0, theta=0.6):
    """Loads the parameters into the library, which plays the tournaments.  Returns a dict of figures
    and per-problem rows."""
    group, us, pred, stats, cfgs, shapes = table
    train_mask = split_mask(len(us), seed)
    P.ranker_set_params(flat)
    layers = unflatten(flat)
    out = {"rows": []}
    for name, sel in (("train", train_mask), ("held_out", ~train_mask)):
        I, J = ordered_pairs(group, sel)
        apart = np.abs(np.log(us[I] / us[J])) > 0.01
        p = forward(layers, network_inputs(stats, I[apart], J[apart]))
        out["pair_accuracy_" + name] = float(np.mean((p[:, 0] > 0.5) == (us[I[apart]] < us[J[apart]])))
        out["pairs_" + name] = int(apart.sum())
    for g in np.unique(group):
        everything = np.where(group == g)[0]
        held = np.where((group == g) & ~train_mask)[0]
        row = {"shape": list(shapes[g]), "variants": len(everything), "held_out": len(held)}
        for key, idx in (("all", everything), ("held", held)):
            wins, order = P.ranker_tournament([list(stats[i]) for i in idx], theta)
            best = us[idx].min()
            top = max(1, len(idx) // 20)
            row["learned_" + key] = float(us[idx[order[0]]] / best)
            row["learned_top5pct_" + key] = float(us[idx[order[:top]]].min() / best)
            row["model_" + key] = float(us[idx[np.argmin(pred[idx])]] / best)
            if key == "all":
                row["learned_cfg"] = cfgs[idx[order[0]]].as_dict()
                row["learned_us"] = float(us[idx[order[0]]])
                row["best_us"] = float(best)
                row["wins"] = int(wins[order[0]])
        out["rows"].append(row)
    for k in ("learned_all", "model_all", "learned_held", "model_held", "learned_top5pct_all"):
        vals = np.array([r[k] for r in out["rows"]])
        out["mean_" + k], out["max_" + k] = float(vals.mean()), float(vals.max())
    return out


def write_report(res, path, command, note=""):
    def name(c):
        if c["algo"] == 2:
            return "pointwise 32x64"
        if c["algo"] == 1:
            return "patch %dx%d/%dx%d cb %d split %d" % (c["bm"], c["bn"], c["wm"], c["wn"], c["cb"], c["split_k"])
        return "gather %dx%dx%d/%dx%d split %d%s" % (c["bm"], c["bn"], c["bk"], c["wm"], c["wn"], c["split_k"],
                                                     (" tail" if c["raster"] >= 2 else "") +
                                                     (" tap" if c["layout"] == 2 else ""))
    o = ["# Learned ranking (pairwise network + tournament) against the sweep: fp32 convolution suite\n",
         "Commands (the sweeps on the MI355X, the rest on the host):\n", command, ""]
    o.append("Pairs of variants of one problem more than 1 %% apart, ordered correctly by the network: "
             "%.1f %% of %d training pairs, %.1f %% of %d pairs among the held-out 30 %% of variants.\n"
             % (100 * res["pair_accuracy_train"], res["pairs_train"], 100 * res["pair_accuracy_held_out"],
                res["pairs_held_out"]))
    o.append("Time of the tournament's winner / time of the fastest variant (1.000 = the sweep's best), next to the "
             "same ratio for the reuse model's pick; `all` = tournament among every measured variant of the problem, "
             "`held-out` = among the variants the training never saw.\n")
    o.append("| (N,C,H,W,K,R,S,stride,pad) | variants | learned pick | learned / best | model / best | best of learned top 5 % / best | held-out variants | learned / best (held-out) | model / best (held-out) |")
    o.append("|---|---|---|---|---|---|---|---|---|")
    for r in res["rows"]:
        o.append("| %s | %d | %s | %.3f | %.3f | %.3f | %d | %.3f | %.3f |"
                 % (tuple(r["shape"]), r["variants"], name(r["learned_cfg"]), r["learned_all"], r["model_all"],
                    r["learned_top5pct_all"], r["held_out"], r["learned_held"], r["model_held"]))
    o.append("\nMean (max) over the %d problems: learned %.3f (%.3f), reuse model %.3f (%.3f); held-out: learned %.3f "
             "(%.3f), reuse model %.3f (%.3f); best of the learned top 5 %%: %.3f (%.3f)."
             % (len(res["rows"]), res["mean_learned_all"], res["max_learned_all"], res["mean_model_all"],
                res["max_model_all"], res["mean_learned_held"], res["max_learned_held"], res["mean_model_held"],
                res["max_model_held"], res["mean_learned_top5pct_all"], res["max_learned_top5pct_all"]))
    if note:
        o.append("\n" + note)
    with open(path, "w") as f:
        f.write("\n".join(o) + "\n")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--import-sweeps", nargs="+", default=[])
    ap.add_argument("--train", action="store_true")
    ap.add_argument("--report", default="")
    ap.add_argument("--report-command",
                    default="    python bench.py --batch B --sweep --sweep-out nB.json --no-cpu --no-sgemm --no-bf16 --no-fusion --no-cold   (B = 16, 32, 64, 128)\n"
                            "    python -m paper_2006_02230_amd.ranker_train --import-sweeps n16.json n32.json n64.json n128.json\n"
                            "    python -m paper_2006_02230_amd.ranker_train --train --report profiles/conv_suite_fp32_learned_ranking.md\n",
                    help="text of the commands, quoted in the report")
    ap.add_argument("--report-note", default="", help="a closing paragraph for the report")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--epochs", type=int, default=30)
    ap.add_argument("--margin", type=float, default=0.01)
    ap.add_argument("--sizes-only", action="store_true")
    args = ap.parse_args()
    if args.import_sweeps:
        files = [f for pat in args.import_sweeps for f in sorted(glob.glob(pat))]
        print("packed %d problems, %d measured variants" % import_sweeps(files))
    if args.sizes_only:
        table = load_table(sizes_only=True)
        flat = train(table, args.seed, args.epochs, margin=args.margin)
        res = evaluate(table, flat, args.seed)
        print(json.dumps({k: v for k, v in res.items() if k != "rows"}))
        return
    table = None
    if args.train:
        table = load_table()
        flat = train(table, args.seed, args.epochs, margin=args.margin)
        write_params(flat, P.RANKER_PARAMS_PATH,
                     ["Trained on 70 %% of %d measured variants of %d problems (seed %d, %d epochs)."
                      % (len(table[1]), len(table[5]), args.seed, args.epochs)])
    if args.report:
        table = table or load_table()
        res = evaluate(table, read_params(P.RANKER_PARAMS_PATH), args.seed)
        write_report(res, args.report, args.report_command, args.report_note)
        print(json.dumps({k: v for k, v in res.items() if k != "rows"}))


if __name__ == "__main__":
    main()
