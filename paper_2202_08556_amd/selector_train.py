"""Train the data-aware selector (paper Sec. 5) from sweep timings and compile it into the library.

    D=paper_2202_08556_amd/selector_data
    python -m paper_2202_08556_amd.selector_train \
        --train $D/train.jsonl $D/families.jsonl $D/train_N2_N4.jsonl --eval $D/eval.jsonl \
        --also-score $D/odd.jsonl $D/eval_N2_N4.jsonl $D/odd_N2_N4.jsonl

(train_N2_N4.jsonl = the train and families sweeps run again with --ns 2,4; eval_N2_N4 and odd_N2_N4
likewise for the two never-trained-on sets.)

The paper trains a gradient-boosted tree classifier (LightGBM) on `nnz, mat_size, std_row, N`
(Table 2).  LightGBM is not available here, so the model is a small gradient-boosted forest built
from scikit-learn regression trees: every tree predicts, for all 8 algorithms at once, the log of
the slow-down against the best algorithm on that input (squared loss, shrinkage), and the selector
picks the algorithm with the smallest predicted slow-down.  Training on slow-downs instead of
arg-min labels makes near-ties harmless.  The model is written as JSON (selector_model.json) and
as C tables (csrc/selector_model.inc) that da_spmm_select walks.

Figure of merit (Fig. 1 caption, Sec. 5.1): geometric mean over inputs of time(best)/time(chosen).
"""
from __future__ import annotations

import argparse
import json
import os

import numpy as np

PKG = os.path.dirname(os.path.abspath(__file__))
MODEL_JSON = os.path.join(PKG, "selector_model.json")
MODEL_INC = os.path.join(PKG, "csrc", "selector_model.inc")
ALGOS = ["RB+RM+SR", "RB+RM+PR", "RB+CM+SR", "RB+CM+PR", "EB+RM+SR", "EB+RM+PR", "EB+CM+SR", "EB+CM+PR"]
NUM_FEATURES = 7


def feature_vector(f: dict) -> np.ndarray:
    """Must match the vector built in csrc/da_spmm_select.cpp."""
    lg = lambda x: np.log2(max(float(x), 1.0))
    mean = float(f["row_nnz_mean"])
    mx = float(f["row_nnz_max"])
    return np.array([
        lg(f["rows"]), lg(f["nnz"]), np.log2(mean + 1.0),
        (float(f["row_nnz_std"]) / mean) if mean > 0 else 0.0,
        np.log2(mx + 1.0), lg(f["N"]),
        np.log2(mx / mean + 1.0) if mean > 0 else 0.0,
    ])


def load(paths):
    X, T, meta = [], [], []
    for p in paths:
        for line in open(p):
            r = json.loads(line)
            X.append(feature_vector(r["features"]))
            T.append(r["times_us"])
            meta.append((r["set"], r["name"], r["N"]))
    return np.array(X), np.array(T, dtype=np.float64), meta


def normalized_performance(T, chosen):
    best = T.min(axis=1)
    return float(np.exp(np.mean(np.log(best / T[np.arange(len(T)), chosen]))))


# ------------------------------------------------------------------------------------------
# model = list of trees; tree = dict(feature[], threshold[], left[], right[], value[][8])
# ------------------------------------------------------------------------------------------
def walk(model, x):
    score = np.zeros(8)
    for t in model["trees"]:
        i = 0
        while t["feature"][i] >= 0:
            i = t["left"][i] if x[t["feature"][i]] <= t["threshold"][i] else t["right"][i]
        score += np.array(t["value"][i])
    return int(np.argmax(score))           # ties -> lowest id, as in the C code


def predict(model, X):
    return np.array([walk(model, x) for x in X])


def fit(X, T, Xval=None, Tval=None, n_trees=60, depth=5, lr=0.15, min_leaf=4, seed=0, slack=0.0):
    from sklearn.tree import DecisionTreeRegressor
    Y = np.log(T / T.min(axis=1, keepdims=True))          # log slow-down, >= 0
    Y = np.minimum(Y, np.log(50.0))                        # a 50x loss is as bad as it needs to be
    base = Y.mean(axis=0)
    trees = [dict(feature=[-1], threshold=[0.0], left=[0], right=[0], value=[(-base).tolist()])]
    F = np.tile(base, (len(X), 1))
    scores = []
    rng = np.random.RandomState(seed)
    for it in range(n_trees):
        reg = DecisionTreeRegressor(max_depth=depth, min_samples_leaf=min_leaf, random_state=rng.randint(1 << 30))
        reg.fit(X, Y - F)
        tr = reg.tree_
        F += lr * reg.predict(X)
        trees.append(dict(feature=[int(f) if f >= 0 else -1 for f in tr.feature],
                          threshold=[float(t) for t in tr.threshold],
                          left=[int(c) for c in tr.children_left], right=[int(c) for c in tr.children_right],
                          value=[(-lr * tr.value[i, :, 0]).tolist() for i in range(tr.node_count)]))
        if Xval is not None:
            scores.append(normalized_performance(Tval, predict(dict(trees=trees), Xval)))
    if Xval is None:
        return dict(trees=trees)
    # the smallest forest whose validation score is within `slack` of the best one: the last few
    # thousandths cost most of the trees
    keep = next(i for i, sc in enumerate(scores) if sc >= max(scores) - slack)
    return dict(trees=trees[:keep + 2], validation_score=scores[keep])


def write_inc(model, path, note):
    nodes, leaves, roots = [], [], []
    for t in model["trees"]:
        off = len(nodes)
        roots.append(off)
        for i in range(len(t["feature"])):
            if t["feature"][i] < 0:
                nodes.append((-1, 0.0, len(leaves), 0))
                leaves.append(t["value"][i])
            else:
                nodes.append((t["feature"][i], t["threshold"][i], off + t["left"][i], off + t["right"][i]))
    with open(path, "w") as f:
        f.write("// Selector model: a gradient-boosted forest of regression trees over the feature vector built in\n"
                "// da_spmm_select.cpp; a leaf holds minus the predicted log slow-down of each algorithm and the\n"
                "// selector takes the arg-max of the summed leaves.  Written by selector_train.py -- do not edit.\n")
        f.write(f"// {note}\n")
        f.write("// Node layout: feature < 0 marks a leaf whose `left` field indexes kLeafScores.\n")
        f.write(f"static const int kNumTrees = {len(roots)};\n")
        f.write(f"static const int kTreeRoot[{len(roots)}] = {{" + ", ".join(map(str, roots)) + "};\n")
        f.write(f"static const SelNode kNodes[{len(nodes)}] = {{\n")
        for n in nodes:
            f.write(f"    {{{n[0]}, {n[1]!r}, {n[2]}, {n[3]}}},\n")
        f.write("};\n")
        f.write(f"static const float kLeafScores[{len(leaves)}][8] = {{\n")
        for v in leaves:
            f.write("    {" + ", ".join(f"{x:.6g}f" for x in v) + "},\n")
        f.write("};\n")


def report(name, T, chosen, lines):
    lines.append(f"{name}: {len(T)} inputs; selector normalised performance {normalized_performance(T, chosen):.4f}")
    for a in range(8):
        lines.append(f"    static {ALGOS[a]}: {normalized_performance(T, np.full(len(T), a)):.4f}"
                     f"   (best on {int(np.sum(T.argmin(axis=1) == a))} inputs, chosen on {int(np.sum(chosen == a))})")
    loss = T[np.arange(len(T)), chosen] / T.min(axis=1)
    lines.append(f"    worst slow-down of the selector {loss.max():.2f}x; inputs with > 1.25x: {int(np.sum(loss > 1.25))}")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--train", nargs="+", required=True)
    ap.add_argument("--eval", nargs="+", required=True)
    ap.add_argument("--also-score", nargs="*", default=[],
                    help="further never-trained-on sets, scored with the shipped model and reported one by one")
    ap.add_argument("--trees", type=int, default=240)
    ap.add_argument("--depth", type=int, nargs="+", default=[4, 5, 6],
                    help="tree depths to try; the held-out tenth of the training sets picks one")
    ap.add_argument("--slack", type=float, default=0.003,
                    help="take the smallest forest whose validation score is within this of the best")
    ap.add_argument("--report", default=os.path.join(PKG, "selector_data", "report.txt"))
    ap.add_argument("--no-write", action="store_true")
    args = ap.parse_args()
    Xtr, Ttr, _ = load(args.train)
    Xev, Tev, _ = load(args.eval)
    lines = []
    # (a) the paper's protocol on the pooled data: 40 % train, 10 % validation, 50 % test
    Xall, Tall = np.vstack([Xtr, Xev]), np.vstack([Ttr, Tev])
    perm = np.random.RandomState(1).permutation(len(Xall))
    n4, n5 = int(0.4 * len(perm)), int(0.5 * len(perm))
    itr, iva, ite = perm[:n4], perm[n4:n5], perm[n5:]
    def fit_best(X, T, Xv, Tv):
        """One model per depth; the validation part picks the depth (and, inside fit, the number of trees)."""
        models = [fit(X, T, Xv, Tv, n_trees=args.trees, depth=d, slack=args.slack) for d in args.depth]
        top = max(mm["validation_score"] for mm in models)
        best = min((i for i in range(len(models)) if models[i]["validation_score"] >= top - args.slack),
                   key=lambda i: len(models[i]["trees"]))
        models[best]["depth"] = args.depth[best]
        return models[best]

    m = fit_best(Xall[itr], Tall[itr], Xall[iva], Tall[iva])
    report("pooled 40/10/50 split, test half (Sec. 5.2 protocol)", Tall[ite], predict(m, Xall[ite]), lines)
    # (b) shipped model: trained on the training sets only (10 % of them held out to pick the
    #     number of trees), scored on the never-seen evaluation sweep
    perm = np.random.RandomState(2).permutation(len(Xtr))
    nv = max(1, len(perm) // 10)
    model = fit_best(Xtr[perm[nv:]], Ttr[perm[nv:]], Xtr[perm[:nv]], Ttr[perm[:nv]])
    report("evaluation sweep (64 matrices x 6 N, disjoint seeds from training)", Tev, predict(model, Xev), lines)
    report("training sets (resubstitution)", Ttr, predict(model, Xtr), lines)
    for p in args.also_score:
        Xo, To, _ = load([p])
        report(f"{os.path.basename(p)} (never trained on)", To, predict(model, Xo), lines)
    # (c) feature ablation with the paper's protocol: its own four features (Table 2) against the
    #     extended set compiled into the library.  Columns of the feature vector: 0 log2 rows,
    #     1 log2 nnz, 2 log2(mean+1), 3 std/mean, 4 log2(max+1), 5 log2 N, 6 log2(max/mean+1).
    std_abs = Xall[:, 3] * (2.0 ** Xall[:, 2] - 1.0)                 # std of the row length itself
    paper4 = np.column_stack([Xall[:, 1], Xall[:, 0], np.log2(std_abs + 1.0), Xall[:, 5]])
    for label, Xf in (("paper's 4 features (nnz, mat_size, std_row, N)", paper4),
                      ("without the dispersion features (rows, nnz, mean, N)", Xall[:, [0, 1, 2, 5]]),
                      ("all 7 features", Xall)):
        mm = fit_best(Xf[itr], Tall[itr], Xf[iva], Tall[iva])
        lines.append(f"ablation, pooled 40/10/50 test half, {label}: "
                     f"{normalized_performance(Tall[ite], predict(mm, Xf[ite])):.4f}")
    lines.append(f"model: {len(model['trees'])} trees, depth <= {model['depth']} (picked among {args.depth} and up to "
                 f"{args.trees} trees by the held-out tenth of the training sets); "
                 f"trained on {len(Xtr)} inputs from {', '.join(os.path.basename(p) for p in args.train)}")
    text = "\n".join(lines)
    print(text)
    if not args.no_write:
        json.dump(model, open(MODEL_JSON, "w"))
        write_inc(model, MODEL_INC, f"trained on {len(Xtr)} inputs; evaluation-sweep normalised performance "
                                    f"{normalized_performance(Tev, predict(model, Xev)):.4f}")
        os.makedirs(os.path.dirname(args.report), exist_ok=True)
        open(args.report, "w").write(text + "\n")


if __name__ == "__main__":
    main()
