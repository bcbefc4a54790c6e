#!/usr/bin/env python3
"""Which hardware counters explain run time across configurations: the paper's counter-selection
step (Section 3.2.3, Eq. 1), applied to this library's own kernels.

Eq. 1 asks for a sparse weight vector a with  min ||t - D a||_2^2  subject to  ||a||_0 <= kappa,
where D (N runs x C counters) holds counter values and t (N) the run times.  The paper solves it
with Ensemble Orthogonal Matching Pursuit: a greedy pursuit that, at each step, does not take the
single most correlated counter but keeps the top tau candidates and samples one of them with
probability proportional to its correlation strength; the pursuit is repeated to form an ensemble,
and the top k (= 5 in the paper) counters are reported.

Readings where the paper is silent: columns of D are centred and scaled to unit norm and t is
centred (counters differ by orders of magnitude); constant columns are dropped; "correlation
strength" is |d_j . r| with r the current residual; after each pick the weights on the chosen
columns are re-fitted by least squares (the "orthogonal" in OMP); a counter's importance is its
mean, over the ensemble, of |weight| on the unit-norm column (so a counter never picked scores 0);
kappa, tau and the ensemble size are parameters (the paper gives no values).  The random numbers
are an input: `draws[e][s]` in [0, 1) decides the pick of ensemble member e at step s, so a run is
reproducible and testable.  This is CPU-side analysis code (numpy); no GPU is involved.
"""
import argparse
import csv
import glob
import os
import sys

import numpy as np


def standardise(D, t):
    """Centre t; centre the columns of D and scale them to unit norm; drop constant columns.
    Returns (Dn, tn, kept column indices)."""
    D = np.asarray(D, dtype=np.float64)
    t = np.asarray(t, dtype=np.float64)
    Dc = D - D.mean(axis=0)
    norms = np.sqrt((Dc * Dc).sum(axis=0))
    keep = np.nonzero(norms > 1e-12 * max(1.0, np.abs(D).max()))[0]
    return Dc[:, keep] / norms[keep], t - t.mean(), keep


def pursuit(Dn, tn, kappa, tau, draws):
    """One ensemble member on standardised data.  Returns (support in pick order, weights on it)."""
    n, c = Dn.shape
    support = []
    residual = tn.copy()
    weights = np.zeros(0)
    for step in range(min(kappa, c, n)):
        strength = np.abs(Dn.T @ residual)
        strength[support] = -1.0
        if strength.max() <= 1e-14 * max(1.0, np.linalg.norm(tn)):
            break                                   # nothing left to explain
        order = np.argsort(-strength, kind="stable")[:tau]
        order = order[strength[order] > 0]
        p = strength[order] / strength[order].sum()
        pick = int(order[min(np.searchsorted(np.cumsum(p), draws[step], side="right"), len(order) - 1)])
        support.append(pick)
        weights, *_ = np.linalg.lstsq(Dn[:, support], tn, rcond=None)
        residual = tn - Dn[:, support] @ weights
    return support, weights


def ensemble_omp(D, t, kappa, tau, draws):
    """draws: array (members, >= kappa) of numbers in [0, 1).  Returns a dict with
    importance (per original column), members (list of (support, weights, residual norm)) and kept."""
    Dn, tn, keep = standardise(D, t)
    draws = np.asarray(draws, dtype=np.float64)
    importance = np.zeros(np.asarray(D).shape[1])
    members = []
    for e in range(draws.shape[0]):
        support, weights = pursuit(Dn, tn, kappa, tau, draws[e])
        for j, w in zip(support, weights):
            importance[keep[j]] += abs(w) / draws.shape[0]
        res = tn - (Dn[:, support] @ weights if support else 0.0)
        members.append(([int(keep[j]) for j in support], weights, float(np.linalg.norm(res))))
    return {"importance": importance, "members": members, "kept": keep, "target_norm": float(np.linalg.norm(tn))}


def top_k(result, names, k=5):
    order = np.argsort(-result["importance"], kind="stable")
    return [(names[j], float(result["importance"][j])) for j in order[:k] if result["importance"][j] > 0]


# ---------------------------------------------------------------- rocprofv3 front end

def matrix_from_rocprof(root):
    """Rows = kernel dispatch groups (kernel name x grid size), columns = counters; the target is the
    mean kernel duration from the kernel trace.  Only rows present in every file are used."""
    per = {}
    for path in sorted(glob.glob(os.path.join(root, "**", "*_counter_collection.csv"), recursive=True)):
        with open(path) as f:
            for row in csv.DictReader(f):
                key = (row["Kernel_Name"], row["Grid_Size"])
                per.setdefault(key, {}).setdefault(row["Counter_Name"], []).append(float(row["Counter_Value"]))
    dur = {}
    for path in sorted(glob.glob(os.path.join(root, "**", "*_kernel_trace.csv"), recursive=True)):
        with open(path) as f:
            for row in csv.DictReader(f):
                grid = row.get("Grid_Size") or str(int(row["Grid_Size_X"]) * int(row.get("Grid_Size_Y", 1)) * int(row.get("Grid_Size_Z", 1)))
                dur.setdefault((row["Kernel_Name"], grid), []).append(int(row["End_Timestamp"]) - int(row["Start_Timestamp"]))
    keys = sorted(k for k in per if k in dur)
    counters = sorted(set.intersection(*(set(per[k]) for k in keys))) if keys else []
    D = np.array([[np.mean(per[k][c]) for c in counters] for k in keys])
    t = np.array([np.mean(dur[k]) for k in keys])
    return keys, counters, D, t


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("dir", help="directory with rocprofv3 CSV output (kernel trace and counter collections)")
    ap.add_argument("--kappa", type=int, default=5)
    ap.add_argument("--tau", type=int, default=3)
    ap.add_argument("--members", type=int, default=200)
    ap.add_argument("--seed", type=int, default=42)
    ap.add_argument("--k", type=int, default=5)
    ap.add_argument("--kernel-filter", default="", help="only rows whose kernel name contains this text")
    args = ap.parse_args()
    keys, counters, D, t = matrix_from_rocprof(args.dir)
    rows = [i for i, k in enumerate(keys) if args.kernel_filter in k[0]]
    if len(rows) < 3 or not counters:
        print("not enough rows/counters in %s" % args.dir, file=sys.stderr)
        return 1
    D, t = D[rows], t[rows]
    draws = np.random.RandomState(args.seed).random_sample((args.members, args.kappa))
    res = ensemble_omp(D, t, args.kappa, args.tau, draws)
    print("%d runs x %d counters; kappa %d, tau %d, %d ensemble members" % (len(rows), len(counters), args.kappa, args.tau, args.members))
    print("mean residual / ||t - mean||: %.3f" % (np.mean([m[2] for m in res["members"]]) / res["target_norm"]))
    for name, score in top_k(res, counters, args.k):
        print("  %-44s %.3f" % (name, score))
    return 0


if __name__ == "__main__":
    sys.exit(main())
