"""Approximation error of S^ against S on the paper's synthetic workload (Sec. 4.2, Tables 3-4),
computed with the CPU oracle only -- TEST INFRASTRUCTURE, like the rest of this package.

Workload: Q, K with independent U(0,1) entries, N = d = 64, scale 1, repeated `draws` times with
a fresh projection seed each; block size l (rows of a Q block) and group size G* as in the
tables. The paper does not say how its "percentage of the current error relative to the true
value" is aggregated, nor which column of a group is sampled; this module computes the
candidates side by side:

  readings of the error figure (each gives one number per experiment; min / max / mean are then
  taken over the experiments, which is how Tables 3-4 are laid out):
    elementwise   mean over the matrix of |S^ - S| / |S|
    signed_mean   | mean over the matrix of (S^ - S) / S |      (errors of opposite sign cancel)
    matrix_sum    | sum(S^ - S) | / sum(S)
    softmax       mean over the matrix of |P^ - P| / P, P = softmax(S / sqrt(d)) row-wise
  representative (which member of a group, in sorted order, is sampled): first, middle, last --
  obtained by rotating the members inside every group of the oracle's permutation, which
  leaves the fused sums unchanged.

Run `python -m oracle.error_study` for the full table (about a minute).
"""
import numpy as np

from . import lsh_group, params, scores

READINGS = ("elementwise", "signed_mean", "matrix_sum", "softmax")
PAPER_TABLE3 = {1: (4e-4, 3.45, 0.9), 2: (2e-3, 3.4, 0.87), 4: (2e-3, 3.4, 0.87), 8: (1e-3, 3.4, 0.87)}     # l -> (min, max, mean) %, G* = 2
PAPER_TABLE4 = {2: (2e-3, 3.4, 0.87), 4: (4e-2, 5.4, 1.73), 8: (7e-2, 9.25, 2.48), 16: (6e-3, 16.5, 4.96)}  # G* -> (min, max, mean) %, l = 2


def rotate_groups(perm, G, r):
    """Member r of every group (in sorted order) moves to the front: it becomes the sample."""
    d = perm.shape[-1]
    return np.roll(perm.reshape(-1, d // G, G), -r, axis=2).reshape(perm.shape).copy()


def experiment_errors(l, G, draws=100, N=64, d=64, representative="first", grouping="lsh", gray_mode=0, seed=0):
    """-> {reading: array of `draws` per-experiment errors (fractions, not percent)}."""
    rng = np.random.default_rng(seed)
    r = {"first": 0, "middle": G // 2, "last": G - 1}[representative]
    out = {k: [] for k in READINGS}
    for i in range(draws):
        q = rng.random((1, 1, N, d), dtype=np.float32)
        k = rng.random((1, 1, N, d), dtype=np.float32)
        p = params(1, 1, 1, N, d, l, d // G, lsh_seed=i, scale=1.0, gray_mode=gray_mode)
        if grouping == "lsh":
            perm = lsh_group(q, p)[1]
        else:   # groups of index neighbours: what reducing the contraction costs without the LSH
            perm = np.broadcast_to(np.arange(d, dtype=np.uint8), (1, 1, (N + l - 1) // l, d)).copy()
        s_hat, s = scores(q, k, p, perm=rotate_groups(perm, G, r))
        rel = (s_hat - s) / s
        out["elementwise"].append(np.abs(rel).mean())
        out["signed_mean"].append(abs(rel.mean()))
        out["matrix_sum"].append(abs((s_hat - s).sum()) / s.sum())
        c = 1.0 / np.sqrt(d)
        pr = np.exp(c * (s - s.max(1, keepdims=True)))
        pr /= pr.sum(1, keepdims=True)
        ph = np.exp(c * (s_hat - s_hat.max(1, keepdims=True)))
        ph /= ph.sum(1, keepdims=True)
        out["softmax"].append((np.abs(ph - pr) / pr).mean())
    return {k: np.asarray(v) for k, v in out.items()}


def summary(errors):
    """(min, max, mean) in percent over the experiments, per reading."""
    return {k: (100 * v.min(), 100 * v.max(), 100 * v.mean()) for k, v in errors.items()}


def main():
    cases = [(1, 2), (2, 2), (4, 2), (8, 2), (2, 4), (2, 8), (2, 16)]
    print("U(0,1), N = d = 64, 100 experiments; min / max / mean over the experiments, in percent\n")
    print("| l | G* | paper | " + " | ".join(READINGS) + " | elementwise, index groups |")
    print("|---|---|---|" + "---|" * (len(READINGS) + 1))
    for l, G in cases:
        paper = PAPER_TABLE3[l] if G == 2 else PAPER_TABLE4[G]
        s = summary(experiment_errors(l, G))
        naive = summary(experiment_errors(l, G, grouping="index"))["elementwise"]
        cells = " | ".join("%.2g / %.3g / %.3g" % s[k] for k in READINGS)
        print(f"| {l} | {G} | {paper[0]:g} / {paper[1]:g} / {paper[2]:g} | {cells} | %.2g / %.3g / %.3g |" % naive)
    print("\nWhich member of a group is sampled (elementwise mean, percent):\n")
    print("| l | G* | first | middle | last |")
    print("|---|---|---|---|---|")
    for l, G in cases:
        row = [summary(experiment_errors(l, G, representative=r))["elementwise"][2] for r in ("first", "middle", "last")]
        print(f"| {l} | {G} | " + " | ".join("%.2f" % x for x in row) + " |")


if __name__ == "__main__":
    main()
