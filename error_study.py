#!/usr/bin/env python3
"""Approximation-error study of DistrAttention on the five synthetic configurations (GPU path).

For every configuration the output of the DistrAttention kernel is compared with the output of
the exact kernel (both through the C ABI, same inputs) for
  * the LSH grouping with the default Gray map (hash = position of the sign word in the Gray
    sequence) and with the literal table lookup (Sec. 3.2),
  * a grouping that ignores the data (channels grouped by index: the identity permutation),
which separates what the LSH buys from what merely reducing the contraction costs. It also
prints, from the CPU oracle, the paper's own synthetic experiment (Sec. 4.2, Tables 3-4:
U(0,1), N = d = 64, relative error of the approximate scores) for both Gray maps.

Usage: python error_study.py            (needs the GPU; prints a markdown report)
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)


def paper_experiment():
    import oracle
    print("## Sec. 4.2 experiment with the CPU oracle: U(0,1), N = d = 64, 100 draws, mean / max of |S^ - S| / |S| in %\n")
    print("| block size l | G* | default Gray map (rank) | literal Gray table | channels grouped by index |")
    print("|---|---|---|---|---|")
    rng = np.random.default_rng(0)
    N = d = 64
    draws = [(rng.random((1, 1, N, d), dtype=np.float32), rng.random((1, 1, N, d), dtype=np.float32)) for _ in range(100)]
    for l, G in [(1, 2), (2, 2), (4, 2), (8, 2), (2, 4), (2, 8), (2, 16)]:
        cells = []
        for mode in (0, 1, None):
            means, maxs = [], []
            for rep, (q, k) in enumerate(draws):
                p = oracle.params(1, 1, 1, N, d, l, d // G, gray_mode=mode or 0, lsh_seed=rep, scale=1.0)
                perm = None
                if mode is None:
                    perm = np.broadcast_to(np.arange(d, dtype=np.uint8), (1, 1, (N + l - 1) // l, d)).copy()
                s_hat, s = oracle.scores(q, k, p, perm=perm)
                rel = np.abs(s_hat - s) / np.abs(s)
                means.append(rel.mean())
                maxs.append(rel.max())
            cells.append(f"{100 * np.mean(means):.2f} / {100 * np.max(maxs):.1f}")
        print(f"| {l} | {G} | {cells[0]} | {cells[1]} | {cells[2]} |")
    print("\nPaper, Table 3 (G* = 2): mean 0.9 / 0.87 / 0.87 / 0.87 for l = 1, 2, 4, 8; Table 4 (l = 2): mean 0.87 / 1.73 / "
          "2.48 / 4.96, max 3.4 / 5.4 / 9.25 / 16.5 for G* = 2, 4, 8, 16.\n")


def gpu_study():
    import torch

    import paper_2507_17245_amd as da
    import workloads as W

    print("## Output error of the DistrAttention kernel against the exact kernel (same inputs, GPU, full sizes)\n")
    print("mean-abs / max-abs of O_distr - O_exact over all outputs; rms(O_exact) for scale.\n")
    print("| config | n_groups (G*) | rms(O) | LSH, default Gray map | LSH, literal Gray table | grouped by index (no LSH) |")
    print("|---|---|---|---|---|---|")
    for name in ("vit", "llama", "mid", "long"):
        cfg = W.CONFIGS[name]
        q, k, v = (torch.from_numpy(x).cuda().to(torch.bfloat16) for x in W.make(cfg))
        o_ex = torch.empty_like(q)
        da.distr_attn_exact_fwd_ex(q, k, v, o_ex, da.make_params(q, k, v, Br=cfg.Br, causal=cfg.causal))
        torch.cuda.synchronize()
        ref = o_ex.float()
        rms = float(ref.pow(2).mean().sqrt())
        ident = torch.arange(cfg.d, dtype=torch.uint8, device="cuda").expand(cfg.B, cfg.H, cfg.Tq, cfg.d).contiguous()
        # "mid": every group size of the paper's Table 4 (G* = 2, 4, 8, 16)
        groups = (64, 32, 16, 8) if name == "mid" else (cfg.n_groups,)
        for ng in groups:
            cells = []
            for kw in (dict(gray_mode=0), dict(gray_mode=1), dict(perm_in=ident)):
                o = torch.empty_like(q)
                p = da.make_params(q, k, v, Br=cfg.Br, n_groups=ng, causal=cfg.causal, lsh_seed=cfg.lsh_seed,
                                   n_planes=cfg.n_planes, **kw)
                da.distr_attn_fwd_ex(q, k, v, o, p)
                torch.cuda.synchronize()
                diff = (o.float() - ref).abs()
                cells.append(f"{float(diff.mean()):.4f} / {float(diff.max()):.3f}")
                del o, diff
            print(f"| {name} | {ng} ({cfg.d // ng}) | {rms:.3f} | {cells[0]} | {cells[1]} | {cells[2]} |", flush=True)
        del q, k, v, o_ex, ref
        torch.cuda.empty_cache()


if __name__ == "__main__":
    paper_experiment()
    gpu_study()
