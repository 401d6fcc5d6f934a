#!/usr/bin/env python3
"""How the cost of the LSH stage and the gain of DistrAttention scale with the sequence length
and with the Q block size (GPU path; the paper's token-length experiment, Sec. 4.5 / Table 10,
and its block-size discussion, Sec. 3.3 / Table 2, on this hardware).

For N = 1k .. 32k (one batch, 16 heads, d = 128 and d = 64, G* = 2, causal and not) the script
times, through the C ABI and with HIP events on the launch stream,
  * the LSH kernel, the key pre-pass and the DistrAttention kernel one by one,
  * the whole forward (the three launches back to back),
  * the exact kernel,
and prints a markdown table: the share of the LSH stage in the forward and the speed-up over the
exact kernel. A second table repeats the N = 8192 row for Br = 64 and Br = 128.

Usage: python scaling_study.py          (needs the GPU; inputs are seeded N(0,1) rounded to bf16)
"""
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)


def main():
    import torch

    import paper_2507_17245_amd as da

    dev = "cuda:0"

    def ev_time(fn, reps):
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    def row(B, H, N, d, Br, n_groups, causal):
        g = torch.Generator(device=dev).manual_seed(N + d)
        q, k, v = (torch.randn((B, H, N, d), device=dev, generator=g).to(torch.bfloat16) for _ in range(3))
        o = torch.empty_like(q)
        Tq = (N + Br - 1) // Br
        perm = torch.zeros((B, H, Tq, d), dtype=torch.uint8, device=dev)
        common = dict(Br=Br, causal=causal)
        p_full = da.make_params(q, k, v, n_groups=n_groups, **common)
        p_lsh = da.make_params(q, k, v, n_groups=n_groups, perm_out=perm, **common)
        kt = torch.empty(da.distr_attn_kt_bytes(p_full), dtype=torch.uint8, device=dev)
        p_attn = da.make_params(q, k, v, n_groups=n_groups, perm_in=perm, kt_in=kt, **common)
        p_ex = da.make_params(q, k, v, **common)
        reps = 20 if N <= 8192 else 8
        t_lsh = ev_time(lambda: da.distr_attn_lsh_group(q, p_lsh), reps)
        t_kt = ev_time(lambda: da.distr_attn_key_prepass(k, kt, p_full), reps)
        t_attn = ev_time(lambda: da.distr_attn_fwd_ex(q, k, v, o, p_attn), reps)
        t_full = ev_time(lambda: da.distr_attn_fwd_ex(q, k, v, o, p_full), reps)
        t_ex = ev_time(lambda: da.distr_attn_exact_fwd_ex(q, k, v, o, p_ex), reps)
        return t_lsh, t_kt, t_attn, t_full, t_ex

    print("## LSH cost and speed-up against the sequence length (B=1, H=16, Br=128, Bc=64, G*=2)\n")
    print("| d | causal | N | LSH kernel ms | key pre-pass ms | distr attention kernel ms | whole forward ms | "
          "LSH share of forward | exact kernel ms | speed-up |")
    print("|---|---|---|---|---|---|---|---|---|---|")
    for d in (128, 64):
        for causal in (False, True):
            for N in (1024, 2048, 4096, 8192, 16384, 32768):
                t_lsh, t_kt, t_attn, t_full, t_ex = row(1, 16, N, d, 128, d // 2, causal)
                print(f"| {d} | {'yes' if causal else 'no'} | {N} | {t_lsh:.4f} | {t_kt:.4f} | {t_attn:.4f} | {t_full:.4f} | "
                      f"{100 * t_lsh / t_full:.1f} % | {t_ex:.4f} | {t_ex / t_full:.3f} |", flush=True)

    print("\n## Q block size (B=4, H=16, N=8192, d=128, non-causal; Bc=64)\n")
    print("| Br | n_groups | whole forward ms | exact kernel ms | speed-up |")
    print("|---|---|---|---|---|")
    for Br in (64, 128):
        for ng in (64, 32):
            t_lsh, t_kt, t_attn, t_full, t_ex = row(4, 16, 8192, 128, Br, ng, False)
            print(f"| {Br} | {ng} | {t_full:.4f} | {t_ex:.4f} | {t_ex / t_full:.3f} |", flush=True)


if __name__ == "__main__":
    main()
