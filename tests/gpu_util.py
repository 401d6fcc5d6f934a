"""Helpers of the GPU parity tests: host arrays -> device tensors, one call through the C ABI,
results back as numpy. No arithmetic of the method lives here."""
import numpy as np
import torch

import oracle
import paper_2507_17245_amd as da

BF16_MAX_ABS, BF16_MEAN_ABS, F32_MAX_ABS = 2e-2, 2e-3, 1e-4   # tolerances of the parity bar


def to_dev(x, dtype):
    t = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    return t.to(torch.bfloat16) if dtype == "bf16" else t     # exact: values are bf16-representable


def run_gpu(cfg, q, k, v, distr=True, want_tables=False, n_groups=None, lsh_seed=None, gray_mode=0,
            scale=0.0, perm_in=None, lse_out=None, want_perm_only=False):
    """One forward through the C ABI. -> (o float64 numpy, perm uint8 or None, hash uint32 or None).
    scale 0 = the library's default 1/sqrt(d); perm_in: a grouping table (numpy uint8) to use
    instead of the LSH stage; lse_out: a float32 device tensor [B, H, N] the call fills with the
    rows' log-sum-exp; want_perm_only: ask for the permutation table alone (no hashes), which the
    bf16 attention kernel's own LSH stage then writes (returned in place of perm)."""
    tq, tk, tv = (to_dev(x, cfg.dtype) for x in (q, k, v))
    o = torch.full_like(tq, float("nan"))
    perm = hsh = None
    if want_tables:
        shape = (cfg.B, cfg.Hkv, cfg.Tk, cfg.d) if cfg.side == 1 else (cfg.B, cfg.H, cfg.Tq, cfg.d)
        perm = torch.zeros(shape, dtype=torch.uint8, device="cuda")
        hsh = torch.zeros(shape, dtype=torch.int32, device="cuda")
    if want_perm_only:
        perm = torch.full((cfg.B, cfg.H, cfg.Tq, cfg.d), 255, dtype=torch.uint8, device="cuda")
    t_perm_in = None if perm_in is None else torch.from_numpy(np.ascontiguousarray(perm_in, dtype=np.uint8)).cuda()
    p = da.make_params(tq, tk, tv, Br=cfg.Br, Bc=cfg.Bc,
                       n_groups=cfg.n_groups if n_groups is None else n_groups, causal=cfg.causal,
                       lsh_seed=cfg.lsh_seed if lsh_seed is None else lsh_seed,
                       n_planes=cfg.n_planes, gray_mode=gray_mode, perm_out=perm, hash_out=hsh,
                       softmax_scale=scale, perm_in=t_perm_in, side=cfg.side, lse_out=lse_out)
    if distr:
        da.distr_attn_fwd_ex(tq, tk, tv, o, p)
    else:
        da.distr_attn_exact_fwd_ex(tq, tk, tv, o, p)
    torch.cuda.synchronize()
    o_np = o.float().cpu().numpy().astype(np.float64)
    if want_tables:
        return o_np, perm.cpu().numpy(), hsh.cpu().numpy().view(np.uint32)
    if want_perm_only:
        return o_np, perm.cpu().numpy(), None
    return o_np, None, None


def run_gpu_lsh(cfg, q, gray_mode=0):
    tq = to_dev(q, cfg.dtype)
    perm = torch.zeros((cfg.B, cfg.H, cfg.Tq, cfg.d), dtype=torch.uint8, device="cuda")
    hsh = torch.zeros((cfg.B, cfg.H, cfg.Tq, cfg.d), dtype=torch.int32, device="cuda")
    p = da.make_params(tq, tq, tq, Br=cfg.Br, Bc=cfg.Bc, n_groups=cfg.n_groups, causal=cfg.causal,
                       lsh_seed=cfg.lsh_seed, n_planes=cfg.n_planes, gray_mode=gray_mode,
                       perm_out=perm, hash_out=hsh)
    da.distr_attn_lsh_group(tq, p)
    torch.cuda.synchronize()
    return perm.cpu().numpy(), hsh.cpu().numpy().view(np.uint32)


def oracle_params(cfg, n_groups=None, lsh_seed=None, gray_mode=0, scale=None):
    return oracle.params(cfg.B, cfg.H, cfg.Hkv, cfg.N, cfg.d, cfg.Br,
                         cfg.n_groups if n_groups is None else n_groups, causal=cfg.causal,
                         n_planes=cfg.n_planes, gray_mode=gray_mode,
                         lsh_seed=cfg.lsh_seed if lsh_seed is None else lsh_seed, scale=scale,
                         Nk=cfg.n_keys, side=cfg.side, Bc=cfg.Bc)


def oracle_tables(cfg, q, k, gray_mode=0):
    """(hash, perm) of the blocks the grouping is taken from: the Q blocks, or, for the mirrored
    form, the K blocks of Bc rows of every kv head."""
    if cfg.side == 1:
        pk = oracle.params(cfg.B, cfg.Hkv, cfg.Hkv, cfg.n_keys, cfg.d, cfg.Bc, cfg.n_groups, n_planes=cfg.n_planes,
                           gray_mode=gray_mode, lsh_seed=cfg.lsh_seed)
        return oracle.lsh_group(k, pk)[:2]
    return oracle.lsh_group(q, oracle_params(cfg, gray_mode=gray_mode))[:2]


def assert_close(got, want, dtype, what="", recorded=None):
    """The parity bar; `recorded` = (max-abs, mean-abs) measured for this case when it was last
    tuned: the errors may then not exceed three times those either, so that a regression far
    inside the bar still fails."""
    err = np.abs(got - want)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    if dtype == "bf16":
        assert err.max() <= BF16_MAX_ABS, f"{what}: max-abs {err.max():.4g}"
        assert err.mean() <= BF16_MEAN_ABS, f"{what}: mean-abs {err.mean():.4g}"
    else:
        assert err.max() <= F32_MAX_ABS, f"{what}: max-abs {err.max():.4g}"
    if recorded is not None:
        assert err.max() <= 3 * recorded[0], f"{what}: max-abs {err.max():.4g} > 3 x recorded {recorded[0]:.3g}"
        assert err.mean() <= 3 * recorded[1], f"{what}: mean-abs {err.mean():.4g} > 3 x recorded {recorded[1]:.3g}"
    return float(err.max()), float(err.mean())
