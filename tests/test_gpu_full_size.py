"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

Group tables (hash, permutation) of EVERY query block are compared bit for bit with the oracle.
Outputs are compared on a deterministic sample of query blocks (first two, middle, last two and
three seeded random ones per head) that the oracle computes one by one over all visible keys."""
import numpy as np
import pytest

import oracle
import workloads as W

pytestmark = pytest.mark.gpu

CASES = [("vit", 32), ("llama", 32), ("mid", 128), ("mid", 64), ("mid", 32), ("long", 64)]
# (max-abs, mean-abs) against the oracle on the sampled blocks, as measured when the kernels were
# last tuned: {case: (distr, exact)}. The test fails beyond three times these, far inside the
# 2e-2 / 2e-3 bar, so that a loss of accuracy shows up even where the bar is loose.
RECORDED = {
    ("vit", 32): ((2.9e-3, 2.2e-4), (4.2e-3, 2.4e-4)),
    ("llama", 32): ((1.3e-2, 8.0e-4), (1.2e-2, 7.6e-4)),
    ("mid", 128): ((1.2e-3, 4.9e-5), (1.2e-3, 4.9e-5)),
    ("mid", 64): ((9.7e-4, 3.9e-5), (1.2e-3, 4.9e-5)),
    ("mid", 32): ((1.1e-3, 4.0e-5), (1.2e-3, 4.9e-5)),
    ("long", 64): ((7.7e-3, 1.5e-4), (8.9e-3, 2.4e-4)),
}
_inputs = {}


def inputs(name):
    if name not in _inputs:
        _inputs.clear()                      # keep one configuration in host memory at a time
        _inputs[name] = W.make(W.CONFIGS[name])
    return _inputs[name]


@pytest.mark.parametrize("name,n_groups", CASES, ids=[f"{n}-k{g}" for n, g in CASES])
def test_full_size_parity(name, n_groups):
    import gpu_util as U
    cfg = W.CONFIGS[name].scaled(n_groups=n_groups)
    print(f"case {cfg}", flush=True)
    q, k, v = inputs(name)
    p = U.oracle_params(cfg)
    o_gpu, perm_gpu, hash_gpu = U.run_gpu(cfg, q, k, v, distr=True, want_tables=True)
    hash_ref, perm_ref, _ = oracle.lsh_group(q, p)
    assert np.array_equal(hash_gpu, hash_ref), "hashes differ"
    assert np.array_equal(perm_gpu, perm_ref), "permutations differ"
    heads = range(cfg.H) if cfg.N <= 4096 else range(0, cfg.H, 4)
    batches = sorted({0, cfg.B - 1})
    tiles = [(b, h, t) for b in batches for (_, h, t) in W.sample_tiles(cfg, heads=heads)]
    print(f"  oracle on {len(tiles)} query blocks", flush=True)

    def gather(o):
        out = np.full((len(tiles), cfg.Br, cfg.d), np.nan)
        for i, (b, h, t) in enumerate(tiles):
            rows = min(cfg.Br, cfg.N - t * cfg.Br)
            out[i, :rows] = o[b, h, t * cfg.Br:t * cfg.Br + rows]
        return out

    ref = oracle.distr_fwd_tiles(q, k, v, p, tiles)
    valid = ~np.isnan(ref)
    got = gather(o_gpu)
    assert np.array_equal(~np.isnan(got), valid)
    mx, mean = U.assert_close(got[valid], ref[valid], cfg.dtype, "distr", recorded=RECORDED[(name, n_groups)][0])
    print(f"  distr: max-abs {mx:.3g} mean-abs {mean:.3g}", flush=True)
    assert np.isfinite(o_gpu).all()
    # the call bench.py times asks for no tables: the attention kernel then does the LSH stage of
    # its own Q block, and must give the same output bit for bit
    o_self, _, _ = U.run_gpu(cfg, q, k, v, distr=True, want_tables=False)
    assert np.array_equal(o_self, o_gpu), "in-kernel LSH and LSH kernel disagree"
    if cfg.dtype == "bf16" and n_groups < cfg.d:
        # and its table, written on request, is the oracle's on every block
        _, perm_own, _ = U.run_gpu(cfg, q, k, v, distr=True, want_perm_only=True)
        assert np.array_equal(perm_own, perm_ref), "table of the attention kernel's own LSH stage differs"
    del o_gpu, o_self
    o_ex, _, _ = U.run_gpu(cfg, q, k, v, distr=False)
    ref_ex = oracle.exact_fwd_tiles(q, k, v, p, tiles)
    mx, mean = U.assert_close(gather(o_ex)[valid], ref_ex[valid], cfg.dtype, "exact", recorded=RECORDED[(name, n_groups)][1])
    print(f"  exact: max-abs {mx:.3g} mean-abs {mean:.3g}", flush=True)
    assert np.isfinite(o_ex).all()
    if n_groups == cfg.d:   # groups of one channel: the approximation is the exact product (Sec. 3.1)
        approx = np.abs(got[valid] - gather(o_ex)[valid])
        assert approx.max() <= 2e-2
