"""GPU parity for every (head dim, Q block rows Br, K/V tile rows Bc) the bf16 kernels are built
for (the paper's block sizes l and m, Sec. 3.3): exact and DistrAttention against the oracle.
The result depends on Br (one grouping per Q block) and not on Bc."""
import numpy as np
import pytest

import oracle
import workloads as W

pytestmark = pytest.mark.gpu

SHAPES = [(d, Br, Bc) for d in (64, 128) for Br in (64, 128, 256) for Bc in (32, 64, 128)]


@pytest.mark.parametrize("d,Br,Bc", SHAPES, ids=[f"d{d}-Br{Br}-Bc{Bc}" for d, Br, Bc in SHAPES])
def test_block_sizes(d, Br, Bc):
    import gpu_util as U
    base = "vit" if d == 64 else "mid"
    for causal, N, Nk in ((False, 333, 0), (True, 700, 0), (True, 130, 450)):
        for ng in (d // 2, d // 4):
            cfg = W.CONFIGS[base].scaled(B=1, H=4, Hkv=2, N=N, Nk=Nk, causal=causal, Br=Br, Bc=Bc, n_groups=ng,
                                         data_seed=8000 + d + Br + Bc)
            q, k, v = W.make(cfg)
            p = U.oracle_params(cfg)
            print(f"case {cfg}", flush=True)
            o_gpu, perm_gpu, hash_gpu = U.run_gpu(cfg, q, k, v, distr=True, want_tables=True)
            hash_ref, perm_ref = U.oracle_tables(cfg, q, k)
            assert np.array_equal(hash_gpu, hash_ref) and np.array_equal(perm_gpu, perm_ref)
            U.assert_close(o_gpu, oracle.distr_fwd(q, k, v, p), "bf16", "distr")
            o_self, _, _ = U.run_gpu(cfg, q, k, v, distr=True)
            assert np.array_equal(o_self, o_gpu), "in-kernel LSH and LSH kernel disagree"
        o_ex, _, _ = U.run_gpu(cfg, q, k, v, distr=False)
        U.assert_close(o_ex, oracle.exact_fwd(q, k, v, p), "bf16", "exact")


def test_float_path_takes_blocks_of_256_rows():
    import gpu_util as U
    for d in (64, 128):
        cfg = W.CONFIGS["tiny"].scaled(N=600, d=d, Br=256, n_groups=d // 2, H=2, Hkv=1, causal=True, recipe="normal",
                                       n_planes=16)
        q, k, v = W.make(cfg)
        p = U.oracle_params(cfg)
        o_gpu, perm_gpu, _ = U.run_gpu(cfg, q, k, v, distr=True, want_tables=True)
        assert np.array_equal(perm_gpu, U.oracle_tables(cfg, q, k)[1])
        U.assert_close(o_gpu, oracle.distr_fwd(q, k, v, p), "f32", "distr")
