"""GPU parity for a key count different from the query count (decode against a cache, cross
attention; Sec. 2.1 with an N x Nk score matrix) and for the mirrored form of Sec. 3.1 / Fig. 4
right (sample K, fuse Q, one grouping per K block), against the CPU oracle."""
import numpy as np
import pytest

import oracle
import workloads as W

pytestmark = pytest.mark.gpu


def small(name, **kw):
    return W.CONFIGS[name].scaled(**kw)


@pytest.mark.parametrize("Nq", [1, 64, 300])
@pytest.mark.parametrize("Nk", [300, 4096])
@pytest.mark.parametrize("causal", [False, True])
def test_other_key_count(Nq, Nk, causal):
    import gpu_util as U
    for base, kw in (("llama", dict(H=4, Hkv=2)), ("long", dict(H=2, Hkv=1)), ("vit", dict(B=1, H=2, Hkv=2)),
                     ("mid", dict(B=1, H=2, Hkv=2, n_groups=32, Br=64))):
        cfg = small(base, N=Nq, Nk=Nk, causal=causal, data_seed=7000 + Nq + Nk, **kw)
        q, k, v = W.make(cfg)
        p = U.oracle_params(cfg)
        print(f"case {cfg}", flush=True)
        o_gpu, perm_gpu, hash_gpu = U.run_gpu(cfg, q, k, v, distr=True, want_tables=True)
        hash_ref, perm_ref = U.oracle_tables(cfg, q, k)
        assert np.array_equal(hash_gpu, hash_ref) and np.array_equal(perm_gpu, perm_ref)
        U.assert_close(o_gpu, oracle.distr_fwd(q, k, v, p), cfg.dtype, "distr")
        o_self, _, _ = U.run_gpu(cfg, q, k, v, distr=True)
        assert np.array_equal(o_self, o_gpu), "in-kernel LSH and LSH kernel disagree"
        o_ex, _, _ = U.run_gpu(cfg, q, k, v, distr=False)
        U.assert_close(o_ex, oracle.exact_fwd(q, k, v, p), cfg.dtype, "exact")


@pytest.mark.parametrize("Nq", [1, 200])
def test_decode_against_a_full_length_cache(Nq):
    """A few queries against the key count of the largest configuration (N_k = 32768, d = 128, and
    N_k = 16384 at d = 64 with grouped heads): the shape of decoding against a cache, every row
    against the oracle."""
    import gpu_util as U
    for base, kw in (("long", dict(H=4, Hkv=2, Nk=32768)), ("llama", dict(H=8, Hkv=2, Nk=16384))):
        cfg = small(base, N=Nq, causal=True, data_seed=7100 + Nq, **kw)
        q, k, v = W.make(cfg)
        p = U.oracle_params(cfg)
        print(f"case {cfg}", flush=True)
        o_gpu, perm_gpu, _ = U.run_gpu(cfg, q, k, v, distr=True, want_tables=True)
        assert np.array_equal(perm_gpu, U.oracle_tables(cfg, q, k)[1])
        U.assert_close(o_gpu, oracle.distr_fwd(q, k, v, p), cfg.dtype, "distr")
        o_ex, _, _ = U.run_gpu(cfg, q, k, v, distr=False)
        U.assert_close(o_ex, oracle.exact_fwd(q, k, v, p), cfg.dtype, "exact")


@pytest.mark.parametrize("Nq,Nk,causal", [(1, 200, False), (64, 300, True), (150, 150, True), (300, 70, False)])
def test_other_key_count_float_path(Nq, Nk, causal):
    import gpu_util as U
    for d, Br, ng in ((64, 64, 32), (128, 128, 16)):
        cfg = small("tiny", N=Nq, Nk=Nk, causal=causal, d=d, Br=Br, n_groups=ng, H=2, Hkv=1, recipe="normal")
        q, k, v = W.make(cfg)
        p = U.oracle_params(cfg)
        print(f"case {cfg}", flush=True)
        o_gpu, perm_gpu, _ = U.run_gpu(cfg, q, k, v, distr=True, want_tables=True)
        assert np.array_equal(perm_gpu, U.oracle_tables(cfg, q, k)[1])
        U.assert_close(o_gpu, oracle.distr_fwd(q, k, v, p), "f32", "distr")
        o_ex, _, _ = U.run_gpu(cfg, q, k, v, distr=False)
        U.assert_close(o_ex, oracle.exact_fwd(q, k, v, p), "f32", "exact")


@pytest.mark.parametrize("Bc", [32, 64, 128])
@pytest.mark.parametrize("Nq,Nk,causal", [(256, 256, False), (100, 333, True), (1, 130, False), (200, 200, True)])
def test_mirrored_form(Nq, Nk, causal, Bc):
    """side = 1: the K blocks' tables bit for bit, the output within the float tolerance, and the
    caller's table honoured."""
    import gpu_util as U
    for d, Br, ng, recipe in ((64, 64, 32, "latent_pairs"), (128, 128, 32, "normal"), (64, 128, 64, "normal")):
        cfg = small("tiny", N=Nq, Nk=Nk, causal=causal, d=d, Br=Br, Bc=Bc, n_groups=ng, H=4, Hkv=2, B=2,
                    recipe=recipe, side=1, n_planes=16)
        q, k, v = W.make(cfg)
        p = U.oracle_params(cfg)
        print(f"case {cfg}", flush=True)
        o_gpu, perm_gpu, hash_gpu = U.run_gpu(cfg, q, k, v, distr=True, want_tables=True)
        hash_ref, perm_ref = U.oracle_tables(cfg, q, k)
        assert np.array_equal(hash_gpu, hash_ref) and np.array_equal(perm_gpu, perm_ref)
        U.assert_close(o_gpu, oracle.distr_fwd(q, k, v, p), "f32", "mirrored")
        o_ws, _, _ = U.run_gpu(cfg, q, k, v, distr=True)      # table in the library's workspace
        assert np.array_equal(o_ws, o_gpu)
        if ng < d:     # it differs from the form that samples Q
            o_q, _, _ = U.run_gpu(cfg.scaled(side=0, Bc=64), q, k, v, distr=True)
            assert np.abs(o_q - o_gpu).max() > 1e-4
        rng = np.random.default_rng(3)
        table = np.stack([rng.permutation(d) for _ in range(cfg.B * cfg.Hkv * cfg.Tk)]).astype(np.uint8)
        table = table.reshape(cfg.B, cfg.Hkv, cfg.Tk, d)
        o_t, _, _ = U.run_gpu(cfg, q, k, v, distr=True, perm_in=table)
        U.assert_close(o_t, oracle.distr_fwd(q, k, v, p, perm=table), "f32", "mirrored, caller's table")


@pytest.mark.parametrize("Nq,Nk,causal,Bc", [(256, 256, False, 64), (100, 333, True, 32), (200, 200, True, 128)])
def test_mirrored_form_on_bf16_tensors(Nq, Nk, causal, Bc):
    """side = 1 with bf16 tensors runs the float-arithmetic kernel (values converted on load, the
    output rounded on store): the K blocks' tables bit for bit, the output within the bf16 bar."""
    import gpu_util as U
    for d, Br, ng in ((64, 64, 32), (128, 128, 32), (128, 64, 64)):
        cfg = small("vit", B=2, H=4, Hkv=2, N=Nq, Nk=Nk, causal=causal, d=d, Br=Br, Bc=Bc, n_groups=ng,
                    side=1, n_planes=16)
        assert cfg.dtype == "bf16"
        q, k, v = W.make(cfg)
        p = U.oracle_params(cfg)
        print(f"case {cfg}", flush=True)
        o_gpu, perm_gpu, hash_gpu = U.run_gpu(cfg, q, k, v, distr=True, want_tables=True)
        hash_ref, perm_ref = U.oracle_tables(cfg, q, k)
        assert np.array_equal(hash_gpu, hash_ref) and np.array_equal(perm_gpu, perm_ref)
        U.assert_close(o_gpu, oracle.distr_fwd(q, k, v, p), "bf16", "mirrored, bf16 tensors")
        o_ws, _, _ = U.run_gpu(cfg, q, k, v, distr=True)      # table in the library's workspace
        assert np.array_equal(o_ws, o_gpu)
