"""GPU parity of the boundary's options against the CPU oracle: a caller-chosen softmax scale
(1.0 is the literal S = Q K^T of Sec. 2.1), a caller-provided grouping table, the input-range
limits of the half-precision reduced product, and the block order used for large causal problems."""
import numpy as np
import pytest

import oracle
import workloads as W

pytestmark = pytest.mark.gpu


def small(name, **kw):
    return W.CONFIGS[name].scaled(**kw)


@pytest.mark.parametrize("scale", [1.0, 0.05, 0.3])
@pytest.mark.parametrize("base,kw", [("vit", dict(B=1, H=3, Hkv=3, N=150)),
                                     ("long", dict(H=2, Hkv=1, N=300)),
                                     ("tiny", dict(N=130))])
def test_softmax_scale(base, kw, scale):
    import gpu_util as U
    cfg = small(base, **kw)
    q, k, v = W.make(cfg)
    if scale == 1.0:
        # unscaled logits of N(0,1) data have a spread of sqrt(d): bring the inputs down so that
        # the softmax is not one-hot and the comparison says something
        q = W.round_to_bf16(q * 0.5) if cfg.dtype == "bf16" else q * np.float32(0.5)
        k = W.round_to_bf16(k * 0.5) if cfg.dtype == "bf16" else k * np.float32(0.5)
    p = U.oracle_params(cfg, scale=scale)
    print(f"case {cfg} scale {scale}", flush=True)
    o_gpu, perm_gpu, _ = U.run_gpu(cfg, q, k, v, distr=True, want_tables=True, scale=scale)
    assert np.array_equal(perm_gpu, oracle.lsh_group(q, p)[1])
    U.assert_close(o_gpu, oracle.distr_fwd(q, k, v, p), cfg.dtype, "distr")
    o_self, _, _ = U.run_gpu(cfg, q, k, v, distr=True, scale=scale)
    assert np.array_equal(o_self, o_gpu)
    o_ex, _, _ = U.run_gpu(cfg, q, k, v, distr=False, scale=scale)
    U.assert_close(o_ex, oracle.exact_fwd(q, k, v, p), cfg.dtype, "exact")
    # the scale really reached the kernels: the default-scale output is something else
    o_def, _, _ = U.run_gpu(cfg, q, k, v, distr=False)
    assert np.abs(o_def - o_ex).max() > 1e-2


@pytest.mark.parametrize("base,kw", [("vit", dict(B=2, H=2, Hkv=2, N=200)),
                                     ("llama", dict(H=4, Hkv=2, N=300)),
                                     ("mid", dict(B=1, H=2, Hkv=2, N=260, n_groups=32)),
                                     ("tiny", dict(N=200))])
def test_caller_grouping_table(base, kw):
    """perm_in replaces the LSH stage: a random valid table per query block, against the oracle
    run with the same table."""
    import gpu_util as U
    cfg = small(base, **kw)
    q, k, v = W.make(cfg)
    rng = np.random.default_rng(42)
    perm = np.stack([rng.permutation(cfg.d) for _ in range(cfg.B * cfg.H * cfg.Tq)]).astype(np.uint8)
    perm = perm.reshape(cfg.B, cfg.H, cfg.Tq, cfg.d)
    p = U.oracle_params(cfg)
    print(f"case {cfg} perm_in", flush=True)
    o_gpu, _, _ = U.run_gpu(cfg, q, k, v, distr=True, perm_in=perm)
    U.assert_close(o_gpu, oracle.distr_fwd(q, k, v, p, perm=perm), cfg.dtype, "distr with perm_in")
    # the table mattered: the LSH grouping gives another result
    o_lsh, _, _ = U.run_gpu(cfg, q, k, v, distr=True)
    assert np.abs(o_lsh - o_gpu).max() > 1e-3


def test_half_range_clamp_of_the_reduced_product():
    """bf16 DistrAttention holds Q_r (times softmax_scale * log2 e) and K_f in half precision:
    |q| * softmax_scale * log2(e) beyond 65504 and |k| beyond 65504 / G* are clamped (documented
    input limit). The oracle, fed the clamped values and the grouping of the unclamped Q (the
    LSH stage sees the original values), must agree."""
    import gpu_util as U
    for n_groups in (32, 16):
        cfg = small("vit", B=1, H=2, Hkv=2, N=150, n_groups=n_groups)
        G = cfg.d // n_groups
        q, k, v = W.make(cfg)
        q, k = q.copy(), k.copy()
        big = np.float32(2.0 ** 20)
        q[0, 0, 3, 5], q[0, 1, 70, 9], q[0, 0, 149, 60] = big, -big, big
        k[0, 0, 10, 7], k[0, 1, 100, 33], k[0, 0, 64, 0] = big, -big, -big
        p = U.oracle_params(cfg)
        perm = oracle.lsh_group(q, p)[1]
        q_lim = 65504.0 / (np.log2(np.e) / np.sqrt(cfg.d))
        assert float(big) > q_lim
        qc = np.clip(q, -q_lim, q_lim).astype(np.float32)
        kc = np.clip(k, -65504.0 / G, 65504.0 / G).astype(np.float32)
        print(f"case {cfg} clamp", flush=True)
        o_gpu, perm_gpu, _ = U.run_gpu(cfg, q, k, v, distr=True, want_tables=True)
        assert np.array_equal(perm_gpu, perm)
        U.assert_close(o_gpu, oracle.distr_fwd(qc, kc, v, p, perm=perm), "bf16", f"clamped, G*={G}")


@pytest.mark.parametrize("shift", [-8, 10])
def test_inputs_far_from_unit_scale(shift):
    """Q and K scaled by a power of two with the softmax scale compensating: the scores are the
    same numbers, the half-precision operands of the reduced product sit elsewhere in half's
    exponent range (documented range: 2^-14 <= |x| <= 65504 / G* keeps full precision)."""
    import gpu_util as U
    for base, kw in (("llama", dict(H=4, Hkv=2, N=300)), ("mid", dict(B=1, H=2, Hkv=2, N=260))):
        cfg = small(base, **kw)
        q, k, v = W.make(cfg)
        f = np.float32(2.0 ** shift)
        q2, k2 = q * f, k * f                     # exact: powers of two keep bf16 values on the grid
        scale = float(1.0 / np.sqrt(cfg.d) / (float(f) * float(f)))
        p = U.oracle_params(cfg, scale=scale)
        print(f"case {cfg} shift {shift}", flush=True)
        o_gpu, perm_gpu, _ = U.run_gpu(cfg, q2, k2, v, distr=True, want_tables=True, scale=scale)
        assert np.array_equal(perm_gpu, oracle.lsh_group(q2, p)[1])
        U.assert_close(o_gpu, oracle.distr_fwd(q2, k2, v, p), "bf16", "distr")
        o_ex, _, _ = U.run_gpu(cfg, q2, k2, v, distr=False, scale=scale)
        U.assert_close(o_ex, oracle.exact_fwd(q2, k2, v, p), "bf16", "exact")


def test_head_major_causal_order_on_every_block():
    """Causal problems of more than 2048 query blocks are dispatched head by head (longest block
    first inside a head) instead of longest-first over all heads: every block of such a problem
    against the oracle."""
    import gpu_util as U
    cfg = small("vit", B=4, H=16, Hkv=16, N=2100, causal=True, Br=64)
    assert cfg.B * cfg.H * cfg.Tq > 2048
    q, k, v = W.make(cfg)
    p = U.oracle_params(cfg)
    print(f"case {cfg}", flush=True)
    o_gpu, perm_gpu, _ = U.run_gpu(cfg, q, k, v, distr=True, want_tables=True)
    assert np.array_equal(perm_gpu, oracle.lsh_group(q, p)[1])
    U.assert_close(o_gpu, oracle.distr_fwd(q, k, v, p), "bf16", "distr")
    o_ex, _, _ = U.run_gpu(cfg, q, k, v, distr=False)
    U.assert_close(o_ex, oracle.exact_fwd(q, k, v, p), "bf16", "exact")


@pytest.mark.parametrize("base,kw", [("tiny", dict(N=150)), ("vit", dict(B=1, H=3, Hkv=3, N=150)),
                                     ("llama", dict(H=4, Hkv=2, N=300, Nk=421)),
                                     ("mid", dict(B=1, H=2, Hkv=2, N=260, Br=256, Bc=128))])
def test_row_statistics_output(base, kw):
    """lse_out: the logarithm of every row's softmax denominator (Sec. 2.2.2 keeps it as running
    maximum and sum), for the approximate and the exact scores, against the oracle's."""
    import torch

    import gpu_util as U
    cfg = small(base, **kw)
    q, k, v = W.make(cfg)
    p = U.oracle_params(cfg)
    tol = 1e-4 if cfg.dtype == "f32" else 2e-2
    for distr in (True, False):
        lse = torch.full((cfg.B, cfg.H, cfg.N), float("nan"), dtype=torch.float32, device="cuda")
        o, _, _ = U.run_gpu(cfg, q, k, v, distr=distr, lse_out=lse)
        ref = oracle.lse(q, k, p, distr=distr)
        err = np.abs(lse.cpu().numpy().astype(np.float64) - ref)
        print(f"  {base} distr={distr}: lse max-abs {err.max():.3g}", flush=True)
        assert err.max() <= tol
        # asking for the statistics does not change the output
        o2, _, _ = U.run_gpu(cfg, q, k, v, distr=distr)
        assert np.array_equal(o, o2)


def test_debug_mode_synchronises_after_every_launch():
    """DISTR_ATTN_DEBUG=1 (read when the library is first called, hence a process of its own): the
    small end-to-end check (LSH kernel, key pre-pass, both attention kernels) still passes."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    env = dict(os.environ, DISTR_ATTN_DEBUG="1")
    res = subprocess.run([sys.executable, "-c", "import __graft_entry__ as g; g.smoke()"], cwd=root, env=env,
                         capture_output=True, text=True, timeout=110)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-2000:]
