"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs. Group tables (hashes, permutations) must match bit for bit; outputs within
max-abs 2e-2 and mean-abs 2e-3 for bf16 inputs with float accumulation, 1e-4 for float inputs."""
import numpy as np
import pytest

import oracle
import workloads as W

pytestmark = pytest.mark.gpu


def _util():
    import gpu_util
    return gpu_util


def small(name, **kw):
    return W.CONFIGS[name].scaled(**kw)


SMALL_CASES = [
    # several tiles and a ragged tail, in the structure of each benchmark configuration
    small("vit", B=2, H=3, Hkv=3),                                   # N = 197 = 3*64 + 5
    small("llama", H=8, Hkv=2, N=333),                               # causal, GQA, Br 128, ragged
    small("mid", B=1, H=2, Hkv=2, N=520, n_groups=64),
    small("mid", B=1, H=2, Hkv=2, N=520, n_groups=32),
    small("mid", B=1, H=2, Hkv=2, N=520, n_groups=128),              # G* = 1
    small("mid", B=1, H=2, Hkv=2, N=300, n_groups=16),
    small("long", H=2, Hkv=2, N=700),                                # causal, d 128
    small("long", H=4, Hkv=1, N=257, Br=64),                         # Br 64 with d 128, GQA
    small("vit", B=1, H=2, Hkv=2, N=130, n_groups=16),
    small("vit", B=1, H=2, Hkv=1, N=130, n_groups=64, Br=128, causal=True),
    small("vit", B=1, H=2, Hkv=2, N=200, n_groups=16, Br=128),       # d 64, Br 128, G* = 4
    small("long", H=2, Hkv=2, N=200, Br=64, n_groups=16),            # d 128, Br 64, G* = 8
    small("long", H=2, Hkv=1, N=200, Br=64, n_groups=32, causal=False),
    small("mid", B=1, H=2, Hkv=2, N=300, n_groups=8),                # G* = 16: contraction zero-padded to one MFMA step
    small("vit", B=1, H=2, Hkv=1, N=200, n_groups=8, Br=128, causal=True),   # d 64, G* = 8
    small("vit", B=1, H=2, Hkv=2, N=130, n_groups=4),                # d 64, G* = 16, Br 64
    small("long", H=2, Hkv=2, N=200, Br=64, n_groups=8),             # d 128, Br 64, G* = 16
    small("vit", B=8, N=700, causal=True),                           # 1056 short causal blocks of 1..11 tiles (more
                                                                     # blocks than the chip holds at once; blocks of 2-3
                                                                     # tiles once exposed a missing barrier after tile 0)
    small("tiny"),                                                   # float path, full config
    small("tiny", N=150, d=128, n_groups=32, Br=128, causal=True, recipe="normal"),
    small("tiny", N=100, n_groups=1, recipe="normal"),               # float path, one group of all channels
    small("tiny", N=100, n_groups=64, recipe="normal", causal=True), # float path, groups of one channel
    small("tiny", N=70, n_groups=4, H=4, Hkv=2, B=2, recipe="normal"),
]


@pytest.mark.parametrize("cfg", SMALL_CASES, ids=lambda c: f"{c.name}-N{c.N}-d{c.d}-k{c.n_groups}-Br{c.Br}-{'c' if c.causal else 'n'}")
def test_small_cases_match_oracle(cfg):
    U = _util()
    q, k, v = W.make(cfg)
    p = U.oracle_params(cfg)
    print(f"case {cfg}", flush=True)
    o_gpu, perm_gpu, hash_gpu = U.run_gpu(cfg, q, k, v, distr=True, want_tables=True)
    hash_ref, perm_ref, _ = oracle.lsh_group(q, p)
    assert np.array_equal(hash_gpu, hash_ref), "hashes differ"
    assert np.array_equal(perm_gpu, perm_ref), "permutations differ"
    U.assert_close(o_gpu, oracle.distr_fwd(q, k, v, p), cfg.dtype, "distr")
    # without table outputs the bf16 attention kernel hashes and groups its Q block itself:
    # same tables, so the same output bit for bit
    o_self, _, _ = U.run_gpu(cfg, q, k, v, distr=True, want_tables=False)
    assert np.array_equal(o_self, o_gpu), "in-kernel LSH and LSH kernel disagree"
    if cfg.dtype == "bf16" and cfg.n_groups < cfg.d:
        # asked for the table alone, that stage writes it: the oracle's, bit for bit
        o_own, perm_own, _ = U.run_gpu(cfg, q, k, v, distr=True, want_perm_only=True)
        assert np.array_equal(perm_own, perm_ref), "table of the attention kernel's own LSH stage differs"
        assert np.array_equal(o_own, o_gpu)
    o_ex, _, _ = U.run_gpu(cfg, q, k, v, distr=False)
    U.assert_close(o_ex, oracle.exact_fwd(q, k, v, p), cfg.dtype, "exact")


@pytest.mark.parametrize("N", [1, 2, 63, 64, 65, 127, 128, 129])
@pytest.mark.parametrize("causal", [False, True])
def test_edge_lengths(N, causal):
    U = _util()
    for base in ("vit", "mid"):
        cfg = small(base, B=1, H=2, Hkv=2, N=N, causal=causal, data_seed=5000 + N)
        q, k, v = W.make(cfg)
        p = U.oracle_params(cfg)
        print(f"case {cfg}", flush=True)
        o_gpu, perm_gpu, _ = U.run_gpu(cfg, q, k, v, distr=True, want_tables=True)
        assert np.array_equal(perm_gpu, oracle.lsh_group(q, p)[1])
        U.assert_close(o_gpu, oracle.distr_fwd(q, k, v, p), cfg.dtype, "distr")
        o_ex, _, _ = U.run_gpu(cfg, q, k, v, distr=False)
        U.assert_close(o_ex, oracle.exact_fwd(q, k, v, p), cfg.dtype, "exact")


def test_gray_modes_seeds_and_plane_counts():
    U = _util()
    cfg = small("mid", B=1, H=3, Hkv=3, N=400)
    q, _, _ = W.make(cfg)
    for gray_mode in (0, 1):
        for planes in (1, 4, 7, 16, 31, 32):
            for seed in (0, 12345678901234567):
                c = cfg.scaled(n_planes=planes, lsh_seed=seed)
                perm_gpu, hash_gpu = U.run_gpu_lsh(c, q, gray_mode=gray_mode)
                hash_ref, perm_ref, _ = oracle.lsh_group(q, U.oracle_params(c, gray_mode=gray_mode))
                assert np.array_equal(hash_gpu, hash_ref), (gray_mode, planes, seed)
                assert np.array_equal(perm_gpu, perm_ref), (gray_mode, planes, seed)
    # the attention kernel's own LSH stage (no table outputs, up to 16 projections) follows the
    # same options: its output equals the output computed from the LSH kernel's table
    _, k, v = W.make(cfg)
    for gray_mode, planes, seed in ((0, 1, 0), (1, 4, 3), (0, 7, 12345678901234567), (1, 16, 5), (0, 31, 1)):
        c = cfg.scaled(n_planes=planes, lsh_seed=seed)
        o_tab, _, _ = U.run_gpu(c, q, k, v, distr=True, want_tables=True, gray_mode=gray_mode)
        o_self, _, _ = U.run_gpu(c, q, k, v, distr=True, want_tables=False, gray_mode=gray_mode)
        assert np.array_equal(o_tab, o_self), (gray_mode, planes, seed)
    # d = 64: the attention kernel's own stage takes the projections on the matrix pipe
    for base, kw in (("vit", dict(B=1, H=3, Hkv=3, N=200)), ("llama", dict(H=4, Hkv=2, N=400))):
        cfg64 = small(base, **kw)
        q, k, v = W.make(cfg64)
        for gray_mode, planes, seed in ((0, 1, 0), (1, 4, 3), (0, 7, 12345678901234567), (1, 16, 5), (0, 15, 2 ** 63 + 11)):
            c = cfg64.scaled(n_planes=planes, lsh_seed=seed)
            o_tab, perm_gpu, hash_gpu = U.run_gpu(c, q, k, v, distr=True, want_tables=True, gray_mode=gray_mode)
            hash_ref, perm_ref, _ = oracle.lsh_group(q, U.oracle_params(c, gray_mode=gray_mode))
            assert np.array_equal(hash_gpu, hash_ref) and np.array_equal(perm_gpu, perm_ref), (base, gray_mode, planes, seed)
            o_self, _, _ = U.run_gpu(c, q, k, v, distr=True, want_tables=False, gray_mode=gray_mode)
            assert np.array_equal(o_tab, o_self), (base, gray_mode, planes, seed)


def test_degenerate_inputs():
    U = _util()
    cfg = small("vit", B=1, H=2, Hkv=2, N=100)
    q, k, v = W.make(cfg)
    # all-zero queries: every code is 0, the permutation is the identity, attention is uniform
    q0 = np.zeros_like(q)
    o_gpu, perm_gpu, hash_gpu = U.run_gpu(cfg, q0, k, v, distr=True, want_tables=True)
    assert not hash_gpu.any()
    assert np.array_equal(perm_gpu, np.broadcast_to(np.arange(cfg.d, dtype=np.uint8), perm_gpu.shape))
    U.assert_close(o_gpu, np.broadcast_to(v.astype(np.float64).mean(2, keepdims=True), o_gpu.shape), "bf16", "uniform")
    # duplicated channel columns in q (each distinct column twice): the approximation is exact (Eq. 1)
    rng = np.random.default_rng(9)
    place = rng.permutation(cfg.d)
    qd = q.copy()
    qd[..., place[1::2]] = qd[..., place[0::2]]
    p = U.oracle_params(cfg)
    o_gpu, _, _ = U.run_gpu(cfg, qd, k, v, distr=True)
    U.assert_close(o_gpu, oracle.distr_fwd(qd, k, v, p), "bf16", "dup vs oracle distr")
    hashes = oracle.lsh_group(qd, p)[0]
    if all(len(set(hashes[0, h, t].tolist())) == cfg.d // 2 for h in range(2) for t in range(cfg.Tq)):
        U.assert_close(o_gpu, oracle.exact_fwd(qd, k, v, p), "bf16", "dup vs oracle exact")


@pytest.mark.parametrize("base,kw", [("vit", dict(B=1, H=2, Hkv=2, N=128)), ("llama", dict(H=2, Hkv=1, N=384)),
                                     ("llama", dict(H=2, Hkv=1, N=300, Br=256)), ("mid", dict(B=1, H=1, Hkv=1, N=256))])
def test_projections_that_nearly_cancel(base, kw):
    """Columns built so that one projection of every channel sums to almost nothing (signs chosen
    greedily against the running sum, the last rows sized to cancel what is left): the sign of
    such a sum is decided by the rounding of the defining float chain, and the kernel must take
    it that way too -- its matrix-pipe estimate is only trusted away from zero."""
    U = _util()
    import paper_2507_17245_amd as da
    cfg = small(base, **kw)
    q, k, v = W.make(cfg)
    R = da.distr_attn_hyperplanes(cfg.lsh_seed, cfg.n_planes, cfg.Br).astype(np.float64)
    for t in range(cfg.Tq):
        r0, rows = t * cfg.Br, min(cfg.Br, cfg.N - t * cfg.Br)
        for c in range(cfg.d):
            w = R[c % cfg.n_planes, :rows]
            col, run = np.zeros(rows), 0.0
            for r in range(rows):
                if r >= rows - 3 and abs(w[r]) > 0.1:      # closing rows: cancel the rest as well as bf16 allows
                    col[r] = float(W.round_to_bf16(np.array([-run / w[r]], dtype=np.float32))[0])
                else:
                    col[r] = -1.0 if run * w[r] > 0 else 1.0
                run += col[r] * w[r]
            q[:, :, r0:r0 + rows, c] = col
    p = U.oracle_params(cfg)
    hash_ref, perm_ref, proj = oracle.lsh_group(q, p, want_proj=True)
    near_zero = 0
    for c in range(cfg.d):
        near_zero += int((np.abs(proj[..., c, c % cfg.n_planes]) < 1e-4).sum())
    print(f"  {near_zero} of {proj[..., 0].size} targeted sums are below 1e-4 (sum |q||R| is around {0.45 * cfg.Br:.0f})", flush=True)
    assert near_zero > proj[..., 0].size // 2
    o_gpu, perm_gpu, hash_gpu = U.run_gpu(cfg, q, k, v, distr=True, want_tables=True)
    assert np.array_equal(hash_gpu, hash_ref) and np.array_equal(perm_gpu, perm_ref)
    o_self, perm_self, _ = U.run_gpu(cfg, q, k, v, distr=True, want_perm_only=True)    # the attention kernel's own LSH stage
    assert np.array_equal(perm_self, perm_ref), "table of the attention kernel's own LSH stage differs"
    assert np.array_equal(o_self, o_gpu), "in-kernel LSH and LSH kernel disagree"
    U.assert_close(o_gpu, oracle.distr_fwd(q, k, v, p), cfg.dtype, "near-cancelling projections")


def test_runs_are_deterministic_and_short_form_agrees():
    import torch
    import paper_2507_17245_amd as da
    U = _util()
    cfg = small("llama", H=4, Hkv=2, N=600)
    q, k, v = W.make(cfg)
    a, _, _ = U.run_gpu(cfg, q, k, v, distr=True)
    b, _, _ = U.run_gpu(cfg, q, k, v, distr=True)
    assert np.array_equal(a, b)
    tq, tk, tv = (U.to_dev(x, "bf16") for x in (q, k, v))
    o = torch.empty_like(tq)
    da.distr_attn_fwd(tq, tk, tv, o, cfg.Br, cfg.Bc, cfg.n_groups, cfg.lsh_seed, cfg.causal)
    torch.cuda.synchronize()
    assert np.array_equal(o.float().cpu().numpy().astype(np.float64), a)
    oe = torch.empty_like(tq)
    da.distr_attn_exact_fwd(tq, tk, tv, oe, cfg.Br, cfg.Bc, cfg.causal)
    torch.cuda.synchronize()
    e, _, _ = U.run_gpu(cfg, q, k, v, distr=False)
    assert np.array_equal(oe.float().cpu().numpy().astype(np.float64), e)
    # caller-provided workspace gives the same result as the library-owned one
    ws = torch.empty(da.distr_attn_workspace_bytes(da.make_params(tq, tk, tv, Br=cfg.Br, n_groups=cfg.n_groups)),
                     dtype=torch.uint8, device="cuda")
    p = da.make_params(tq, tk, tv, Br=cfg.Br, n_groups=cfg.n_groups, causal=cfg.causal, workspace=ws)
    o2 = torch.empty_like(tq)
    da.distr_attn_fwd_ex(tq, tk, tv, o2, p)
    torch.cuda.synchronize()
    assert torch.equal(o2, o)


def test_key_prepass_is_an_exact_transpose_and_kt_in_is_honoured():
    import torch
    import paper_2507_17245_amd as da
    U = _util()
    cfg = small("mid", B=2, H=4, Hkv=2, N=200)
    q, k, v = W.make(cfg)
    tq, tk, tv = (U.to_dev(x, "bf16") for x in (q, k, v))
    p = da.make_params(tq, tk, tv, Br=cfg.Br, n_groups=cfg.n_groups)
    kt = torch.zeros(da.distr_attn_kt_bytes(p), dtype=torch.uint8, device="cuda")
    da.distr_attn_key_prepass(tk, kt, p)
    torch.cuda.synchronize()
    npad = (cfg.N + 127) // 128 * 128
    got = kt[:cfg.B * cfg.Hkv * cfg.d * npad * 2].view(torch.float16).view(cfg.B, cfg.Hkv, cfg.d, npad).float().cpu().numpy()
    assert np.array_equal(got[..., :cfg.N], np.swapaxes(k, 2, 3))      # bf16 -> half is exact here
    assert not got[..., cfg.N:].any()                                  # zero-filled tail
    # values beyond half's range are clamped to +-65504 / G*
    big = tk.clone()
    big[0, 0, 0, 0] = 1e6
    big[0, 0, 1, 1] = -1e6
    da.distr_attn_key_prepass(big, kt, p)
    torch.cuda.synchronize()
    g2 = kt[:cfg.B * cfg.Hkv * cfg.d * npad * 2].view(torch.float16).view(cfg.B, cfg.Hkv, cfg.d, npad)
    lim = 65504.0 / (cfg.d // cfg.n_groups)
    assert float(g2[0, 0, 0, 0]) == np.float16(lim) and float(g2[0, 0, 1, 1]) == -np.float16(lim)
    # a forward with caller-provided kt equals the forward that runs the pre-pass itself
    da.distr_attn_key_prepass(tk, kt, p)
    o1, o2 = torch.empty_like(tq), torch.empty_like(tq)
    da.distr_attn_fwd_ex(tq, tk, tv, o1, p)
    da.distr_attn_fwd_ex(tq, tk, tv, o2, da.make_params(tq, tk, tv, Br=cfg.Br, n_groups=cfg.n_groups, kt_in=kt))
    torch.cuda.synchronize()
    assert torch.equal(o1, o2)
    # behind the copy: the projection matrix of the LSH stage (Sec. 3.2) for this call's seed,
    # projection count and block rows, as two bf16 pieces that add up to it exactly
    off = cfg.B * cfg.Hkv * cfg.d * npad * 2
    head = kt[off:off + 16].cpu().numpy()
    assert int(head[:8].view(np.uint64)[0]) == cfg.lsh_seed and head[8:16].view(np.int32).tolist() == [16, cfg.Br]
    piece = (16 * (cfg.Br + 8) * 2 + 1023) // 1024 * 1024
    both = kt[off + 1024:off + 1024 + 2 * piece].view(torch.bfloat16).float().cpu().numpy().reshape(2, piece // 2)
    rp = both[:, :16 * (cfg.Br + 8)].reshape(2, 16, cfg.Br + 8)[:, :, :cfg.Br]
    assert np.array_equal(rp[0] + rp[1], da.distr_attn_hyperplanes(cfg.lsh_seed, 16, cfg.Br))
    # d = 64, where the attention kernel's own LSH stage reads that table: one made for another
    # seed or block height is recognised by its header and not used
    cfg = small("llama", H=4, Hkv=2, N=300)
    q, k, v = W.make(cfg)
    tq, tk, tv = (U.to_dev(x, "bf16") for x in (q, k, v))
    common = dict(Br=cfg.Br, n_groups=cfg.n_groups, causal=True)
    p = da.make_params(tq, tk, tv, **common)
    o_ref = torch.empty_like(tq)
    da.distr_attn_fwd_ex(tq, tk, tv, o_ref, p)
    kt = torch.zeros(da.distr_attn_kt_bytes(p), dtype=torch.uint8, device="cuda")
    for other in (dict(lsh_seed=7), dict(Br=64), dict(n_planes=8), dict()):
        da.distr_attn_key_prepass(tk, kt, da.make_params(tq, tk, tv, **{**common, **other}))
        o = torch.empty_like(tq)
        da.distr_attn_fwd_ex(tq, tk, tv, o, da.make_params(tq, tk, tv, kt_in=kt, **common))
        torch.cuda.synchronize()
        assert torch.equal(o, o_ref), other


def test_side_stream_and_back_to_back_calls():
    """Calls are asynchronous on the given stream: several forwards queued on a side stream without
    host synchronisation in between (library-owned workspace reused) give the same results as
    isolated calls."""
    import torch
    import paper_2507_17245_amd as da
    U = _util()
    cfgs = [small("mid", B=1, H=2, Hkv=2, N=300, n_groups=64), small("vit", B=1, H=4, Hkv=4, N=130)]
    data = [W.make(c) for c in cfgs]
    expect = [U.run_gpu(c, *d, distr=True)[0] for c, d in zip(cfgs, data)]
    side = torch.cuda.Stream()
    outs = []
    with torch.cuda.stream(side):
        for _ in range(3):
            for c, (q, k, v) in zip(cfgs, data):
                tq, tk, tv = (U.to_dev(x, "bf16") for x in (q, k, v))
                o = torch.empty_like(tq)
                p = da.make_params(tq, tk, tv, Br=c.Br, n_groups=c.n_groups, causal=c.causal, lsh_seed=c.lsh_seed)
                assert p.stream == side.cuda_stream
                da.distr_attn_fwd_ex(tq, tk, tv, o, p)
                outs.append(o)
    side.synchronize()
    for i, o in enumerate(outs):
        assert np.array_equal(o.float().cpu().numpy().astype(np.float64), expect[i % 2])


def test_forward_replays_from_a_hip_graph():
    """With a caller-provided workspace a forward is launches only (no allocation, no host
    synchronisation, no memset), so it can be captured once and replayed: every replay, with the
    program's own eager work and synchronisations in between, must equal the eager result on the
    inputs of that moment."""
    import torch
    import paper_2507_17245_amd as da
    U = _util()
    for cfg in (small("mid", B=1, H=2, Hkv=2, N=300, n_groups=64), small("llama", H=8, Hkv=2, N=333)):
        q, k, v = W.make(cfg)
        tq, tk, tv = (U.to_dev(x, "bf16") for x in (q, k, v))
        o_graph, o_eager = torch.empty_like(tq), torch.empty_like(tq)
        common = dict(Br=cfg.Br, n_groups=cfg.n_groups, causal=cfg.causal, lsh_seed=cfg.lsh_seed)
        ws_bytes = da.distr_attn_workspace_bytes(da.make_params(tq, tk, tv, **common))
        ws_graph = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
        ws_eager = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.graph(graph, stream=side):
            da.distr_attn_fwd_ex(tq, tk, tv, o_graph, da.make_params(tq, tk, tv, workspace=ws_graph, **common))
        torch.cuda.synchronize()
        gen = torch.Generator(device="cuda").manual_seed(5)
        for rep in range(4):
            if rep:   # new inputs in the captured buffers
                for t in (tq, tk, tv):
                    t.copy_(torch.randn(t.shape, device="cuda", generator=gen).to(torch.bfloat16))
            o_graph.fill_(float("nan"))
            da.distr_attn_fwd_ex(tq, tk, tv, o_eager, da.make_params(tq, tk, tv, workspace=ws_eager, **common))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(o_graph.view(torch.int16), o_eager.view(torch.int16)), (cfg.name, rep)
