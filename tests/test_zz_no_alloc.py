"""The entry point that allocates nothing (distr_attn_fwd_noalloc) against distr_attn_fwd_ex, which
it shares its kernels with: same output bit for bit, on two calls in a row (the second on a smaller
input, so stale contents of the shared scratch array would show), on both ways through the LSH
stage, and no device allocation while it runs."""
import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu


def small(name, **kw):
    return W.CONFIGS[name].scaled(**kw)


def test_no_alloc_entry_matches_the_allocating_one():
    import torch
    import gpu_util as U
    import oracle
    import paper_2507_17245_amd as da
    cases = [small("llama", H=8, Hkv=2, N=700), small("llama", H=4, Hkv=2, N=333),        # second call: smaller
             small("mid", B=1, H=2, Hkv=2, N=520), small("vit", B=2, H=3, Hkv=3, N=130)]
    for want_tables in (False, True):     # LSH stage inside the attention kernel / as its own kernel (table in the scratch)
        for cfg in cases:
            q, k, v = W.make(cfg)
            tq, tk, tv = (U.to_dev(x, "bf16") for x in (q, k, v))
            common = dict(Br=cfg.Br, n_groups=cfg.n_groups, causal=cfg.causal, lsh_seed=cfg.lsh_seed)
            hsh = torch.zeros((cfg.B, cfg.H, cfg.Tq, cfg.d), dtype=torch.int32, device="cuda") if want_tables else None
            o_ref = torch.full_like(tq, float("nan"))
            da.distr_attn_fwd_ex(tq, tk, tv, o_ref, da.make_params(tq, tk, tv, hash_out=hsh, **common))
            torch.cuda.synchronize()
            o = torch.full_like(tq, float("nan"))
            p = da.make_params(tq, tk, tv, hash_out=hsh, **common)
            print(f"case {cfg} tables={want_tables}", flush=True)
            # torch's allocator counts every allocation it ever served; tensors of earlier tests
            # may be collected meanwhile, so the bytes in use can only be compared one way
            events = torch.cuda.memory_stats()["allocation.all.allocated"]
            before = torch.cuda.memory_allocated()
            da.distr_attn_fwd_noalloc(tq, tk, tv, o, p)
            torch.cuda.synchronize()
            assert torch.cuda.memory_stats()["allocation.all.allocated"] == events
            assert torch.cuda.memory_allocated() <= before
            assert torch.equal(o.view(torch.int16), o_ref.view(torch.int16)), (cfg.name, want_tables)
            op = U.oracle_params(cfg)
            U.assert_close(o.float().cpu().numpy().astype(np.float64), oracle.distr_fwd(q, k, v, op), "bf16", "no-alloc vs oracle")


def test_no_alloc_entry_refuses_what_does_not_fit():
    import torch
    import paper_2507_17245_amd as da
    limit = da.distr_attn_noalloc_max_bytes()
    assert limit == 32 << 20
    # K^T of this problem: 1 * 8 * 128 * 20480 * 2 bytes = 40 MiB > 32 MiB
    B, H, N, d = 1, 8, 20480, 128
    q = torch.zeros((B, H, N, d), dtype=torch.bfloat16, device="cuda")
    o = torch.empty_like(q)
    p = da.make_params(q, q, q, Br=128, n_groups=64)
    assert da.distr_attn_kt_bytes(p) > limit
    with pytest.raises(da.DistrAttnError) as e:
        da.distr_attn_fwd_noalloc(q, q, q, o, p)
    assert e.value.code == da.DA_ERR_WORKSPACE
    # with the caller's own K^T the rest of the scratch fits
    kt = torch.empty(da.distr_attn_kt_bytes(p), dtype=torch.uint8, device="cuda")
    da.distr_attn_key_prepass(q, kt, p)
    da.distr_attn_fwd_noalloc(q, q, q, o, da.make_params(q, q, q, Br=128, n_groups=64, kt_in=kt))
    torch.cuda.synchronize()
    assert torch.isfinite(o.float()).all()
