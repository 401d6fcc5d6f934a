"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every declared
symbol, rejects bad arguments before touching a device, and its projection-matrix generator
agrees with the oracle's independently written one."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2507_17245_amd as da

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "distr_attn.h")).read()
    declared = set(re.findall(r"\b(distr_attn_\w+)\s*\(", header))
    assert declared == set(da.EXPORTS)
    L = da.lib()
    for name in declared:
        assert getattr(L, name) is not None
    assert "gfx950" in da.distr_attn_version()


def test_struct_layout_matches_header_order():
    header = open(os.path.join(ROOT, "include", "distr_attn.h")).read()
    body = header[header.index("typedef struct {"):header.index("} da_params;")]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    names = []
    for decl in body.split("{", 1)[1].split(";"):
        decl = decl.strip()
        if not decl:
            continue
        for part in decl.split(","):
            names.append(re.findall(r"(\w+)\s*$", part.strip())[0])
    assert names == [f[0] for f in da.DaParams._fields_]


def test_hyperplanes_match_the_oracle_generator():
    for seed, planes, Br in [(0, 16, 128), (7, 4, 64), (2 ** 63 + 5, 32, 128), (123456789, 1, 1)]:
        assert np.array_equal(da.distr_attn_hyperplanes(seed, planes, Br), oracle.hyperplanes(seed, planes, Br))


def _params(**kw):
    base = dict(B=1, H=4, Hkv=2, N=100, d=64, Br=64, Bc=64, n_groups=32, causal=0, lsh_seed=0,
                dtype=da.DA_BF16, n_planes=0, softmax_scale=0.0, gray_mode=0)
    base.update(kw)
    p = da.DaParams()
    for k, v in base.items():
        setattr(p, k, v)
    return p


FAKE = ctypes.c_void_p(0x1000)   # never dereferenced: every check below fails on the host first
FAKE_O = ctypes.c_void_p(0x2000)


@pytest.mark.parametrize("kw,code", [
    (dict(B=0), da.DA_ERR_INVALID_ARG),
    (dict(N=-3), da.DA_ERR_INVALID_ARG),
    (dict(H=3, Hkv=2), da.DA_ERR_INVALID_ARG),
    (dict(n_groups=24), da.DA_ERR_INVALID_ARG),          # 64 % 24 != 0: groups have a constant size
    (dict(n_groups=0), da.DA_ERR_INVALID_ARG),
    (dict(dtype=5), da.DA_ERR_INVALID_ARG),
    (dict(causal=2), da.DA_ERR_INVALID_ARG),
    (dict(gray_mode=3), da.DA_ERR_INVALID_ARG),
    (dict(softmax_scale=-1.0), da.DA_ERR_INVALID_ARG),
    (dict(d=96, n_groups=48), da.DA_ERR_UNSUPPORTED),
    (dict(Br=32), da.DA_ERR_UNSUPPORTED),
    (dict(Bc=96), da.DA_ERR_UNSUPPORTED),
    (dict(Br=512), da.DA_ERR_UNSUPPORTED),
    (dict(Bc=32, n_groups=8), da.DA_ERR_UNSUPPORTED),     # tiles other than 64 rows: 16, 32, 64 groups or d
    (dict(side=1, Bc=96), da.DA_ERR_UNSUPPORTED),         # the mirrored form: K blocks of 32, 64 or 128 rows
    (dict(side=2), da.DA_ERR_INVALID_ARG),
    (dict(Nk=50, causal=1), da.DA_ERR_INVALID_ARG),       # causal with fewer keys than queries
    (dict(Nk=-1), da.DA_ERR_INVALID_ARG),
    (dict(n_planes=33), da.DA_ERR_UNSUPPORTED),
    (dict(n_groups=2), da.DA_ERR_UNSUPPORTED),            # groups of 32 channels: more than the bf16 kernels take
    (dict(d=128, n_groups=4), da.DA_ERR_UNSUPPORTED),
    (dict(N=1 << 23, d=128, n_groups=64), da.DA_ERR_UNSUPPORTED),   # a head of 4 GiB: 32-bit tile offsets
])
def test_bad_arguments_fail_on_the_host(kw, code):
    p = _params(**kw)
    rc = da.lib().distr_attn_fwd_ex(FAKE, FAKE, FAKE, FAKE_O, ctypes.byref(p))
    assert rc == code
    assert da.lib().distr_attn_last_error()


def test_pointer_checks():
    L = da.lib()
    p = _params()
    assert L.distr_attn_fwd_ex(None, FAKE, FAKE, FAKE_O, ctypes.byref(p)) == da.DA_ERR_INVALID_ARG
    assert L.distr_attn_fwd_ex(FAKE, FAKE, FAKE, FAKE, ctypes.byref(p)) == da.DA_ERR_INVALID_ARG      # o aliases q
    assert L.distr_attn_fwd_ex(ctypes.c_void_p(0x1004), FAKE, FAKE, FAKE_O, ctypes.byref(p)) == da.DA_ERR_INVALID_ARG
    assert L.distr_attn_exact_fwd_ex(FAKE, FAKE, FAKE, FAKE_O, None) == da.DA_ERR_INVALID_ARG
    assert L.distr_attn_lsh_group(FAKE, ctypes.byref(p)) == da.DA_ERR_INVALID_ARG                     # no output given
    assert L.distr_attn_fwd(FAKE, FAKE, FAKE, FAKE_O, 1, 4, 3, 64, 64, 64, 64, 32, 0, 0) == da.DA_ERR_INVALID_ARG
    assert L.distr_attn_exact_fwd(FAKE, FAKE, FAKE, FAKE_O, 1, 4, 2, 64, 80, 64, 64, 0) == da.DA_ERR_UNSUPPORTED
    assert L.distr_attn_hyperplanes(0, 16, 64, None) == da.DA_ERR_INVALID_ARG
    # caller workspace too small
    p = _params(workspace=0x3000, workspace_bytes=16)
    assert L.distr_attn_fwd_ex(FAKE, FAKE, FAKE, FAKE_O, ctypes.byref(p)) == da.DA_ERR_WORKSPACE


def test_workspace_bytes():
    p = _params(B=2, H=4, Hkv=4, N=197, d=64, Br=64)
    need = da.distr_attn_workspace_bytes(p)
    assert need >= 2 * 4 * 4 * 64 and need % 256 == 0
    assert da.distr_attn_workspace_bytes(_params(n_groups=7)) == 0


def test_backward_argument_checks_happen_on_the_host():
    L = da.lib()
    L.distr_attn_bwd_ex.argtypes = [ctypes.c_void_p] * 9 + [ctypes.POINTER(da.DaParams)]
    ptrs = [ctypes.c_void_p(0x10000 * (i + 1)) for i in range(9)]
    call = lambda p, a=ptrs: L.distr_attn_bwd_ex(*a, ctypes.byref(p))
    assert call(_params(side=1)) == da.DA_ERR_UNSUPPORTED                       # no backward of the mirrored form
    assert call(_params(N=1 << 24, d=128, n_groups=64)) == da.DA_ERR_UNSUPPORTED   # a head of 4 GiB
    assert call(_params(n_groups=24)) == da.DA_ERR_INVALID_ARG
    assert call(_params(), ptrs[:6] + [ptrs[0]] + ptrs[7:]) == da.DA_ERR_INVALID_ARG   # dq aliases q
    assert call(_params(), ptrs[:6] + [ptrs[6], ptrs[6], ptrs[8]]) == da.DA_ERR_INVALID_ARG   # dk is dq
    assert call(_params(), [None] + ptrs[1:]) == da.DA_ERR_INVALID_ARG


def test_backward_workspace_bytes():
    """Table + 8 bytes per query row + a copy of q; grouped-query shapes whose dK/dV launch is
    split over the query heads add float partial sums of dk and dv per query head of a kv head;
    float tensors need the table only."""
    al = lambda n: (n + 255) // 256 * 256
    B, H, N, d, Br = 2, 4, 197, 64, 64
    table = al(B * H * ((N + Br - 1) // Br) * d)
    rows = B * H * N
    mha = da.distr_attn_bwd_workspace_bytes(_params(B=B, H=H, Hkv=H, N=N, d=d, Br=Br))
    assert mha == table + 2 * al(rows * 4) + al(rows * d * 2)
    gqa = da.distr_attn_bwd_workspace_bytes(_params(B=B, H=H, Hkv=2, N=N, d=d, Br=Br))
    assert gqa == mha + al(2 * (H // 2) * B * 2 * N * d * 4)
    assert da.distr_attn_bwd_workspace_bytes(_params(B=B, H=H, Hkv=H, N=N, d=d, Br=Br, dtype=da.DA_F32)) == table
    assert da.distr_attn_bwd_workspace_bytes(_params(n_groups=7)) == 0


def test_bench_refuses_more_than_one_gpu_and_reads_its_traffic_figure():
    """Host logic of bench.py that needs no GPU: the one-GPU rule and the profile line it quotes."""
    import json
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                         capture_output=True, text=True, timeout=120)
    assert res.returncode != 0
    assert "ONE GPU" in (res.stdout + res.stderr)
    with open(os.path.join(root, "profiles", "attn_bf16_long_hbm_traffic.md")) as f:
        lines = [l for l in f if l.startswith("bench-traffic:")]
    assert len(lines) == 1
    rec = json.loads(lines[0].split(":", 1)[1])
    assert rec["workload"] == "long" and rec["hbm_bytes_per_launch"] > 5e8


class _FakeTensor:
    """Stand-in with the attributes the binding inspects; its pointer is never dereferenced because
    every case below is rejected by the binding before the library is called."""

    def __init__(self, shape, dtype=None, cuda=True, contiguous=True, itemsize=2):
        import torch
        self.shape = tuple(shape)
        self.dtype = torch.bfloat16 if dtype is None else dtype
        self.is_cuda = cuda
        self._contiguous = contiguous
        self._itemsize = itemsize

    def dim(self):
        return len(self.shape)

    def is_contiguous(self):
        return self._contiguous

    def numel(self):
        return int(np.prod(self.shape))

    def element_size(self):
        return self._itemsize

    def data_ptr(self):
        return 0x1000


def test_binding_rejects_bad_output_and_side_buffers(monkeypatch):
    """The binding checks o and the optional device buffers on the host: a small or strided buffer
    would otherwise be written or read past its end on the device."""
    import torch
    monkeypatch.setattr(da, "_current_stream", lambda: ctypes.c_void_p(0))
    q = _FakeTensor((1, 4, 100, 64))
    k = _FakeTensor((1, 2, 100, 64))
    good = dict(Br=64, n_groups=32)
    p = da.make_params(q, k, k, **good)
    for bad_o in (_FakeTensor((1, 4, 99, 64)), _FakeTensor((1, 4, 100, 64), dtype=torch.float32, itemsize=4),
                  _FakeTensor((1, 4, 100, 64), cuda=False), _FakeTensor((1, 4, 100, 64), contiguous=False)):
        for call in (lambda o: da.distr_attn_fwd_ex(q, k, k, o, p), lambda o: da.distr_attn_exact_fwd_ex(q, k, k, o, p),
                     lambda o: da.distr_attn_fwd(q, k, k, o, 64, 64, 32), lambda o: da.distr_attn_exact_fwd(q, k, k, o, 64, 64)):
            with pytest.raises(ValueError):
                call(bad_o)
    n_table = 1 * 4 * 2 * 64
    small = _FakeTensor((n_table - 1,), dtype=torch.uint8, itemsize=1)
    for name in ("perm_out", "perm_in"):
        with pytest.raises(ValueError, match=name):
            da.make_params(q, k, k, **good, **{name: small})
    with pytest.raises(ValueError, match="hash_out"):
        da.make_params(q, k, k, **good, hash_out=_FakeTensor((n_table - 1,), dtype=torch.int32, itemsize=4))
    with pytest.raises(ValueError, match="perm_out"):
        da.make_params(q, k, k, **good, perm_out=_FakeTensor((n_table,), dtype=torch.uint8, itemsize=1, cuda=False))
    with pytest.raises(ValueError, match="kt_in"):
        da.make_params(q, k, k, **good, kt_in=_FakeTensor((100,), dtype=torch.uint8, itemsize=1))
    # params made for other tensors are refused
    q2 = _FakeTensor((1, 4, 101, 64))
    k2 = _FakeTensor((1, 2, 101, 64))
    with pytest.raises(ValueError, match="another shape"):
        da.distr_attn_fwd_ex(q2, k2, k2, _FakeTensor((1, 4, 101, 64)), p)


def test_workspace_need_follows_what_the_call_writes():
    """kt_in removes the K^T copy from the scratch a call needs and perm_in / the in-kernel LSH
    stage remove the table: a workspace that only holds the rest is accepted (the call then fails
    later, on the host, at the misaligned kt_in -- nothing is launched)."""
    L = da.lib()
    p = _params(workspace=0x3000 << 8, workspace_bytes=16, kt_in=0x1001)
    assert L.distr_attn_fwd_ex(FAKE, FAKE, FAKE, FAKE_O, ctypes.byref(p)) == da.DA_ERR_INVALID_ARG
    assert b"kt_in" in L.distr_attn_last_error()
