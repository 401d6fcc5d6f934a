"""Python binding of libdistr_attn.so (DistrAttention forward for MI355X / gfx950).

Argument marshalling only: every step of the path runs in the library's HIP kernels.
Tensors are torch tensors on the GPU (torch provides device memory and streams, nothing
else); names mirror the C entry points declared in include/distr_attn.h. There is no
fallback: a missing library or a failing call raises.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdistr_attn.so")

DA_OK, DA_ERR_INVALID_ARG, DA_ERR_UNSUPPORTED, DA_ERR_WORKSPACE, DA_ERR_HIP = 0, -1, -2, -3, -4
DA_BF16, DA_F32 = 0, 1

EXPORTS = (
    "distr_attn_fwd", "distr_attn_exact_fwd", "distr_attn_fwd_ex", "distr_attn_exact_fwd_ex",
    "distr_attn_fwd_noalloc", "distr_attn_noalloc_max_bytes",
    "distr_attn_bwd_ex", "distr_attn_exact_bwd_ex",
    "distr_attn_lsh_group", "distr_attn_key_prepass", "distr_attn_kt_bytes",
    "distr_attn_workspace_bytes", "distr_attn_bwd_workspace_bytes", "distr_attn_hyperplanes",
    "distr_attn_set_stream", "distr_attn_release", "distr_attn_last_error", "distr_attn_version",
)


class DaParams(ctypes.Structure):
    """Mirror of da_params."""
    _fields_ = [
        ("B", ctypes.c_int), ("H", ctypes.c_int), ("Hkv", ctypes.c_int), ("N", ctypes.c_int),
        ("d", ctypes.c_int), ("Br", ctypes.c_int), ("Bc", ctypes.c_int), ("n_groups", ctypes.c_int),
        ("causal", ctypes.c_int), ("lsh_seed", ctypes.c_uint64), ("dtype", ctypes.c_int),
        ("n_planes", ctypes.c_int), ("softmax_scale", ctypes.c_float), ("gray_mode", ctypes.c_int),
        ("stream", ctypes.c_void_p), ("workspace", ctypes.c_void_p),
        ("workspace_bytes", ctypes.c_size_t), ("perm_out", ctypes.c_void_p),
        ("hash_out", ctypes.c_void_p), ("perm_in", ctypes.c_void_p), ("kt_in", ctypes.c_void_p),
        ("Nk", ctypes.c_int), ("side", ctypes.c_int), ("lse_out", ctypes.c_void_p),
    ]


class DistrAttnError(RuntimeError):
    def __init__(self, code, message):
        super().__init__(f"distr_attn error {code}: {message}")
        self.code = code


_lib = None


def lib():
    """The loaded C library. Raises if it has not been built (python -m paper_2507_17245_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python paper_2507_17245_amd/build.py`")
        L = ctypes.CDLL(LIB_PATH)
        vp, ci, u64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64
        L.distr_attn_fwd.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, ci, u64, ci]
        L.distr_attn_exact_fwd.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, ci]
        L.distr_attn_noalloc_max_bytes.restype = ctypes.c_size_t
        for name in ("distr_attn_fwd_ex", "distr_attn_exact_fwd_ex", "distr_attn_fwd_noalloc"):
            getattr(L, name).argtypes = [vp, vp, vp, vp, ctypes.POINTER(DaParams)]
        for name in ("distr_attn_bwd_ex", "distr_attn_exact_bwd_ex"):
            getattr(L, name).argtypes = [vp] * 9 + [ctypes.POINTER(DaParams)]
        L.distr_attn_lsh_group.argtypes = [vp, ctypes.POINTER(DaParams)]
        L.distr_attn_key_prepass.argtypes = [vp, vp, ctypes.POINTER(DaParams)]
        for name in ("distr_attn_workspace_bytes", "distr_attn_bwd_workspace_bytes", "distr_attn_kt_bytes"):
            getattr(L, name).argtypes = [ctypes.POINTER(DaParams)]
            getattr(L, name).restype = ctypes.c_size_t
        L.distr_attn_hyperplanes.argtypes = [u64, ci, ci, ctypes.POINTER(ctypes.c_float)]
        L.distr_attn_set_stream.argtypes = [vp]
        L.distr_attn_last_error.restype = ctypes.c_char_p
        L.distr_attn_version.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _check(rc):
    if rc != DA_OK:
        raise DistrAttnError(rc, lib().distr_attn_last_error().decode())


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def _current_stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_code(t):
    import torch
    if t.dtype == torch.bfloat16:
        return DA_BF16
    if t.dtype == torch.float32:
        return DA_F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _shapes(q, k, v):
    if q.dim() != 4 or k.dim() != 4 or tuple(v.shape) != tuple(k.shape):
        raise ValueError("q must be [B,H,N,d]; k, v must be [B,Hkv,Nk,d]")
    B, H, N, d = q.shape
    if k.shape[0] != B or k.shape[3] != d:
        raise ValueError("k, v do not match q")
    for t in (q, k, v):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("tensors must be contiguous and on the GPU")
    if not (q.dtype == k.dtype == v.dtype):
        raise TypeError("q, k, v must share a dtype")
    return B, H, k.shape[1], N, d


def _check_out(q, o):
    """o is written by the kernels with q's shape and element type: anything else would be
    written out of bounds on the device."""
    if tuple(o.shape) != tuple(q.shape) or o.dtype != q.dtype:
        raise ValueError("o must have the shape and dtype of q")
    if not o.is_cuda or not o.is_contiguous():
        raise ValueError("o must be contiguous and on the GPU")


def _check_buffer(t, name, min_bytes):
    """An optional device buffer the library reads or writes `min_bytes` of."""
    if t is None:
        return
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous and on the GPU")
    have = t.numel() * t.element_size()
    if have < min_bytes:
        raise ValueError(f"{name} holds {have} bytes, {min_bytes} needed")


def make_params(q, k, v, Br, Bc=64, n_groups=None, causal=False, lsh_seed=0, n_planes=0,
                softmax_scale=0.0, gray_mode=0, workspace=None, perm_out=None, hash_out=None,
                perm_in=None, kt_in=None, side=0, lse_out=None):
    """side=1: the mirrored form (sample K, fuse Q, one grouping per K block of Bc rows); the
    tables are then [B, Hkv, ceil(Nk/Bc), d]. Nk is taken from k's shape. lse_out: float32
    [B, H, N] that receives the rows' log-sum-exp (what a backward pass needs)."""
    B, H, Hkv, N, d = _shapes(q, k, v)
    Nk = k.shape[2]
    p = DaParams()
    p.B, p.H, p.Hkv, p.N, p.d, p.Br, p.Bc = B, H, Hkv, N, d, Br, Bc
    p.Nk = Nk
    p.side = side
    p.n_groups = d if n_groups is None else n_groups
    p.causal = int(bool(causal))
    p.lsh_seed = lsh_seed
    p.dtype = _dtype_code(q)
    p.n_planes = n_planes
    p.softmax_scale = softmax_scale
    p.gray_mode = gray_mode
    p.stream = _current_stream().value
    if side == 1:
        n_table = B * Hkv * ((Nk + Bc - 1) // Bc) * d if Bc > 0 else 0
    else:
        n_table = B * H * ((N + Br - 1) // Br) * d if Br > 0 else 0
    _check_buffer(workspace, "workspace", 0)
    _check_buffer(perm_out, "perm_out", n_table)
    _check_buffer(hash_out, "hash_out", 4 * n_table)
    _check_buffer(perm_in, "perm_in", n_table)
    if workspace is not None:
        p.workspace = workspace.data_ptr()
        p.workspace_bytes = workspace.numel() * workspace.element_size()
    p.perm_out = perm_out.data_ptr() if perm_out is not None else None
    p.hash_out = hash_out.data_ptr() if hash_out is not None else None
    p.perm_in = perm_in.data_ptr() if perm_in is not None else None
    p.kt_in = kt_in.data_ptr() if kt_in is not None else None
    if kt_in is not None:
        _check_buffer(kt_in, "kt_in", distr_attn_kt_bytes(p))
    if lse_out is not None:
        import torch
        if lse_out.dtype != torch.float32:
            raise TypeError("lse_out must be float32")
        _check_buffer(lse_out, "lse_out", 4 * B * H * N)
        p.lse_out = lse_out.data_ptr()
    return p


def distr_attn_fwd(q, k, v, o, Br, Bc, n_groups, lsh_seed=0, causal=False):
    """Short form: bf16, 16 projections, scale 1/sqrt(d), on torch's current stream."""
    B, H, Hkv, N, d = _shapes(q, k, v)
    if _dtype_code(q) != DA_BF16:
        raise TypeError("the short form takes bf16 tensors; use distr_attn_fwd_ex for float")
    _check_out(q, o)
    lib().distr_attn_set_stream(_current_stream())
    if k.shape[2] != N:
        raise ValueError("the short form takes N keys; use distr_attn_fwd_ex for Nk != N")
    _check(lib().distr_attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), B, H, Hkv, N, d, Br, Bc,
                                n_groups, lsh_seed, int(bool(causal))))
    return o


def distr_attn_exact_fwd(q, k, v, o, Br, Bc, causal=False):
    B, H, Hkv, N, d = _shapes(q, k, v)
    if _dtype_code(q) != DA_BF16:
        raise TypeError("the short form takes bf16 tensors; use distr_attn_exact_fwd_ex for float")
    _check_out(q, o)
    lib().distr_attn_set_stream(_current_stream())
    if k.shape[2] != N:
        raise ValueError("the short form takes N keys; use distr_attn_exact_fwd_ex for Nk != N")
    _check(lib().distr_attn_exact_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), B, H, Hkv, N, d, Br, Bc,
                                      int(bool(causal))))
    return o


def _check_ex(q, k, v, o, params):
    B, H, Hkv, N, d = _shapes(q, k, v)
    _check_out(q, o)
    if (params.B, params.H, params.Hkv, params.N, params.d, params.dtype, params.Nk or N) != \
            (B, H, Hkv, N, d, _dtype_code(q), k.shape[2]):
        raise ValueError("params were made for tensors of another shape or dtype")


def distr_attn_fwd_ex(q, k, v, o, params):
    _check_ex(q, k, v, o, params)
    _check(lib().distr_attn_fwd_ex(_ptr(q), _ptr(k), _ptr(v), _ptr(o), ctypes.byref(params)))
    return o


def distr_attn_fwd_noalloc(q, k, v, o, params):
    """distr_attn_fwd_ex on the library's fixed scratch array: allocates nothing."""
    _check_ex(q, k, v, o, params)
    _check(lib().distr_attn_fwd_noalloc(_ptr(q), _ptr(k), _ptr(v), _ptr(o), ctypes.byref(params)))
    return o


def distr_attn_noalloc_max_bytes():
    return int(lib().distr_attn_noalloc_max_bytes())


def distr_attn_exact_fwd_ex(q, k, v, o, params):
    _check_ex(q, k, v, o, params)
    _check(lib().distr_attn_exact_fwd_ex(_ptr(q), _ptr(k), _ptr(v), _ptr(o), ctypes.byref(params)))
    return o


def _bwd(name, q, k, v, o, dout, lse, dq, dk, dv, params):
    import torch
    _check_ex(q, k, v, o, params)
    _check_out(q, dout)
    _check_out(q, dq)
    _check_out(k, dk)
    _check_out(k, dv)
    if lse.dtype != torch.float32:
        raise TypeError("lse must be float32")
    _check_buffer(lse, "lse", 4 * params.B * params.H * params.N)
    _check(getattr(lib(), name)(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(dout), _ptr(lse), _ptr(dq), _ptr(dk),
                                _ptr(dv), ctypes.byref(params)))
    return dq, dk, dv


def distr_attn_bwd_ex(q, k, v, o, dout, lse, dq, dk, dv, params):
    """Backward of distr_attn_fwd_ex (bf16 tensors: matrix-core kernels; float tensors: float
    arithmetic): fills dq, dk, dv. o and lse are the forward's output and lse_out."""
    return _bwd("distr_attn_bwd_ex", q, k, v, o, dout, lse, dq, dk, dv, params)


def distr_attn_exact_bwd_ex(q, k, v, o, dout, lse, dq, dk, dv, params):
    return _bwd("distr_attn_exact_bwd_ex", q, k, v, o, dout, lse, dq, dk, dv, params)


def distr_attn_lsh_group(q, params):
    _check(lib().distr_attn_lsh_group(_ptr(q), ctypes.byref(params)))


def distr_attn_key_prepass(k, kt_out, params):
    if not k.is_cuda or not k.is_contiguous():
        raise ValueError("k must be contiguous and on the GPU")
    _check_buffer(kt_out, "kt_out", distr_attn_kt_bytes(params))
    _check(lib().distr_attn_key_prepass(_ptr(k), _ptr(kt_out), ctypes.byref(params)))
    return kt_out


def distr_attn_kt_bytes(params):
    return int(lib().distr_attn_kt_bytes(ctypes.byref(params)))


def distr_attn_workspace_bytes(params):
    return int(lib().distr_attn_workspace_bytes(ctypes.byref(params)))


def distr_attn_bwd_workspace_bytes(params):
    return int(lib().distr_attn_bwd_workspace_bytes(ctypes.byref(params)))


def distr_attn_hyperplanes(seed, n_planes, Br):
    """-> numpy float32 [n_planes, Br] (host): the projection matrix the kernels generate."""
    import numpy as np
    out = np.empty((n_planes, Br), dtype=np.float32)
    _check(lib().distr_attn_hyperplanes(seed, n_planes, Br,
                                        out.ctypes.data_as(ctypes.POINTER(ctypes.c_float))))
    return out


def distr_attn_release():
    _check(lib().distr_attn_release())


def distr_attn_version():
    return lib().distr_attn_version().decode()
