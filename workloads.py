"""Seeded synthetic inputs for the five benchmark configurations.

Shared by the tests, the oracle legs and the GPU legs. Holds no arithmetic of the
method itself: only random draws, the value structure each configuration asks for,
and rounding to bf16-representable floats. Every tensor is a float32 numpy array
(q: [B,H,N,d]; k, v: [B,Hkv,N,d]); bf16 configurations hold values that a bf16
stores exactly, so the oracle (float in, double arithmetic) and the GPU path
(bf16 in) see the same numbers.

The configurations stand in for the paper's attention-only timing workloads
(random tensors of ViT-B/16, Llama-1B and long-sequence shapes, Sec. 4.5, 4.7, 4.8).
"""
from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Config:
    name: str
    B: int
    H: int
    Hkv: int
    N: int
    d: int
    dtype: str        # "bf16" or "f32"
    causal: bool
    Br: int
    Bc: int
    n_groups: int
    n_planes: int
    recipe: str       # value structure, see make()
    data_seed: int
    lsh_seed: int = 0
    Nk: int = 0       # keys / values per head; 0 = N (decode against a cache, cross attention: Nk != N)
    side: int = 0     # 1 = the mirrored form (sample K, fuse Q, one grouping per K block of Bc rows)

    @property
    def n_keys(self):
        return self.Nk if self.Nk > 0 else self.N

    @property
    def Tk(self):
        return (self.n_keys + self.Bc - 1) // self.Bc

    @property
    def Tq(self):
        return (self.N + self.Br - 1) // self.Br

    def exact_flops(self):
        """4*B*H*N^2*d: the FLOP count of exact attention, the unit of the headline metric."""
        return 4.0 * self.B * self.H * float(self.N) ** 2 * self.d

    def scaled(self, **kw):
        return replace(self, **kw)


CONFIGS = {
    "tiny": Config("tiny", 1, 1, 1, 256, 64, "f32", False, 64, 64, 32, 4, "latent_pairs", 1000),
    "vit": Config("vit", 64, 12, 12, 197, 64, "bf16", False, 64, 64, 32, 16, "noisy_copies", 1001),
    "llama": Config("llama", 1, 32, 8, 4096, 64, "bf16", True, 128, 64, 32, 16, "channel_scales", 1002),
    "mid": Config("mid", 4, 16, 16, 8192, 128, "bf16", False, 128, 64, 64, 16, "rho_pairs", 1003),
    "long": Config("long", 1, 16, 16, 32768, 128, "bf16", True, 128, 64, 64, 16, "low_rank", 1004),
}
MID_GROUP_SWEEP = (128, 64, 32)


def round_to_bf16(x):
    """Nearest-even rounding of float32 values to the bf16 grid, returned as float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def _normal(rng, shape):
    return rng.standard_normal(shape, dtype=np.float32)


def make(cfg: Config):
    """-> (q, k, v) float32 arrays for the configuration, deterministic in cfg.data_seed."""
    rng = np.random.default_rng(cfg.data_seed)
    B, H, Hkv, N, d = cfg.B, cfg.H, cfg.Hkv, cfg.N, cfg.d
    qs, ks = (B, H, N, d), (B, Hkv, cfg.n_keys, d)
    pi = rng.permutation(d)  # partner channels are not index neighbours
    if cfg.recipe == "latent_pairs":
        # d/2 latent columns per head; channels pi[2p], pi[2p+1] = latent p + 0.1 noise each
        def paired(shape):
            z = _normal(rng, shape[:-1] + (d // 2,))
            x = np.empty(shape, dtype=np.float32)
            x[..., pi[0::2]] = z + 0.1 * _normal(rng, z.shape)
            x[..., pi[1::2]] = z + 0.1 * _normal(rng, z.shape)
            return x
        q, k, v = paired(qs), paired(ks), _normal(rng, ks)
    elif cfg.recipe == "noisy_copies":
        # a quarter of the channels are noisy copies (sigma 0.1) of distinct other channels;
        # the same pairing in q, k and v
        n_copy = d // 4
        dst, src = pi[:n_copy], pi[n_copy:2 * n_copy]
        def copied(shape):
            x = _normal(rng, shape)
            x[..., dst] = x[..., src] + 0.1 * _normal(rng, shape[:-1] + (n_copy,))
            return x
        q, k, v = copied(qs), copied(ks), copied(ks)
    elif cfg.recipe == "channel_scales":
        # N(0,1) * (1 + s), s ~ LogNormal(0, 0.5) per (head, channel)
        sq = rng.lognormal(0.0, 0.5, size=(1, H, 1, d)).astype(np.float32)
        sk = rng.lognormal(0.0, 0.5, size=(1, Hkv, 1, d)).astype(np.float32)
        q = _normal(rng, qs) * (1.0 + sq)
        k = _normal(rng, ks) * (1.0 + sk)
        v = _normal(rng, ks)
    elif cfg.recipe == "rho_pairs":
        # channel pairs with correlation 0.9: x_a = z, x_b = 0.9 z + sqrt(1 - 0.81) noise
        def corr(shape):
            x = _normal(rng, shape)
            a, b = pi[0::2], pi[1::2]
            x[..., b] = 0.9 * x[..., a] + np.float32(np.sqrt(1.0 - 0.81)) * x[..., b]
            return x
        q, k, v = corr(qs), corr(ks), _normal(rng, ks)
    elif cfg.recipe == "low_rank":
        # rank-32 component shared by q and k of a head (same mixing matrix) + 0.3 noise
        rank = 32
        def lowrank(shape, w):  # w: [heads, rank, d]
            x = np.empty(shape, dtype=np.float32)
            for b in range(shape[0]):
                for h in range(shape[1]):
                    x[b, h] = _normal(rng, (shape[2], rank)) @ w[h] + 0.3 * _normal(rng, (shape[2], d))
            return x
        w = _normal(rng, (H, rank, d)) / np.float32(np.sqrt(rank))
        q = lowrank(qs, w)
        k = lowrank(ks, w[:: H // Hkv])
        v = _normal(rng, ks)
    elif cfg.recipe == "uniform":
        # U(0,1) entries: the paper's own synthetic data (Sec. 4.2, 4.7, 4.8)
        q = rng.random(qs, dtype=np.float32)
        k = rng.random(ks, dtype=np.float32)
        v = rng.random(ks, dtype=np.float32)
    elif cfg.recipe == "normal":
        q, k, v = _normal(rng, qs), _normal(rng, ks), _normal(rng, ks)
    else:
        raise ValueError(f"unknown recipe {cfg.recipe}")
    if cfg.dtype == "bf16":
        q, k, v = round_to_bf16(q), round_to_bf16(k), round_to_bf16(v)
    return q, k, v


def make_grad(cfg: Config):
    """-> dout float32 [B, H, N, d]: a seeded N(0,1) output gradient for the backward-pass tests."""
    rng = np.random.default_rng(cfg.data_seed + 4242)
    g = _normal(rng, (cfg.B, cfg.H, cfg.N, cfg.d))
    return round_to_bf16(g) if cfg.dtype == "bf16" else g


def sample_tiles(cfg: Config, n_random=3, batch=0, heads=None):
    """Deterministic sample of Q blocks (b, h, t): first two, middle, last two and a few seeded
    random ones, for every head in `heads` (default: all) of one batch entry."""
    Tq = cfg.Tq
    base = sorted({0, min(1, Tq - 1), Tq // 2, max(Tq - 2, 0), Tq - 1})
    rng = np.random.default_rng(cfg.data_seed + 77)
    extra = [int(t) for t in rng.integers(0, Tq, size=n_random)] if Tq > len(base) else []
    ts = sorted(set(base) | set(extra))
    heads = range(cfg.H) if heads is None else heads
    return [(batch, h, t) for h in heads for t in ts]
