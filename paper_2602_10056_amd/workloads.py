"""Seeded synthetic attention inputs shaped like the paper's workloads.

This module only draws random numbers and shapes them; it contains none of the
method's arithmetic and loads no native code, so both the HIP path and the CPU
oracle can be fed from it.  Every array is generated in float64 with
numpy.random.default_rng, rounded ONCE to the storage type (fp32 or bf16) and
returned as float32 holding exactly representable values, so both consumers
see identical numbers.

Workloads (Q: [batch, q_heads, m, d], K: [batch, kv_heads, n, d],
V: [batch, kv_heads, n, d_v]; m = n and d_v = d unless stated; beta = 1/sqrt(d)):

  1  one head, n=1024, d=64, r=64, fp32; i.i.d. N(0,1), keys scaled by 1/sqrt(d)
     (the Gaussian inputs of the paper's FlashAttention-2 study, Sec. 5.4)
  2  4 x 8 heads, n=4096, d=64, r=128, bf16; per head rank-32 Gaussian factor
     model plus 0.1 N(0,1) noise for each of Q, K, V
  3  16 heads, n=16384, d=128, r=256, bf16; keys and queries from a 64-component
     Gaussian mixture (unit-Gaussian centres, within-cluster sigma 0.25),
     values N(0,1): cluster-structured, ViT/diffusion-like token statistics
  4  32 query heads sharing 8 key/value heads, n=32768, d=128, r=512, bf16;
     N(0,1) entries, then a rotary position rotation of Q and K
  5  8 heads, n=131072, d=128, r=1024, bf16; keys with log-normal norms
     (sigma 0.5) times uniform directions, 16 leading "sink" keys of 4x norm
  6  binned (Sec. 2.5): 8 heads, n=65536, d=64, r=64 in B=16 bins, bf16; Q, K, V
     all i.i.d. N(0,1) -- the setting of the paper's FlashAttention-2 comparison
     (Sec. 5.4: d=64, r=64, B=16, n from 2^13 to 2^18; head count not stated)

  7  binned, m != n and d_v != d: the single attention layer of the paper's image
     generation benchmark (Sec. 5.1: Q 4096 x 64, K 1024 x 64, V 1024 x 256,
     r=96, B=8); 8 images x 1 head, fp32; tokens from a 64-component Gaussian
     mixture as in workload 3 (the benchmark's real activations need the model)
  8  binned with one pivot per bin: the first tokens-to-token layer of the
     paper's image classification benchmark (Sec. 5.2: n=m=3136, d=64,
     r=B=224, i.e. bins of 14 keys); 8 images x 1 head, fp32; mixture tokens

Shapes 1-5 use one bin (B = 1); `bins` can be overridden for any of them.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Shape:
    name: str
    batch: int
    q_heads: int
    kv_heads: int
    n: int
    d: int
    r: int
    dtype: str          # "f32" | "bf16"
    data_seed: int
    uniform_seed: int
    bins: int = 1       # B of Alg. 2
    m_: int = 0         # queries per head (0: n)
    dv_: int = 0        # value width (0: d)

    @property
    def m(self):
        return self.m_ or self.n

    @property
    def dv(self):
        return self.dv_ or self.d

    @property
    def problems(self):
        return self.batch * self.kv_heads

    @property
    def group(self):
        return self.q_heads // self.kv_heads

    @property
    def beta(self):
        return 1.0 / float(np.sqrt(self.d))


SHAPES = {
    1: Shape("cfg1_gauss_f32", 1, 1, 1, 1024, 64, 64, "f32", 0, 201),
    2: Shape("cfg2_lowrank_bf16", 4, 8, 8, 4096, 64, 128, "bf16", 102, 202),
    3: Shape("cfg3_mixture_bf16", 1, 16, 16, 16384, 128, 256, "bf16", 103, 203),
    4: Shape("cfg4_gqa_rope_bf16", 1, 32, 8, 32768, 128, 512, "bf16", 104, 204),
    5: Shape("cfg5_heavytail_bf16", 1, 8, 8, 131072, 128, 1024, "bf16", 105, 205),
    6: Shape("cfg6_gauss_binned_bf16", 1, 8, 8, 65536, 64, 64, "bf16", 106, 206, bins=16),
    7: Shape("cfg7_imagegen_layer_f32", 8, 1, 1, 1024, 64, 96, "f32", 107, 207, bins=8, m_=4096, dv_=256),
    8: Shape("cfg8_t2t_layer1_f32", 8, 1, 1, 3136, 64, 224, "f32", 108, 208, bins=224),
}


def shape(cfg, **override):
    """The catalogue shape `cfg`, optionally shrunk (n=, r=, batch=, q_heads=,
    kv_heads=, bins=) for tests that keep the recipe but not the size."""
    s = SHAPES[cfg]
    if override:
        fields = {k: getattr(s, k) for k in s.__dataclass_fields__}
        fields.update(override)
        s = Shape(**fields)
    if s.q_heads % s.kv_heads:
        raise ValueError("q_heads must be a multiple of kv_heads")
    if s.bins < 1 or s.n % s.bins or s.r % s.bins:
        raise ValueError("bins must divide n and r")
    return s


def round_to_storage(x, dtype):
    """float64 -> nearest value of the storage type (ties to even), as float32."""
    x32 = np.asarray(x, dtype=np.float64).astype(np.float32)
    if dtype == "f32":
        return x32
    if dtype != "bf16":
        raise ValueError(dtype)
    bits = x32.view(np.uint32).astype(np.uint64)
    bits = (bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000
    return bits.astype(np.uint32).view(np.float32).reshape(x32.shape)


def bf16_bits(x32):
    """The uint16 bit patterns of float32 values that are exactly bf16."""
    b = np.ascontiguousarray(x32, dtype=np.float32).view(np.uint32)
    if np.any(b & 0xFFFF):
        raise ValueError("values are not bf16-representable")
    return (b >> 16).astype(np.uint16)


def _rope(x, d):
    """Rotate coordinate pairs (2j, 2j+1) of row t by the angle t * 10000^(-2j/d)."""
    n = x.shape[-2]
    j = np.arange(d // 2)
    ang = np.arange(n)[:, None] * (10000.0 ** (-2.0 * j / d))[None, :]
    c, s = np.cos(ang), np.sin(ang)
    out = np.empty_like(x)
    out[..., 0::2] = x[..., 0::2] * c - x[..., 1::2] * s
    out[..., 1::2] = x[..., 0::2] * s + x[..., 1::2] * c
    return out


def _head_rng(s, kind, b, h):
    return np.random.default_rng([s.data_seed, kind, b, h])


def make_kv_head(cfg, s, b, h):
    """(K [n,d], V [n,dv]) of key/value head (b, h), storage-rounded float32."""
    g = _head_rng(s, 0, b, h)
    n, d, dv = s.n, s.d, s.dv
    if dv != d and cfg not in (3, 7, 8):
        raise ValueError("this recipe has d_v = d")
    if cfg == 1:
        K = g.standard_normal((n, d)) / np.sqrt(d)
        V = g.standard_normal((n, d))
    elif cfg == 2:
        K = g.standard_normal((n, 32)) @ (g.standard_normal((32, d)) / np.sqrt(32.0)) \
            + 0.1 * g.standard_normal((n, d))
        V = g.standard_normal((n, 32)) @ (g.standard_normal((32, d)) / np.sqrt(32.0)) \
            + 0.1 * g.standard_normal((n, d))
    elif cfg in (3, 7, 8):
        mu = _centres(s, b, h)
        K = mu[g.integers(0, 64, size=n)] + 0.25 * g.standard_normal((n, d))
        V = g.standard_normal((n, dv))
    elif cfg == 4:
        K = _rope(g.standard_normal((n, d)), d)
        V = g.standard_normal((n, d))
    elif cfg == 5:
        z = g.standard_normal(n)
        dirs = g.standard_normal((n, d))
        dirs /= np.linalg.norm(dirs, axis=1, keepdims=True)
        norms = np.sqrt(d) * np.exp(0.5 * z)
        norms[:min(16, n)] = 4.0 * np.sqrt(d)
        K = norms[:, None] * dirs
        V = g.standard_normal((n, d))
    elif cfg == 6:
        K = g.standard_normal((n, d))
        V = g.standard_normal((n, d))
    else:
        raise ValueError(cfg)
    return round_to_storage(K, s.dtype), round_to_storage(V, s.dtype)


def _centres(s, b, h_kv):
    return np.random.default_rng([s.data_seed, 2, b, h_kv]).standard_normal((64, s.d))


def make_q_head(cfg, s, b, hq):
    """Q [m,d] of query head (b, hq), storage-rounded float32."""
    g = _head_rng(s, 1, b, hq)
    n, d = s.m, s.d
    if cfg == 2:
        Q = g.standard_normal((n, 32)) @ (g.standard_normal((32, d)) / np.sqrt(32.0)) \
            + 0.1 * g.standard_normal((n, d))
    elif cfg in (3, 7, 8):
        mu = _centres(s, b, hq // s.group)
        Q = mu[g.integers(0, 64, size=n)] + 0.25 * g.standard_normal((n, d))
    elif cfg == 4:
        Q = _rope(g.standard_normal((n, d)), d)
    elif cfg in (1, 5, 6):
        Q = g.standard_normal((n, d))
    else:
        raise ValueError(cfg)
    return round_to_storage(Q, s.dtype)


def uniforms(s):
    """Pre-drawn pivot uniforms u[problems, r] in [0,1), one per RPNys step."""
    return np.random.default_rng(s.uniform_seed).random((s.problems, s.r))


def make(cfg, **override):
    """All tensors of workload `cfg`: dict with Q [B,Hq,m,d], K [B,Hkv,n,d], V [B,Hkv,n,dv]
    (float32 holding storage-exact values), u [B*Hkv, r], and the Shape."""
    s = shape(cfg, **override)
    Q = np.empty((s.batch, s.q_heads, s.m, s.d), dtype=np.float32)
    K = np.empty((s.batch, s.kv_heads, s.n, s.d), dtype=np.float32)
    V = np.empty((s.batch, s.kv_heads, s.n, s.dv), dtype=np.float32)
    for b in range(s.batch):
        for h in range(s.kv_heads):
            K[b, h], V[b, h] = make_kv_head(cfg, s, b, h)
        for h in range(s.q_heads):
            Q[b, h] = make_q_head(cfg, s, b, h)
    return {"shape": s, "Q": Q, "K": K, "V": V, "u": uniforms(s)}
