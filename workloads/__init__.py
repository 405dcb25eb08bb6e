"""Seeded synthetic inputs for the PiKV decode path.

This module draws random numbers and lays them out; it holds none of the method's
arithmetic (no logits, softmax, attention, utilities or selection).  Both the CPU
oracle's tests and the HIP path's tests/benchmark take their inputs from here, so the
two sides see identical bits.

Host-side cases are numpy (bfloat16 carried as ``uint16`` bit patterns); the large
benchmark-sized caches are drawn directly in device memory with a seeded torch
generator and can be copied back shard by shard for the oracle.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np


# ----------------------------------------------------------------- bf16 <-> f32 bits
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bfloat16 bit pattern (uint16).  Finite inputs."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(a: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(a, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def encode(a: np.ndarray, dtype: str) -> np.ndarray:
    """float array -> storage array of the case's dtype ('f32' or 'bf16')."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a if dtype == "f32" else f32_to_bf16_bits(a)


def decode(a: np.ndarray, dtype: str) -> np.ndarray:
    """storage array -> float32 values."""
    return a if dtype == "f32" else bf16_bits_to_f32(a)


# ------------------------------------------------------------------------ geometry
@dataclass
class Geometry:
    """Shape of one layer's expert-sharded cache and of one decode step over it."""
    B: int
    Hq: int
    Hkv: int
    D: int
    E: int
    S: int
    k: int
    rank: int = 0                 # 0: dense rows [., D]; r > 0: rank-r codes [., r]
    dtype: str = "bf16"           # 'f32' | 'bf16'
    per_head_routing: bool = False  # True: one routing decision per (sequence, head)
    name: str = ""
    tq: int = 1                   # draft queries per sequence folded into Hq (multi-query tile)
    token_major: bool = False     # q / y rows in the caller's [tq, heads] order (else kv head first)

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def width(self) -> int:
        return self.rank if self.rank else self.D

    @property
    def d_r(self) -> int:
        """Length of the vector the router sees: one head (per-head routing), all heads of the
        token, or - token-major multi-query step - all heads of the tile's first query."""
        if self.per_head_routing:
            return self.D
        return (self.Hq // self.tq if self.token_major else self.Hq) * self.D

    @property
    def route_rows(self) -> int:
        return self.B * (self.Hq if self.per_head_routing else 1)

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def kv_bytes_per_step(self, n_mean: Optional[float] = None) -> int:
        """K and V (or code) bytes of the selected shards: what one step must read."""
        n = self.S if n_mean is None else n_mean
        return int(self.B * self.Hkv * self.k * n * 2 * self.width * self.elem_bytes)


# The five workload shapes the build is specified on (full sizes).
CONFIGS = {
    "c1_tiny_f32": Geometry(B=1, Hq=4, Hkv=4, D=64, E=4, S=256, k=2, dtype="f32",
                            per_head_routing=True, name="c1_tiny_f32"),
    "c2_bf16_decode": Geometry(B=8, Hq=32, Hkv=32, D=128, E=16, S=4096, k=2,
                               name="c2_bf16_decode"),
    "c3_long_context": Geometry(B=1, Hq=32, Hkv=8, D=128, E=16, S=8192, k=4,
                                name="c3_long_context"),
    "c4_streaming": Geometry(B=32, Hq=32, Hkv=32, D=128, E=8, S=2048, k=2,
                             name="c4_streaming"),
    "c5_compressed": Geometry(B=16, Hq=32, Hkv=32, D=128, E=16, S=2048, k=2, rank=32,
                              name="c5_compressed"),
}

# Widening beyond the five specified workloads ("next" rows of the scope table).
# Multi-query tile: Tq draft tokens of a sequence attend to the same selected shards in one pass
# (speculative decoding).  Laid out as [B, Hkv, Tq*G, D] the Tq*G query rows of a kv head are
# simply a larger grouped-query group, so the long-context workload with Tq = 4 is a geometry
# with Hq = 4*32 query rows over the same 8 kv heads (group 16 = a full MFMA tile).
# Wider tiles keep the tokens' natural layout, q [B, Tq, heads, D] (token_major): Tq = 8 on the
# long-context shape (32 rows per kv head, two 16-row tiles) and Tq = 16 on the same shards with
# 16 query heads over 4 kv heads (64 rows per kv head, four tiles; Hq stays within 256 rows).
EXTRA_CONFIGS = {
    "c3_long_context_tq4": Geometry(B=1, Hq=128, Hkv=8, D=128, E=16, S=8192, k=4,
                                    name="c3_long_context_tq4", tq=4),
    "c3_long_context_tq8": Geometry(B=1, Hq=256, Hkv=8, D=128, E=16, S=8192, k=4,
                                    name="c3_long_context_tq8", tq=8, token_major=True),
    "c3_kv4_tq16": Geometry(B=1, Hq=256, Hkv=4, D=128, E=16, S=8192, k=4,
                            name="c3_kv4_tq16", tq=16, token_major=True),
}
CONFIGS.update(EXTRA_CONFIGS)


def routing_rows(g: "Geometry", q):
    """The rows the router sees, [route_rows, d_r], of queries q [B, Hq, D] held in the caller's
    layout (numpy array or torch tensor).  Token-major multi-query step: the heads of the first
    query of every sequence.  Layout only."""
    if g.token_major and g.tq > 1 and not g.per_head_routing:
        x = q.reshape(g.B, g.Hq, g.D)[:, :g.Hq // g.tq].reshape(g.B, g.d_r)
        return x.contiguous() if hasattr(x, "contiguous") else np.ascontiguousarray(x)
    return q.reshape(g.route_rows, g.d_r)


def token_major_rows(Hq: int, Hkv: int, tq: int) -> np.ndarray:
    """perm[h] = row, in the caller's [tq, heads] order, of internal query row h (internal order:
    kv head, draft query, head of the group).  Layout only."""
    heads, group = Hq // tq, Hq // Hkv
    g = heads // Hkv
    perm = np.empty(Hq, np.int64)
    for hk in range(Hkv):
        for t in range(tq):
            for gg in range(g):
                perm[hk * group + t * g + gg] = t * heads + hk * g + gg
    return perm


def zipf_bias(E: int, s: float, rng: np.random.Generator) -> np.ndarray:
    """log of a Zipf(s) popularity law over a seeded permutation of the experts."""
    ranks = rng.permutation(E) + 1
    p = ranks.astype(np.float64) ** (-s)
    p /= p.sum()
    return np.log(p).astype(np.float32)


# --------------------------------------------------------------------- host cases
@dataclass
class HostCase:
    geo: Geometry
    q: np.ndarray                       # [B,Hq,D] storage dtype
    W_r: np.ndarray                     # [d_r,E]  storage dtype
    bias: Optional[np.ndarray]          # [E] f32 or None
    K_shards: List[np.ndarray]          # B*E arrays [Hkv,S,width]
    V_shards: List[np.ndarray]
    U_K: Optional[np.ndarray]           # [Hkv,rank,D] storage dtype
    U_V: Optional[np.ndarray]
    n_valid: np.ndarray                 # [B,E] int32
    utility: np.ndarray                 # [B,E,S] f32
    extra: dict = field(default_factory=dict)

    def clone(self) -> "HostCase":
        return HostCase(self.geo, self.q.copy(), self.W_r.copy(),
                        None if self.bias is None else self.bias.copy(),
                        [s.copy() for s in self.K_shards], [s.copy() for s in self.V_shards],
                        None if self.U_K is None else self.U_K.copy(),
                        None if self.U_V is None else self.U_V.copy(),
                        self.n_valid.copy(), self.utility.copy(), dict(self.extra))


def make_host_case(geo: Geometry, seed: int = 0, *, kv: str = "normal", w_sigma: float = 0.02,
                   zipf_s: float = 0.0, n_valid="full", utility0: str = "zero") -> HostCase:
    """Draw one layer's cache and one step's query on the host.

    kv: 'normal' (N(0,1)) or 'lognormal_token' (N(0,1) times one LogNormal(0,0.5) factor
        per (sequence, shard, slot), shared by heads and by K and V).
    n_valid: 'full', 'ragged' (seeded lengths in [0,S], including an empty and a full
        shard when there is room) or an int array [B,E].
    utility0: 'zero' or 'exp' (Exp(1)/S, distinct positive values).
    Draw order is fixed: W_r, q, K (shard by shard), V, U_K, U_V, bias, n_valid, utility.
    """
    rng = np.random.default_rng(seed)
    g = geo
    w = g.width
    W_r = rng.standard_normal((g.d_r, g.E)) * w_sigma
    q = rng.standard_normal((g.B, g.Hq, g.D))
    nsh = g.B * g.E
    Kf = [rng.standard_normal((g.Hkv, g.S, w)) for _ in range(nsh)]
    Vf = [rng.standard_normal((g.Hkv, g.S, w)) for _ in range(nsh)]
    if kv == "lognormal_token":
        for i in range(nsh):
            f = rng.lognormal(0.0, 0.5, size=(1, g.S, 1))
            Kf[i] = Kf[i] * f
            Vf[i] = Vf[i] * f
    U_K = U_V = None
    if g.rank:
        U_K = encode(rng.standard_normal((g.Hkv, g.rank, g.D)) / np.sqrt(g.rank), g.dtype)
        U_V = encode(rng.standard_normal((g.Hkv, g.rank, g.D)) / np.sqrt(g.rank), g.dtype)
    bias = zipf_bias(g.E, zipf_s, rng) if zipf_s > 0 else None
    if isinstance(n_valid, str):
        if n_valid == "full":
            nv = np.full((g.B, g.E), g.S, np.int32)
        elif n_valid == "ragged":
            nv = rng.integers(1, g.S + 1, size=(g.B, g.E)).astype(np.int32)
            flat = nv.reshape(-1)
            if flat.size >= 3:
                flat[rng.integers(0, flat.size)] = 0
                flat[(rng.integers(0, flat.size) + 1) % flat.size] = g.S
        else:
            raise ValueError(n_valid)
    else:
        nv = np.ascontiguousarray(n_valid, dtype=np.int32).reshape(g.B, g.E)
    if utility0 == "zero":
        u = np.zeros((g.B, g.E, g.S), np.float32)
    elif utility0 == "exp":
        u = (rng.exponential(1.0, size=(g.B, g.E, g.S)) / g.S).astype(np.float32)
    else:
        raise ValueError(utility0)
    return HostCase(g, encode(q, g.dtype), encode(W_r, g.dtype), bias,
                    [encode(x, g.dtype) for x in Kf], [encode(x, g.dtype) for x in Vf],
                    U_K, U_V, nv, u)


def make_c1(seed: int = 0) -> HostCase:
    """Config 1: tiny fp32 case; default_rng(seed), draw order W_r, q, K, V; W_r ~ N(0,1)."""
    return make_host_case(CONFIGS["c1_tiny_f32"], seed, w_sigma=1.0)


def draw_new_kv(geo: Geometry, seed: int):
    """One new token's K and V rows [B,Hkv,width] (storage dtype) for an append."""
    rng = np.random.default_rng(seed)
    kn = rng.standard_normal((geo.B, geo.Hkv, geo.width))
    vn = rng.standard_normal((geo.B, geo.Hkv, geo.width))
    return encode(kn, geo.dtype), encode(vn, geo.dtype)


def draw_queries(geo: Geometry, seed: int) -> np.ndarray:
    """A fresh query batch [B,Hq,D] (storage dtype)."""
    rng = np.random.default_rng(seed)
    return encode(rng.standard_normal((geo.B, geo.Hq, geo.D)), geo.dtype)


# ------------------------------------------------------------------- device cases
def make_device_layers(geo: Geometry, n_layers: int, seed: int, device, *, kv: str = "normal",
                       w_sigma: float = 0.02, zipf_s: float = 0.0, utility0: str = "zero"):
    """Draw ``n_layers`` independent cache instances of ``geo`` directly in device memory.

    Returns a list of dicts of torch tensors: q [B,Hq,D], W_r [d_r,E], bias [E] or None,
    K, V [B,E,Hkv,S,width] (one allocation per layer; shard (b,e) is K[b,e]),
    U_K, U_V, n_valid [B,E] int32 (full), utility [B,E,S] f32.  bf16 values are rounded
    to nearest even by torch's conversion.
    """
    import torch

    tdt = torch.float32 if geo.dtype == "f32" else torch.bfloat16
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    nprng = np.random.default_rng(seed)
    g = geo
    layers = []
    for _ in range(n_layers):
        def randn(*shape):
            return torch.randn(*shape, generator=gen, device=device, dtype=torch.float32)

        W_r = (randn(g.d_r, g.E) * w_sigma).to(tdt)
        q = randn(g.B, g.Hq, g.D).to(tdt)
        K = torch.empty((g.B, g.E, g.Hkv, g.S, g.width), device=device, dtype=tdt)
        V = torch.empty_like(K)
        for b in range(g.B):           # shard-row at a time keeps the fp32 temporaries small
            for dst in (K, V):
                t = randn(g.E, g.Hkv, g.S, g.width)
                dst[b].copy_(t)
                del t
        if kv == "lognormal_token":
            for b in range(g.B):
                f = torch.exp(0.5 * randn(g.E, 1, g.S, 1))
                K[b] = (K[b].float() * f).to(tdt)
                V[b] = (V[b].float() * f).to(tdt)
        U_K = U_V = None
        if g.rank:
            U_K = (randn(g.Hkv, g.rank, g.D) / float(np.sqrt(g.rank))).to(tdt)
            U_V = (randn(g.Hkv, g.rank, g.D) / float(np.sqrt(g.rank))).to(tdt)
        bias = None
        if zipf_s > 0:
            bias = torch.from_numpy(zipf_bias(g.E, zipf_s, nprng)).to(device)
        n_valid = torch.full((g.B, g.E), g.S, device=device, dtype=torch.int32)
        if utility0 == "exp":
            u = torch.empty((g.B, g.E, g.S), device=device, dtype=torch.float32)
            u.exponential_(1.0, generator=gen)
            u /= g.S
        else:
            u = torch.zeros((g.B, g.E, g.S), device=device, dtype=torch.float32)
        layers.append(dict(q=q, W_r=W_r, bias=bias, K=K, V=V, U_K=U_K, U_V=U_V,
                           n_valid=n_valid, utility=u))
    return layers


def to_host(t, dtype: str) -> np.ndarray:
    """torch tensor (f32/bf16/int32) -> numpy storage array as the oracle wants it."""
    import torch

    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16).copy()
    return t.numpy().copy()
