"""Seeded synthetic inputs shaped like the paper's Llama-2-7B decode workloads.

This module serves both the CPU oracle's tests and the GPU path's tests and
benchmark.  It holds input *recipes* only: random draws, the offline
factorisation that produces (A, B) from a random W (Sec. 2.2 display:
A = U_r sqrt(S_r), B = sqrt(S_r) V_r^T), the Hadamard fold of Sec. 3.4
(A R, R^T B), the rank draw that stands in for the Fisher rank search, and the
down-projection x . A that fills the cache.  None of the decode-time
arithmetic (RoPE, scores, softmax, value contraction, quantizer) lives here.

All randomness is numpy.random.default_rng with explicit seeds; the draw order
inside each function is fixed and documented so that results are reproducible.
"""

from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

D_HEAD = 128


@dataclass
class Layer:
    """Shape metadata of one compressed attention layer (host side)."""
    n_heads: int
    d_head: int
    group_head_off: List[int]
    k_rank_off: List[int]
    v_rank_off: List[int]
    rope_theta: float = 10000.0
    quant_block: int = 128
    q_per_kv: int = 1                  # grouped-query attention: query heads per key/value head (n_heads counts the latter)

    @property
    def n_q_heads(self) -> int:
        return self.n_heads * self.q_per_kv

    @property
    def n_groups(self) -> int:
        return len(self.group_head_off) - 1

    @property
    def R_k(self) -> int:
        return self.k_rank_off[-1]

    @property
    def R_v(self) -> int:
        return self.v_rank_off[-1]

    def group_size(self, j: int) -> int:
        return self.group_head_off[j + 1] - self.group_head_off[j]

    def b_elems(self, which: str) -> int:
        off = self.k_rank_off if which == "k" else self.v_rank_off
        return sum((off[j + 1] - off[j]) * self.group_size(j) * self.d_head for j in range(self.n_groups))


def uniform_layer(n_heads: int, group_size: int, rank_k: int, rank_v: Optional[int] = None,
                  d_head: int = D_HEAD, rope_theta: float = 10000.0, q_per_kv: int = 1) -> Layer:
    assert n_heads % group_size == 0
    ng = n_heads // group_size
    rank_v = rank_k if rank_v is None else rank_v
    return Layer(n_heads, d_head,
                 [j * group_size for j in range(ng + 1)],
                 [j * rank_k for j in range(ng + 1)],
                 [j * rank_v for j in range(ng + 1)], rope_theta, q_per_kv=q_per_kv)


def ragged_layer(n_heads: int, group_size: int, k_ranks, v_ranks, d_head: int = D_HEAD,
                 rope_theta: float = 10000.0, q_per_kv: int = 1) -> Layer:
    ng = n_heads // group_size
    assert len(k_ranks) == ng and len(v_ranks) == ng
    return Layer(n_heads, d_head,
                 [j * group_size for j in range(ng + 1)],
                 [0] + list(np.cumsum(k_ranks).astype(int)),
                 [0] + list(np.cumsum(v_ranks).astype(int)), rope_theta, q_per_kv=q_per_kv)


# ------------------------------------------------------------------ ranks

def draw_ranks(seed: int, stream: int, n_groups: int, total: int = 2048,
               lo: int = 96, hi: int = 416, step: int = 32) -> List[int]:
    """Non-uniform per-group ranks standing in for the Fisher rank search
    (Sec. 3.3): multiples of `step` in [lo, hi] that sum to `total`.

    Draw r_j uniformly from {lo, lo+step, .., hi} with default_rng([seed,
    stream]); rescale by total/sum; round to the nearest multiple of `step`;
    clip to [lo, hi]; then move single `step`s onto/off the groups with the
    largest rounding residual (ties: lowest index) until the sum is `total`.
    """
    assert total % step == 0 and n_groups * lo <= total <= n_groups * hi
    rng = np.random.default_rng([seed, stream])
    choices = np.arange(lo, hi + 1, step)
    raw = rng.choice(choices, size=n_groups).astype(np.float64)
    scaled = raw * (total / raw.sum())
    r = np.clip(np.rint(scaled / step) * step, lo, hi).astype(np.int64)
    resid = scaled - r
    while r.sum() != total:
        if r.sum() < total:
            cand = [j for j in range(n_groups) if r[j] + step <= hi]
            j = max(cand, key=lambda i: (resid[i], -i))
            r[j] += step
            resid[j] -= step
        else:
            cand = [j for j in range(n_groups) if r[j] - step >= lo]
            j = min(cand, key=lambda i: (resid[i], i))
            r[j] -= step
            resid[j] += step
    return [int(v) for v in r]


# ------------------------------------------------------- offline factors

def orthonormal_rows(rng: np.random.Generator, r: int, width: int) -> np.ndarray:
    """[r, width] matrix with orthonormal rows: Q^T from the QR of N(0,1)
    [width, r]."""
    G = rng.standard_normal((width, r))
    Q, _ = np.linalg.qr(G)
    return np.ascontiguousarray(Q.T)


def svd_factor(W: np.ndarray, r: int):
    """W [m, n] -> A = U_r sqrt(S_r) [m, r], B = sqrt(S_r) V_r^T [r, n]
    (Sec. 2.2).  float64."""
    U, S, Vt = np.linalg.svd(np.asarray(W, dtype=np.float64), full_matrices=False)
    rs = np.sqrt(S[:r])
    return U[:, :r] * rs[None, :], rs[:, None] * Vt[:r, :]


def hadamard(n: int) -> np.ndarray:
    """Orthonormal Sylvester-Walsh-Hadamard matrix H_n / sqrt(n), n a power of 2."""
    assert n > 0 and (n & (n - 1)) == 0
    H = np.ones((1, 1), dtype=np.float64)
    while H.shape[0] < n:
        H = np.block([[H, H], [H, -H]])
    return H / np.sqrt(float(n))


def fold_hadamard(A: np.ndarray, B: np.ndarray):
    """(A R, R^T B) with R the orthonormal Hadamard matrix of size rank
    (Sec. 3.4 display).  The product A.B is unchanged."""
    R = hadamard(A.shape[1])
    return A @ R, R.T @ B


def make_factors(layer: Layer, seed: int, which: str, d_model: Optional[int] = None,
                 rotate: bool = False):
    """Per-group (A, B) from a truncated SVD of W ~ N(0, var 1/d_model)
    [d_model, s*d_head]; rng = default_rng([seed, 10 + (which=='v'), j]) per
    group j, one standard_normal draw of W.  Returns A [d_model, R] float64 and
    the concatenated B buffer (flat float64, group j row-major [r_j, s_j*d_h])."""
    d_model = layer.n_q_heads * layer.d_head if d_model is None else d_model
    off = layer.k_rank_off if which == "k" else layer.v_rank_off
    A = np.empty((d_model, off[-1]), dtype=np.float64)
    Bs = []
    for j in range(layer.n_groups):
        rng = np.random.default_rng([seed, 10 + (which == "v"), j])
        width = layer.group_size(j) * layer.d_head
        W = rng.standard_normal((d_model, width)) / np.sqrt(float(d_model))
        r = off[j + 1] - off[j]
        Aj, Bj = svd_factor(W, r)
        if rotate:
            Aj, Bj = fold_hadamard(Aj, Bj)
        A[:, off[j]:off[j + 1]] = Aj
        Bs.append(Bj.reshape(-1))
    return A, np.concatenate(Bs)


def make_orthonormal_B(layer: Layer, seed: int, which: str) -> np.ndarray:
    """Concatenated B with orthonormal rows scaled by sqrt(width / r) per group
    (configuration 1); rng = default_rng([seed, 20 + (which=='v'), j])."""
    off = layer.k_rank_off if which == "k" else layer.v_rank_off
    Bs = []
    for j in range(layer.n_groups):
        rng = np.random.default_rng([seed, 20 + (which == "v"), j])
        r = off[j + 1] - off[j]
        width = layer.group_size(j) * layer.d_head
        Bs.append((orthonormal_rows(rng, r, width) * np.sqrt(width / r)).reshape(-1))
    return np.concatenate(Bs)


# --------------------------------------------------------------- tensors

def round_to(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round float values to the storage dtype and return them as float32
    holding exactly representable values ('f16' or 'bf16')."""
    x = np.asarray(x, dtype=np.float32)
    if dtype == "f16":
        return x.astype(np.float16).astype(np.float32)
    if dtype == "bf16":
        u = x.view(np.uint32).astype(np.uint64)
        u = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16          # round-half-even on bit 16
        return u.astype(np.uint32).view(np.float32).reshape(x.shape)
    raise ValueError(dtype)


def make_latents_cpu(x: np.ndarray, A: np.ndarray, dtype: str = "f16") -> np.ndarray:
    """Cache fill h = x . A as a float32 library GEMM, rounded to the cache
    dtype (input preparation, small shapes).  x [.., d], A [d, R]."""
    return round_to(np.asarray(x, np.float32) @ np.asarray(A, np.float32), dtype)


@dataclass
class Case:
    """One decode-step problem instance; float arrays hold values that are
    exactly representable in `dtype`."""
    name: str
    layer: Layer
    dtype: str
    batch: int
    seq: int
    q: np.ndarray                      # [B, n, d_h]
    q_pos: np.ndarray                  # [B] int32
    Hk: np.ndarray                     # [B, L, R_k]
    Hv: np.ndarray                     # [B, L, R_v]
    Bk: np.ndarray                     # flat
    Bv: np.ndarray                     # flat
    Ak: Optional[np.ndarray] = None    # [d, R_k]
    Av: Optional[np.ndarray] = None
    k_pos: Optional[np.ndarray] = None
    seq_lens: Optional[np.ndarray] = None
    extra: dict = field(default_factory=dict)


def make_case_orthonormal(layer: Layer, batch: int, seq: int, seed: int = 0, dtype: str = "f16") -> Case:
    """Configuration-1 recipe: B with orthonormal rows x sqrt(width/r), latents
    and q ~ N(0,1).  Draw order with default_rng([seed, 1]): Hk, Hv, q."""
    rng = np.random.default_rng([seed, 1])
    Hk = round_to(rng.standard_normal((batch, seq, layer.R_k)), dtype)
    Hv = round_to(rng.standard_normal((batch, seq, layer.R_v)), dtype)
    q = round_to(rng.standard_normal((batch, layer.n_q_heads, layer.d_head)), dtype)
    Bk = round_to(make_orthonormal_B(layer, seed, "k"), dtype)
    Bv = round_to(make_orthonormal_B(layer, seed, "v"), dtype)
    q_pos = np.full((batch,), seq - 1, dtype=np.int32)
    return Case("orthonormal", layer, dtype, batch, seq, q, q_pos, Hk, Hv, Bk, Bv)


def make_case_svd(layer: Layer, batch: int, seq: int, seed: int = 0, dtype: str = "f16",
                  rotate: bool = False, d_model: Optional[int] = None) -> Case:
    """Configuration-2..5 recipe: (A, B) from truncated SVDs of random W,
    latents = x . A with x ~ N(0,1) [B, L, d_model] (default_rng([seed, 2, b])
    per batch element), q ~ N(0,1) from default_rng([seed, 3])."""
    d_model = layer.n_q_heads * layer.d_head if d_model is None else d_model
    Ak, Bk = make_factors(layer, seed, "k", d_model, rotate)
    Av, Bv = make_factors(layer, seed, "v", d_model, rotate)
    Ak16, Av16 = round_to(Ak, dtype), round_to(Av, dtype)
    Hk = np.empty((batch, seq, layer.R_k), np.float32)
    Hv = np.empty((batch, seq, layer.R_v), np.float32)
    for b in range(batch):
        x = round_to(np.random.default_rng([seed, 2, b]).standard_normal((seq, d_model)), dtype)
        Hk[b] = make_latents_cpu(x, Ak16, dtype)
        Hv[b] = make_latents_cpu(x, Av16, dtype)
    q = round_to(np.random.default_rng([seed, 3]).standard_normal((batch, layer.n_q_heads, layer.d_head)), dtype)
    q_pos = np.full((batch,), seq - 1, dtype=np.int32)
    return Case("svd", layer, dtype, batch, seq, q, q_pos, Hk, Hv,
                round_to(Bk, dtype), round_to(Bv, dtype), Ak16, Av16)


# ------------------------------------------------- the five configurations

def config_layer(cfg: str, seed: int = 0) -> Layer:
    """Layer metadata of the named benchmark configuration at full size."""
    if cfg == "1":
        return uniform_layer(8, 4, 128)
    if cfg in ("2", "4"):
        return uniform_layer(32, 4, 256)
    if cfg == "3":
        return ragged_layer(32, 4, draw_ranks(seed, 0, 8), draw_ranks(seed, 1, 8))
    if cfg == "5a":
        return uniform_layer(32, 1, 64)
    if cfg == "5b":
        return uniform_layer(32, 32, 2048)
    if cfg == "2p":
        # the allocation of the paper's latency experiments (Sec. 4.5): keys compressed by 75 %,
        # values by 25 %, i.e. ranks 128 / 384 per group of 4 heads (50 % overall)
        return ragged_layer(32, 4, [128] * 8, [384] * 8)
    if cfg == "gqa":
        # the grouped-query models of Sec. 4.1 (Llama-3-8B, Mistral-7B): 32 query heads on 8 key/value
        # heads, groups of 4 key/value heads at 50 % (rank 256 per side), Llama-3's RoPE base
        return uniform_layer(8, 4, 256, rope_theta=500000.0, q_per_kv=4)
    raise ValueError(cfg)


FULL_SIZES = {            # (batch, seq) at full size
    "1": (1, 1024), "2": (1, 16384), "2-4k": (1, 4096), "2-64k": (1, 65536),
    "3": (4, 16384), "4": (16, 8192), "5a": (8, 16384), "5b": (8, 16384),
    "2p": (1, 16384), "2p-64k": (1, 65536), "gqa": (4, 16384), "gqa-64k": (1, 65536),
}
