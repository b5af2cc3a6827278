"""CPU fp64 oracle for the owner-layer K/V projection that feeds the cache update.

THIS IS TEST INFRASTRUCTURE, NOT A COMPUTE PATH (tests, the smoke check and the benchmark's
cpu_baseline leg only).  It shares no code with the HIP library.

What it follows: Sec. 4.3 of the paper (the leader layer of a sharing group computes and stores
K, V; the other layers of the group skip their K/V projections, which is where the measured
throughput gain comes from) and Alg. 2 (Update only for layers in S).  The projection itself is
the decoder's usual one, K = X W_k^T, V = X W_v^T per token.

Readings where the paper is silent (listed in the design document):
  * Weights are [n_kv_heads * head_dim][hidden] (one row per output feature).
  * Position encoding: the models the paper uses (Llama, Qwen3) rotate K by position before it
    is cached.  The caller passes cos/sin tables [positions][head_dim / 2]; feature i < d/2 of a
    head pairs with feature i + d/2:  k'_i = k_i cos - k_(i+d/2) sin,  k'_(i+d/2) = k_(i+d/2) cos
    + k_i sin, with the table row of the token's absolute position.  V is never rotated.  No
    tables: no rotation.
  * Optional per-head normalisation of K before the rotation (the Qwen3 family normalises each
    head's key vector): k <- k / sqrt(mean_d(k^2) + eps) * weight[d], weight of head_dim entries
    shared by all heads.  No weight: no normalisation.
  * The result is rounded once, to the cache dtype, when it is stored.

Pinned by tests/test_project_oracle_pins.py (identity weights, linearity, the relative-position
property of the rotation, quarter turns, norm preservation, unit root-mean-square after the
normalisation).
"""
from __future__ import annotations

import numpy as np


def project_kv(x, w_k, w_v, n_kv_heads: int, head_dim: int, positions=None, rope_cos=None, rope_sin=None,
               k_norm_weight=None, k_norm_eps: float = 1e-6):
    """x: [B][T][hidden]; w_k, w_v: [n_kv_heads * head_dim][hidden]; positions: int [B][T] (absolute
    position of every token) when tables are given.  Returns K, V as [B][T][n_kv_heads][head_dim]."""
    B, T, _ = x.shape
    k = np.einsum("bth,fh->btf", x, w_k).reshape(B, T, n_kv_heads, head_dim)
    v = np.einsum("bth,fh->btf", x, w_v).reshape(B, T, n_kv_heads, head_dim)
    if k_norm_weight is not None:
        k = k / np.sqrt((k * k).mean(axis=-1, keepdims=True) + k_norm_eps) * k_norm_weight
    if rope_cos is not None:
        half = head_dim // 2
        c = rope_cos[positions][:, :, None, :]     # [B][T][1][d/2]
        s = rope_sin[positions][:, :, None, :]
        lo, hi = k[..., :half].copy(), k[..., half:].copy()
        k[..., :half] = lo * c - hi * s
        k[..., half:] = hi * c + lo * s
    return k, v
