"""CPU fp64 oracle of the synthetic decoder the end-to-end harness runs (test infrastructure only).

The paper's inference benchmark (Sec. 4.3, Tab. 4 / Tab. 5) times a Qwen3-8B-scale decoder whose
layers share K, V in groups; this is that decoder written without a cache: every layer is
evaluated over the whole token sequence with a causal mask, layer l attending (Eq. (3.1)) to the
K, V that layer route[l] computed from ITS input.  A cached implementation (Alg. 2: pre-fill, then
one token at a time, Update only for owners) must give the same logits at every position.

Layer (pre-norm, as in the Llama / Qwen families the paper uses; its own text does not spell the
block out): h = RMSNorm(x); q = rope(h Wq^T); owners: k = rope(h Wk^T), v = h Wv^T;
x += Attn(q, k_src, v_src) Wo^T; h2 = RMSNorm(x); x += (silu(h2 Wg^T) * (h2 Wu^T)) Wd^T.
Logits = RMSNorm(x) E^T with the embedding table E (tied).  Where the weights hold "{l}.q_norm" /
"{l}.k_norm" vectors (Qwen3), every head's q and k are RMS-normalised over the head dimension and
scaled by them before the rotation.
"""
from __future__ import annotations

import numpy as np

from . import project_oracle as P
from . import skv_oracle as O


def rmsnorm(x, w, eps=1e-6):
    return x / np.sqrt((x * x).mean(axis=-1, keepdims=True) + eps) * w


def rope_heads(x, positions, cos, sin):
    """x: [B][T][H][d]; rotate-half by the table row of each token's position."""
    half = x.shape[-1] // 2
    c, s = cos[positions][:, :, None, :], sin[positions][:, :, None, :]
    lo, hi = x[..., :half], x[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def logits_all_positions(w, route, tokens, n_q_heads, n_kv_heads, head_dim, cos, sin):
    """w: dict of float64 arrays (emb [V][h], final_norm [h], per layer l: norm1, wq, wk, wv, wo,
    norm2, wg, wu, wd under keys f"{l}.name"; wk, wv only for owners; optional q_norm, k_norm [d]).  tokens: int [B][T].
    Returns logits [B][T][V]."""
    B, T = tokens.shape
    G = n_q_heads // n_kv_heads
    scale = 1.0 / np.sqrt(head_dim)
    pos = np.broadcast_to(np.arange(T), (B, T))
    x = w["emb"][tokens]
    kv = {}
    for l, src in enumerate(route):
        h = rmsnorm(x, w[f"{l}.norm1"])
        q = np.einsum("bth,fh->btf", h, w[f"{l}.wq"]).reshape(B, T, n_q_heads, head_dim)
        if f"{l}.q_norm" in w:
            q = rmsnorm(q, w[f"{l}.q_norm"])
        q = rope_heads(q, pos, cos, sin)
        if src == l:
            kv[l] = P.project_kv(h, w[f"{l}.wk"], w[f"{l}.wv"], n_kv_heads, head_dim, pos, cos, sin,
                                 k_norm_weight=w.get(f"{l}.k_norm"), k_norm_eps=1e-6)
        k, v = kv[src]
        attn = np.zeros_like(q)
        for b in range(B):
            for hd in range(n_q_heads):
                for t in range(T):
                    attn[b, t, hd] = O.attn_one(q[b, t, hd], k[b, : t + 1, hd // G], v[b, : t + 1, hd // G], scale)
        x = x + np.einsum("btf,hf->bth", attn.reshape(B, T, -1), w[f"{l}.wo"])
        h2 = rmsnorm(x, w[f"{l}.norm2"])
        gate = np.einsum("bth,fh->btf", h2, w[f"{l}.wg"])
        up = np.einsum("bth,fh->btf", h2, w[f"{l}.wu"])
        x = x + np.einsum("btf,hf->bth", gate / (1.0 + np.exp(-gate)) * up, w[f"{l}.wd"])
    return np.einsum("bth,vh->btv", rmsnorm(x, w["final_norm"]), w["emb"])
