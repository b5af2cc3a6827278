"""CPU fp64 oracle for the TRAINING-time side of the paper: Random Cross-Layer Attention.

THIS IS TEST INFRASTRUCTURE, NOT A COMPUTE PATH.  Only the test-suite, the smoke check and the
benchmark's "cpu_baseline" leg may import it.  It shares no code with the HIP library.

What it follows:
  * Sec. 3.2 (R-CLA): for every layer l and every forward pass a decision d ~ Bernoulli(p);
    d = 1: self-attention with (K_l, V_l); d = 0: cross-layer attention with (K_l', V_l'),
    l' uniform over the layers before l.  Every layer still computes its own K, V.
  * Sec. 4.2.3 (ablation): CLA@k, groups of k consecutive layers attend to one layer's K, V
    (layers 0..k-1 share one, and so on); RD-CLA@k, the same fixed source but used only when a
    per-layer, per-step coin says so, else the layer's local K, V.
  * Eq. (3.1): the attention itself, here over a whole sequence with a causal mask, and its
    gradient (the chain rule through softmax written out; no tiling, no recomputation tricks).

Readings where the paper is silent (all listed in the design document):
  * Layers are 0-based here; the first layer has no earlier layer and always self-attends.
  * The coin of RD-CLA@k is Bernoulli(p) with the same meaning of d as in R-CLA (d = 1: local).
  * The shared layer of a CLA@k group is its first layer (as at inference, Sec. 4.3).
  * The random numbers: a counter-based generator, so that the library and this file can draw
    the same decisions independently.  r(seed, step, layer, which) =
    mix(mix(mix(seed) ^ step) ^ (256 layer + which)), mix = the SplitMix64 output function
    (Steele, Lea, Flood 2014).  which = 0: the decision, d = 1 iff (r >> 11) 2^-53 < p;
    which = 1: the source, l' = ((r >> 32) l) >> 32 (0-based, l layers to choose from).
  * Several layers may read one layer's K, V in a pass; its gradient is the sum of theirs.

Pinned by tests/test_rcla_train_oracle_pins.py: the published SplitMix64 outputs, sampling
frequencies, closed forms of the attention (one key, equal keys), finite differences of the
forward (which the backward formulas share nothing with) and the invariants of softmax gradients.
"""
from __future__ import annotations

import numpy as np

_M64 = (1 << 64) - 1

RCLA, CLA_K, RDCLA_K = 0, 1, 2


def mix(x: int) -> int:
    """Output of one SplitMix64 step whose state before the step is x."""
    x = (x + 0x9E3779B97F4A7C15) & _M64
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & _M64
    return x ^ (x >> 31)


def draw(seed: int, step: int, layer: int, which: int) -> int:
    return mix(mix(mix(seed & _M64) ^ (step & _M64)) ^ (256 * layer + which))


def bernoulli(seed: int, step: int, layer: int, p: float) -> int:
    return 1 if (draw(seed, step, layer, 0) >> 11) * 2.0 ** -53 < p else 0


def sample_route(scheme: int, n_layers: int, k: int, p: float, seed: int, step: int) -> list:
    """route[l] = the layer whose K, V layer l attends to in this forward pass (0-based)."""
    route = []
    for l in range(n_layers):
        if scheme == CLA_K:
            route.append(k * (l // k))
        elif scheme == RDCLA_K:
            route.append(l if bernoulli(seed, step, l, p) else k * (l // k))
        elif scheme == RCLA:
            if l == 0 or bernoulli(seed, step, l, p):
                route.append(l)
            else:
                route.append(((draw(seed, step, l, 1) >> 32) * l) >> 32)
        else:
            raise ValueError("unknown scheme")
    return route


def _lens(seq_lens, batch, seq):
    return [seq] * batch if seq_lens is None else [int(n) for n in seq_lens]


def attn_fwd(q, k, v, scale: float, seq_lens=None):
    """q: [B][S][Hq][D], k, v: [B][S][Hkv][D] (float64).  Row i of sequence b attends to keys
    0..i of the same sequence (i < seq_lens[b]).  Returns out [B][S][Hq][D] and
    lse [B][Hq][S] = log sum_j exp(scale <q_i, k_j>); rows at or beyond the length are zero."""
    B, S, Hq, D = q.shape
    G = Hq // k.shape[2]
    out = np.zeros_like(q)
    lse = np.zeros((B, Hq, S))
    for b, n in enumerate(_lens(seq_lens, B, S)):
        for h in range(Hq):
            s = scale * (q[b, :n, h] @ k[b, :n, h // G].T)
            s = np.where(np.tril(np.ones((n, n), dtype=bool)), s, -np.inf)
            m = s.max(axis=1, keepdims=True)
            e = np.exp(s - m)
            z = e.sum(axis=1, keepdims=True)
            out[b, :n, h] = (e / z) @ v[b, :n, h // G]
            lse[b, h, :n] = (m + np.log(z))[:, 0]
    return out, lse


def attn_bwd(q, k, v, d_out, scale: float, seq_lens=None):
    """Gradients of sum(out * d_out) with respect to q, k, v (shapes of q, k, v).  With
    P = softmax(S), S = scale Q K^T (causal):  dV = P^T dO;  dP = dO V^T;
    dS = P o (dP - rowsum(P o dP));  dQ = scale dS K;  dK = scale dS^T Q.
    The heads of a group add their dK, dV into the one kv head they share."""
    B, S, Hq, D = q.shape
    G = Hq // k.shape[2]
    dq, dk, dv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    for b, n in enumerate(_lens(seq_lens, B, S)):
        for h in range(Hq):
            g = h // G
            s = scale * (q[b, :n, h] @ k[b, :n, g].T)
            s = np.where(np.tril(np.ones((n, n), dtype=bool)), s, -np.inf)
            e = np.exp(s - s.max(axis=1, keepdims=True))
            p = e / e.sum(axis=1, keepdims=True)
            do = d_out[b, :n, h]
            dv[b, :n, g] += p.T @ do
            dp = do @ v[b, :n, g].T
            ds = p * (dp - (p * dp).sum(axis=1, keepdims=True))
            dq[b, :n, h] = scale * (ds @ k[b, :n, g])
            dk[b, :n, g] += scale * (ds.T @ q[b, :n, h])
    return dq, dk, dv


def layer_stack_fwd_bwd(qs, ks, vs, d_outs, route, scale: float):
    """One pass over a stack of layers: layer l attends with its own queries qs[l] to
    (ks[route[l]], vs[route[l]]).  Returns the outputs, the per-layer dQ and the per-layer dK, dV
    in which every source layer has collected the gradients of all the layers that read it."""
    L = len(qs)
    outs, dqs = [], []
    dks = [np.zeros_like(ks[0]) for _ in range(L)]
    dvs = [np.zeros_like(vs[0]) for _ in range(L)]
    for l in range(L):
        src = route[l]
        out, _ = attn_fwd(qs[l], ks[src], vs[src], scale)
        dq, dk, dv = attn_bwd(qs[l], ks[src], vs[src], d_outs[l], scale)
        outs.append(out)
        dqs.append(dq)
        dks[src] += dk
        dvs[src] += dv
    return outs, dqs, dks, dvs
