"""CPU fp64 oracle for routed (cross-layer) grouped-query attention over a depth-shared KV cache.

THIS IS TEST INFRASTRUCTURE, NOT A COMPUTE PATH.  Only the test-suite, the smoke check and the
benchmark's "cpu_baseline" leg may import it.  It shares no code with the HIP library: it is the
paper's definitions written out directly, two-pass softmax, float64, no tiling, no online softmax,
no splitting along the key axis.

What it follows (paper of "Stochastic KV Routing"):
  * Sec. 3.1   : a decoder of L layers; layer l has Q_l, K_l, V_l and outputs Attn(Q_l, K_l, V_l).
  * Sec. 3.1.1 : pre-fill writes K/V of T prompt tokens, sampling appends one token's K/V per
                 layer per step; footprint M = L x (T + t) x S.
  * Eq. (3.1)  : cross-layer attention Output_l = Attn(Q_l, K_l', V_l') with l' <= l.
  * Eq. (3.2)  : cache-sharing strategy S and the map mu(l) (nearest preceding cached layer).
  * Alg. 2     : Load / Update happen only for layers in S.
  * Sec. 1 footnote and Fig. 1 caption: per-token cache bytes 2 x layers x kv_heads x head_dim x 2.

Readings where the paper is silent (all listed in the design document):
  * Attn is scaled-dot-product softmax attention; `scale` is an explicit argument.
  * Causality: the query at absolute position p sees keys j <= p.  A prefill of q_b rows over a
    cache of n_b positions puts the rows at the LAST q_b positions (row i sits at n_b - q_b + i).
  * A decode step appends first and then attends over all n_b positions, the new one included,
    so a decode equals the last row of a prefill.
  * GQA: query head h reads kv head h // G with G = n_q_heads // n_kv_heads.
  * Layers are 0-based here (the paper counts from 1).
  * A route is valid iff 0 <= route[l] <= l and route[route[l]] == route[l] (the source owns a
    slot); hence route[0] == 0.  Eq. (3.2) produces monotone routes; Eq. (3.1) allows any l' <= l,
    and so does this oracle.

Every function with a numeric result is pinned by tests/test_oracle_pins.py (closed forms, the
paper's printed byte counts and worked routing example, a library softmax-attention routine in
the identity-route special case, a brute-force C twin, invariants).  No attention OUTPUT value is
printed anywhere in the paper, so output parity is pinned by definition + special cases only.
"""
from __future__ import annotations

import numpy as np


class RouteError(ValueError):
    pass


class NotOwnerError(ValueError):
    pass


# --------------------------------------------------------------------------------------------
# Routing: Eq. (3.2), 0-based.
# --------------------------------------------------------------------------------------------
def mu(strategy, n_layers):
    """Eq. (3.2): route[l] = l if l in S else max{j in S : j < l}.  `strategy` is S, 0-based."""
    S = sorted(set(int(s) for s in strategy))
    for s in S:
        if not 0 <= s < n_layers:
            raise RouteError(f"layer {s} of the strategy is outside [0, {n_layers})")
    route = []
    for l in range(n_layers):
        if l in S:
            route.append(l)
        else:
            earlier = [j for j in S if j < l]
            if not earlier:
                # max over the empty set: Eq. (3.2) is undefined; reading: the first layer
                # must belong to S.
                raise RouteError(f"layer {l} has no preceding cached layer")
            route.append(max(earlier))
    return route


def validate_route(route):
    route = [int(r) for r in route]
    if len(route) == 0:
        raise RouteError("empty route")
    for l, r in enumerate(route):
        if not 0 <= r <= l:
            raise RouteError(f"route[{l}]={r} is not in [0, {l}]")
        if route[r] != r:
            raise RouteError(f"route[{l}]={r} but layer {r} owns no slot")
    return route


def owners(route):
    """Sorted layers that own a cache slot (the strategy S)."""
    route = validate_route(route)
    return [l for l, r in enumerate(route) if r == l]


def slot_of_layer(route):
    """slot(l) = rank of route[l] among the owners."""
    own = owners(route)
    rank = {l: i for i, l in enumerate(own)}
    return [rank[r] for r in validate_route(route)]


# --------------------------------------------------------------------------------------------
# Cache sizing: Sec. 3.1.1 and the per-token formula of the Sec. 1 footnote / Fig. 1 caption.
# --------------------------------------------------------------------------------------------
def kv_bytes_per_token(n_cached_layers, n_kv_heads, head_dim, elem_bytes):
    """2 (K and V) x cached layers x kv heads x head dim x bytes per element."""
    return 2 * n_cached_layers * n_kv_heads * head_dim * elem_bytes


def cache_bytes(n_slots, batch, tokens, n_kv_heads, head_dim, elem_bytes):
    """M = L x (T + t) x S of Sec. 3.1.1 with L replaced by the number of slots |S|, times batch."""
    return batch * tokens * kv_bytes_per_token(n_slots, n_kv_heads, head_dim, elem_bytes)


# --------------------------------------------------------------------------------------------
# The cache (logical image) and the append of Alg. 2 ("Update" only for l in S).
# --------------------------------------------------------------------------------------------
class Cache:
    """Logical cache K, V[slot][b][pos][kv_head][d].

    `vals_*` hold the float64 image of the (exactly representable) input values; `bits_*` hold
    the raw storage words as handed in (uint16 for 16-bit formats, float32 otherwise) so that
    the append can be checked bit for bit.
    """

    def __init__(self, route, batch, max_ctx, n_kv_heads, head_dim, bits_dtype):
        self.route = validate_route(route)
        self.slot = slot_of_layer(self.route)
        self.n_slots = len(owners(self.route))
        shape = (self.n_slots, batch, max_ctx, n_kv_heads, head_dim)
        self.max_ctx = max_ctx
        self.vals_k = np.zeros(shape, dtype=np.float64)
        self.vals_v = np.zeros(shape, dtype=np.float64)
        self.bits_k = np.zeros(shape, dtype=bits_dtype)
        self.bits_v = np.zeros(shape, dtype=bits_dtype)

    def append(self, layer, k_vals, v_vals, k_bits, v_bits, start_pos, new_lens):
        """Write rows [0, new_lens[b]) of k/v[b] to positions start_pos[b] + i of slot(layer).

        k_*/v_*: [batch][max_new][kv_heads][d].  The layer must own its slot.
        """
        if self.route[layer] != layer:
            raise NotOwnerError(f"layer {layer} reads slot of layer {self.route[layer]}; "
                                "it has no cache of its own to update")
        s = self.slot[layer]
        for b in range(self.vals_k.shape[1]):
            n, p0 = int(new_lens[b]), int(start_pos[b])
            if n < 0 or p0 < 0 or p0 + n > self.max_ctx:
                raise ValueError("append outside the cache capacity")
            for i in range(n):
                self.vals_k[s, b, p0 + i] = k_vals[b, i]
                self.vals_v[s, b, p0 + i] = v_vals[b, i]
                self.bits_k[s, b, p0 + i] = k_bits[b, i]
                self.bits_v[s, b, p0 + i] = v_bits[b, i]


def paged_image(logical, block_table, block_size, n_blocks, kv_lens):
    """Physical image [slot][block][block_size][kvh][d] of a logical [slot][b][pos][kvh][d].

    Logical (b, pos) lives in physical block block_table[b][pos // block_size] at offset
    pos % block_size.  Cells no sequence maps to stay zero.
    """
    n_slots, batch, _, hkv, d = logical.shape
    phys = np.zeros((n_slots, n_blocks, block_size, hkv, d), dtype=logical.dtype)
    for b in range(batch):
        for pos in range(int(kv_lens[b])):
            blk = int(block_table[b][pos // block_size])
            phys[:, blk, pos % block_size] = logical[:, b, pos]
    return phys


# --------------------------------------------------------------------------------------------
# Attention: Eq. (3.1) with Attn = softmax(scale * q K^T) V.
# --------------------------------------------------------------------------------------------
def softmax_weights(q, K, scale):
    """Weights of one query vector q[d] over the key rows K[n][d] (two passes, float64)."""
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    if K.shape[0] < 1:
        raise ValueError("softmax over an empty key set is undefined")
    scores = scale * (K @ q)
    m = np.max(scores)
    w = np.exp(scores - m)
    return w / np.sum(w)


def attn_one(q, K, V, scale):
    """out[d] = sum_j softmax_j(scale * <q, K_j>) * V_j[d]."""
    w = softmax_weights(q, K, scale)
    return w @ np.asarray(V, dtype=np.float64)


def attn_position(cache, layer, b, h, n_q_heads, pos_q, q, scale):
    """Layer `layer`, sequence b, query head h at absolute position pos_q: keys 0..pos_q of the
    routed slot, kv head h // G."""
    hkv = cache.vals_k.shape[3]
    if n_q_heads % hkv:
        raise ValueError("query heads must be a multiple of kv heads")
    G = n_q_heads // hkv
    s = cache.slot[layer]
    K = cache.vals_k[s, b, : pos_q + 1, h // G, :]
    V = cache.vals_v[s, b, : pos_q + 1, h // G, :]
    return attn_one(q, K, V, scale)


def decode(cache, layer, q, kv_lens, scale):
    """One query token per sequence: q[b][h][d] sits at position kv_lens[b] - 1."""
    q = np.asarray(q, dtype=np.float64)
    B, Hq, D = q.shape
    out = np.zeros((B, Hq, D), dtype=np.float64)
    for b in range(B):
        n = int(kv_lens[b])
        if n < 1:
            raise ValueError("decode needs at least one cached position")
        for h in range(Hq):
            out[b, h] = attn_position(cache, layer, b, h, Hq, n - 1, q[b, h], scale)
    return out


def prefill(cache, layer, q, q_lens, kv_lens, scale):
    """q[b][i][h][d], i < q_lens[b], sits at absolute position kv_lens[b] - q_lens[b] + i.
    Rows i >= q_lens[b] of the output stay zero."""
    q = np.asarray(q, dtype=np.float64)
    B, S, Hq, D = q.shape
    out = np.zeros((B, S, Hq, D), dtype=np.float64)
    for b in range(B):
        nq, n = int(q_lens[b]), int(kv_lens[b])
        if nq > n or nq > S:
            raise ValueError("more query rows than cached positions")
        for i in range(nq):
            for h in range(Hq):
                out[b, i, h] = attn_position(cache, layer, b, h, Hq, n - nq + i, q[b, i, h], scale)
    return out


# --------------------------------------------------------------------------------------------
# Exact re-association used by key-axis splitting (not in the paper; stated here in float64 so
# that a test can prove the formula against the one-shot definition above).
# --------------------------------------------------------------------------------------------
def partial_state(q, K, V, scale):
    """(m, l, o) of one key range: m = max score, l = sum exp(s - m), o = sum exp(s - m) V."""
    scores = scale * (np.asarray(K, dtype=np.float64) @ np.asarray(q, dtype=np.float64))
    m = np.max(scores)
    w = np.exp(scores - m)
    return m, np.sum(w), w @ np.asarray(V, dtype=np.float64)


def merge_states(states):
    """m = max m_i; l = sum l_i e^{m_i - m}; out = sum o_i e^{m_i - m} / l."""
    m = max(s[0] for s in states)
    l = sum(s[1] * np.exp(s[0] - m) for s in states)
    o = sum(s[2] * np.exp(s[0] - m) for s in states)
    return o / l
