"""Pins for the float64 oracle: everything here is CPU-only and independent of the HIP library.

Each test ties the oracle to something other than itself: numbers the paper prints (fixtures
under tests/golden/), closed forms, a library softmax-attention routine in the special case
where routed attention reduces to textbook causal GQA, a brute-force twin in C, and invariants.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import brute
from oracle import skv_oracle as O

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _rows(name):
    out = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                out.append(line.split())
    return out


def _sdpa_causal_gqa(q, K, V, scale):
    """Library routine: q [S][Hq][D], K/V [n][Hkv][D]; rows sit at the last S positions."""
    S, Hq, D = q.shape
    n, Hkv, _ = K.shape
    G = Hq // Hkv
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]                       # [1][Hq][S][D]
    tk = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(G, 0)[None]
    tv = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(G, 0)[None]
    mask = torch.ones(S, n, dtype=torch.bool).tril(diagonal=n - S)
    o = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask, scale=scale)
    return o[0].permute(1, 0, 2).numpy()


def _filled_cache(route, B, ctx, Hkv, D, rng):
    c = O.Cache(route, B, ctx, Hkv, D, np.float64)
    for l in O.owners(route):
        k = rng.standard_normal((B, ctx, Hkv, D))
        v = rng.standard_normal((B, ctx, Hkv, D))
        c.append(l, k, v, k, v, np.zeros(B, int), np.full(B, ctx))
    return c


# ---------------------------------------------------------------------------------------------
# Routing (Eq. 3.2) and its worked example (Fig. 4).
# ---------------------------------------------------------------------------------------------
def test_fig4_worked_example():
    kv = {r[0]: [int(x) for x in r[1:]] for r in _rows("fig4_route.txt")}
    L = kv["n_layers"][0]
    S0 = [s - 1 for s in kv["strategy_1based"]]
    route = O.mu(S0, L)
    assert [r + 1 for r in route] == kv["source_1based"]
    assert O.owners(route) == S0
    assert O.slot_of_layer(route) == [0, 0, 1, 1, 1]
    full = O.cache_bytes(L, 1, 1000, 8, 128, 2)
    shared = O.cache_bytes(len(O.owners(route)), 1, 1000, 8, 128, 2)
    assert round(100 * (1 - shared / full)) == kv["percent_saved"][0]


@pytest.mark.parametrize("L,g", [(32, 2), (32, 4), (32, 8), (36, 4), (36, 1), (7, 3)])
def test_keep_every_gth_layer(L, g):
    """'Cache only every g-th layer, the others reuse the nearest cached one' (Sec. 1) and the
    leader scheme of Sec. 4.3 both give route[l] = g * floor(l / g)."""
    route = O.mu(range(0, L, g), L)
    assert route == [g * (l // g) for l in range(L)]
    assert len(O.owners(route)) == math.ceil(L / g)
    assert O.slot_of_layer(route) == [l // g for l in range(L)]


def test_mu_is_nearest_preceding_owner_bruteforce():
    rng = np.random.default_rng(7)
    for _ in range(200):
        L = int(rng.integers(1, 12))
        S = [0] + [l for l in range(1, L) if rng.random() < 0.4]
        route = O.mu(S, L)
        for l in range(L):
            cand = [j for j in S if j <= l]
            assert route[l] == cand[-1]
        assert O.validate_route(route) == route
        # the C twin derives the same slot map
        slots, n = brute.slot_map(route)
        assert slots == O.slot_of_layer(route) and n == len(S)


def test_identity_strategy_is_self_attention_route():
    assert O.mu(range(6), 6) == list(range(6))           # l' = l: plain self-attention


@pytest.mark.parametrize("bad", [[1], [0, 2], [0, 1, 1, 2, -1], [0, 0, 1], []])
def test_invalid_routes_rejected(bad):
    # [0,0,1]: layer 2 reads layer 1, which owns no slot
    with pytest.raises(O.RouteError):
        O.validate_route(bad)
    if bad:
        with pytest.raises(ValueError):
            brute.slot_map(bad)


def test_first_layer_must_be_cached():
    with pytest.raises(O.RouteError):
        O.mu([1, 3], 5)


def test_non_monotone_route_allowed():
    # Eq. (3.1) allows any l' <= l that holds a cache
    assert O.slot_of_layer([0, 1, 0, 1, 4]) == [0, 1, 0, 1, 2]


# ---------------------------------------------------------------------------------------------
# Cache bytes: numbers the paper prints.
# ---------------------------------------------------------------------------------------------
def test_per_token_bytes_printed_in_paper():
    for model, L, hkv, d, e, kb in _rows("kv_bytes_per_token.txt"):
        assert O.kv_bytes_per_token(int(L), int(hkv), int(d), int(e)) == int(kb) * 1024, model


def test_table4_kv_cache_column():
    for T, g, mb in _rows("table4_kv_cache_mb.txt"):
        T, g, mb = int(T), int(g), int(mb)
        got = O.cache_bytes(36 // g, 1, T + 128, 8, 128, 2) / 2 ** 20
        assert abs(got - mb) <= 0.5 + 1e-9, (T, g, got, mb)


def test_table5_kv_cache_column():
    for B, g, mb in _rows("table5_kv_cache_mb.txt"):
        B, g, mb = int(B), int(g), int(mb)
        got = O.cache_bytes(36 // g, B, 8192 + 63, 8, 128, 2) / 2 ** 20
        assert abs(got - mb) <= 0.5 + 1e-9, (B, g, got, mb)


def test_cache_scales_as_one_over_g():
    """'KV cache memory scales as 1/g' (Sec. 4.3): 1170 MB -> 293 MB at 8K is the printed 4x."""
    t4 = {(int(T), int(g)): int(mb) for T, g, mb in _rows("table4_kv_cache_mb.txt")}
    for T in (2048, 8192, 16384, 32768):
        assert abs(t4[(T, 1)] / 4 - t4[(T, 4)]) <= 0.75
    for g in (1, 2, 4, 6, 9):
        assert O.cache_bytes(36 // g, 3, 100, 8, 128, 2) * g == O.cache_bytes(36, 3, 100, 8, 128, 2)


def test_cache_bytes_count_distinct_slots():
    c2 = O.Cache([0, 0, 2, 2], 2, 128, 2, 64, np.float32)
    c4 = O.Cache([0, 1, 2, 3], 2, 128, 2, 64, np.float32)
    assert c2.bits_k.nbytes + c2.bits_v.nbytes == O.cache_bytes(2, 2, 128, 2, 64, 4) == 512 * 1024
    assert c4.bits_k.nbytes + c4.bits_v.nbytes == 2 * (c2.bits_k.nbytes + c2.bits_v.nbytes)


# ---------------------------------------------------------------------------------------------
# Attention (Eq. 3.1): closed forms and special cases.
# ---------------------------------------------------------------------------------------------
def test_two_key_closed_form():
    # scores 0 and ln 3  ->  weights 1/4 and 3/4
    K = np.array([[0.0], [math.log(3.0)]])
    V = np.array([[1.0, -2.0], [5.0, 6.0]])
    out = O.attn_one(np.array([2.0]), K, V, 0.5)
    np.testing.assert_allclose(out, [0.25 * 1 + 0.75 * 5, 0.25 * -2 + 0.75 * 6], rtol=0, atol=1e-15)
    w = O.softmax_weights(np.array([2.0]), K, 0.5)
    np.testing.assert_allclose(w, [0.25, 0.75], atol=1e-15)


def test_scale_enters_the_exponent_linearly():
    # three keys on a line: weights proportional to exp(scale * q * k)
    K = np.array([[1.0], [2.0], [4.0]])
    w = O.softmax_weights(np.array([3.0]), K, 0.25)
    e = np.array([math.exp(0.75), math.exp(1.5), math.exp(3.0)])
    np.testing.assert_allclose(w, e / e.sum(), atol=1e-15)


def test_single_key_returns_its_value_exactly():
    rng = np.random.default_rng(3)
    V = rng.standard_normal((1, 16))
    out = O.attn_one(rng.standard_normal(16), rng.standard_normal((1, 16)), V, 0.3)
    assert np.array_equal(out, V[0])


def test_weights_sum_to_one_and_output_in_hull():
    rng = np.random.default_rng(4)
    K, V, q = rng.standard_normal((50, 8)), rng.standard_normal((50, 8)), rng.standard_normal(8)
    w = O.softmax_weights(q, K, 1.0)
    assert abs(w.sum() - 1) < 1e-14 and (w >= 0).all()
    out = O.attn_one(q, K, V, 1.0)
    assert (out <= V.max(0) + 1e-12).all() and (out >= V.min(0) - 1e-12).all()


def test_uniform_cases_give_mean_and_sharp_case_gives_argmax():
    rng = np.random.default_rng(5)
    K, V = rng.standard_normal((9, 4)), rng.standard_normal((9, 4))
    np.testing.assert_allclose(O.attn_one(np.zeros(4), K, V, 1.0), V.mean(0), atol=1e-14)
    same = np.tile(K[:1], (9, 1))
    np.testing.assert_allclose(O.attn_one(rng.standard_normal(4), same, V, 1.0), V.mean(0), atol=1e-14)
    K2 = np.zeros((9, 4))
    K2[6, 0] = 1000.0
    np.testing.assert_allclose(O.attn_one(np.array([1.0, 0, 0, 0]), K2, V, 1.0), V[6], atol=1e-14)


def test_identity_route_equals_library_causal_gqa():
    """l' = l reduces to standard self-attention (Sec. 3.1.2): compare with torch's SDPA."""
    rng = np.random.default_rng(11)
    B, ctx, Hq, Hkv, D, L = 2, 37, 6, 2, 8, 3
    cache = _filled_cache(list(range(L)), B, ctx, Hkv, D, rng)
    scale = 0.37
    for l in range(L):
        q = rng.standard_normal((B, ctx, Hq, D))
        got = O.prefill(cache, l, q, [ctx] * B, [ctx] * B, scale)
        for b in range(B):
            ref = _sdpa_causal_gqa(q[b], cache.vals_k[l, b], cache.vals_v[l, b], scale)
            np.testing.assert_allclose(got[b], ref, atol=1e-12)


def test_routed_layer_reads_its_source_layers_cache():
    """Layer l with route[l] = l' must equal library attention over layer l' K/V, and ragged
    bottom-right aligned chunks must see exactly keys 0..position."""
    rng = np.random.default_rng(12)
    route = [0, 0, 2, 2, 0]
    B, ctx, Hq, Hkv, D = 3, 29, 4, 2, 8
    cache = _filled_cache(route, B, ctx, Hkv, D, rng)
    kv_lens, q_lens = [29, 17, 5], [4, 17, 1]
    for l, src_slot in zip(range(5), [0, 0, 1, 1, 0]):
        q = rng.standard_normal((B, 17, Hq, D))
        got = O.prefill(cache, l, q, q_lens, kv_lens, 0.5)
        for b in range(B):
            n, nq = kv_lens[b], q_lens[b]
            ref = _sdpa_causal_gqa(q[b, :nq], cache.vals_k[src_slot, b, :n], cache.vals_v[src_slot, b, :n], 0.5)
            np.testing.assert_allclose(got[b, :nq], ref, atol=1e-12)
            assert not got[b, nq:].any()


def test_layers_sharing_a_slot_with_equal_queries_agree():
    rng = np.random.default_rng(13)
    cache = _filled_cache([0, 0, 2, 2], 2, 20, 2, 8, rng)
    q = rng.standard_normal((2, 4, 8))
    o = [O.decode(cache, l, q, [20, 11], 0.4) for l in range(4)]
    assert np.array_equal(o[0], o[1]) and np.array_equal(o[2], o[3])
    assert not np.allclose(o[0], o[2])


def test_decode_is_last_prefill_row_and_chunking_is_exact():
    rng = np.random.default_rng(14)
    cache = _filled_cache([0, 0], 2, 24, 2, 8, rng)
    q = rng.standard_normal((2, 24, 4, 8))
    full = O.prefill(cache, 1, q, [24, 24], [24, 24], 0.3)
    dec = O.decode(cache, 1, q[:, -1], [24, 24], 0.3)
    np.testing.assert_allclose(dec, full[:, -1], atol=1e-15)
    # two chunks: rows 0..9 over 10 cached positions, rows 10..23 over 24
    first = O.prefill(cache, 1, q[:, :10], [10, 10], [10, 10], 0.3)
    second = O.prefill(cache, 1, q[:, 10:], [14, 14], [24, 24], 0.3)
    np.testing.assert_allclose(np.concatenate([first, second], 1), full, atol=1e-15)


def test_key_axis_split_and_merge_is_exact():
    rng = np.random.default_rng(15)
    K, V, q = rng.standard_normal((97, 8)) * 3, rng.standard_normal((97, 8)), rng.standard_normal(8)
    whole = O.attn_one(q, K, V, 0.7)
    for cuts in ([0, 97], [0, 1, 97], [0, 32, 64, 96, 97], [0, 50, 51, 90, 97]):
        parts = [O.partial_state(q, K[a:b], V[a:b], 0.7) for a, b in zip(cuts[:-1], cuts[1:])]
        np.testing.assert_allclose(O.merge_states(parts), whole, atol=1e-13)


def test_brute_force_c_twin_agrees_on_tiny_config():
    """Config-1 shape (4 layers, route [0,0,2,2], 4/2 heads, d 64, batch 2, 128 + 1 tokens)."""
    rng = np.random.default_rng(16)
    route = [0, 0, 2, 2]
    B, ctx, Hq, Hkv, D = 2, 129, 4, 2, 64
    cache = _filled_cache(route, B, ctx, Hkv, D, rng)
    for l in range(4):
        q = rng.standard_normal((B, 128, Hq, D))
        a = O.prefill(cache, l, q, [128] * B, [128] * B, 0.125)
        c = brute.attention(cache.vals_k, cache.vals_v, cache.slot[l], q, [128] * B, [128] * B, 0.125)
        np.testing.assert_allclose(a, c, atol=1e-13)
        qd = rng.standard_normal((B, 1, Hq, D))
        a = O.decode(cache, l, qd[:, 0], [129, 77], 0.125)
        c = brute.attention(cache.vals_k, cache.vals_v, cache.slot[l], qd, [1, 1], [129, 77], 0.125)
        np.testing.assert_allclose(a, c[:, 0], atol=1e-13)


# ---------------------------------------------------------------------------------------------
# Append (Alg. 2: Update only for layers in S) and the paged image.
# ---------------------------------------------------------------------------------------------
def test_append_only_for_owner_layers_and_bit_image():
    rng = np.random.default_rng(17)
    c = O.Cache([0, 0, 2, 2], 2, 10, 2, 4, np.uint16)
    kb = rng.integers(0, 65536, (2, 3, 2, 4)).astype(np.uint16)
    vb = rng.integers(0, 65536, (2, 3, 2, 4)).astype(np.uint16)
    kf, vf = kb.astype(np.float64), vb.astype(np.float64)
    with pytest.raises(O.NotOwnerError):
        c.append(1, kf, vf, kb, vb, [0, 0], [3, 3])
    assert not c.bits_k.any() and not c.bits_v.any()
    c.append(2, kf, vf, kb, vb, [4, 7], [3, 2])
    assert np.array_equal(c.bits_k[1, 0, 4:7], kb[0]) and np.array_equal(c.bits_v[1, 1, 7:9], vb[1, :2])
    # the value image follows the same rows: K from the K rows, V from the V rows
    assert np.array_equal(c.vals_k[1, 0, 4:7], kf[0]) and np.array_equal(c.vals_v[1, 0, 4:7], vf[0])
    assert np.array_equal(c.vals_k[1, 1, 7:9], kf[1, :2]) and np.array_equal(c.vals_v[1, 1, 7:9], vf[1, :2])
    assert not c.bits_k[0].any() and not c.bits_k[1, 1, :7].any() and not c.bits_k[1, 1, 9:].any()
    assert not c.bits_k[1, 0, :4].any() and not c.bits_k[1, 0, 7:].any()
    with pytest.raises(ValueError):
        c.append(2, kf, vf, kb, vb, [8, 0], [3, 3])     # 8 + 3 > capacity 10


def test_paged_image_is_a_scatter_of_the_logical_cache():
    rng = np.random.default_rng(18)
    n_slots, B, ctx, Hkv, D, bs = 2, 3, 40, 2, 4, 16
    logical = rng.integers(1, 60000, (n_slots, B, ctx, Hkv, D)).astype(np.uint16)
    lens = [40, 17, 16]
    need = [3, 2, 1]
    perm = rng.permutation(sum(need) + 2)       # two spare physical blocks stay empty
    table = np.zeros((B, 3), dtype=np.int32)
    at = 0
    for b, n in enumerate(need):
        table[b, :n] = perm[at:at + n]
        at += n
    phys = O.paged_image(logical, table, bs, len(perm), lens)
    for b in range(B):
        for pos in range(lens[b]):
            assert np.array_equal(phys[:, table[b, pos // bs], pos % bs], logical[:, b, pos])
    used = sum(lens)
    assert np.count_nonzero(phys.reshape(n_slots, -1, Hkv * D).any(-1)) == n_slots * used
    for spare in perm[at:]:
        assert not phys[:, spare].any()


def test_attention_is_independent_of_physical_placement():
    """Paged == contiguous: gathering the physical image back through any block table gives the
    logical cache, hence the same attention result."""
    rng = np.random.default_rng(19)
    cache = _filled_cache([0, 0, 2], 2, 32, 2, 8, rng)
    lens = [32, 19]
    table = np.array([[3, 0], [1, 2]], dtype=np.int32)
    pk = O.paged_image(cache.vals_k, table, 16, 4, lens)
    pv = O.paged_image(cache.vals_v, table, 16, 4, lens)
    back = O.Cache([0, 0, 2], 2, 32, 2, 8, np.float64)
    for b in range(2):
        for pos in range(lens[b]):
            back.vals_k[:, b, pos] = pk[:, table[b, pos // 16], pos % 16]
            back.vals_v[:, b, pos] = pv[:, table[b, pos // 16], pos % 16]
    q = rng.standard_normal((2, 4, 8))
    for l in range(3):
        assert np.array_equal(O.decode(cache, l, q, lens, 0.35), O.decode(back, l, q, lens, 0.35))
