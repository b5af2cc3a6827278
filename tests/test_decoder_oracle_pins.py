"""Pins of the end-to-end decoder oracle (oracle/decoder_oracle.py): properties the paper's
inference scheme fixes, checked without any cache."""
import numpy as np
import pytest

from oracle import decoder_oracle as D


def _weights(L, hidden, hq, hkv, d, mlp, vocab, route, seed=0, all_kv=False, qk_norm=False):
    rng = np.random.default_rng(seed)
    w = {"emb": rng.standard_normal((vocab, hidden)) * 0.3, "final_norm": np.ones(hidden)}
    for l in range(L):
        w[f"{l}.norm1"] = 1 + 0.1 * rng.standard_normal(hidden)
        w[f"{l}.norm2"] = 1 + 0.1 * rng.standard_normal(hidden)
        w[f"{l}.wq"] = rng.standard_normal((hq * d, hidden)) * 0.2
        if route[l] == l or all_kv:
            w[f"{l}.wk"] = rng.standard_normal((hkv * d, hidden)) * 0.2
            w[f"{l}.wv"] = rng.standard_normal((hkv * d, hidden)) * 0.2
        w[f"{l}.wo"] = rng.standard_normal((hidden, hq * d)) * 0.2
        w[f"{l}.wg"] = rng.standard_normal((mlp, hidden)) * 0.2
        w[f"{l}.wu"] = rng.standard_normal((mlp, hidden)) * 0.2
        w[f"{l}.wd"] = rng.standard_normal((hidden, mlp)) * 0.2
        if qk_norm:
            w[f"{l}.q_norm"] = rng.uniform(0.5, 1.5, d)
            w[f"{l}.k_norm"] = rng.uniform(0.5, 1.5, d)
    return w


def _tables(n, d):
    inv = 10000.0 ** (-np.arange(d // 2) * 2.0 / d)
    ang = np.arange(n)[:, None] * inv[None, :]
    return np.cos(ang), np.sin(ang)


def test_rmsnorm_and_causality_and_skipped_projections():
    x = np.random.default_rng(1).standard_normal((3, 5, 16))
    y = D.rmsnorm(x, np.ones(16), eps=0.0)
    assert np.allclose((y * y).mean(axis=-1), 1.0)                     # unit root-mean-square
    assert np.allclose(D.rmsnorm(7.0 * x, np.ones(16), eps=0.0), y)    # scale invariant

    L, hidden, hq, hkv, d, mlp, vocab = 4, 16, 2, 1, 8, 24, 11
    route = [0, 0, 2, 2]
    cos, sin = _tables(12, d)
    w = _weights(L, hidden, hq, hkv, d, mlp, vocab, route, all_kv=True)
    tok = np.random.default_rng(2).integers(0, vocab, (2, 9))
    base = D.logits_all_positions(w, route, tok, hq, hkv, d, cos, sin)
    # a position's logits do not depend on later tokens (causal mask, Sec. 3.1.1)
    tok2 = tok.copy()
    tok2[:, 6:] = (tok2[:, 6:] + 1) % vocab
    other = D.logits_all_positions(w, route, tok2, hq, hkv, d, cos, sin)
    assert np.array_equal(base[:, :6], other[:, :6]) and not np.allclose(base[:, 6:], other[:, 6:])
    # layers that own no cache never use a K/V projection (Sec. 4.3: they skip it)
    w2 = dict(w)
    for l in (1, 3):
        w2[f"{l}.wk"] = w[f"{l}.wk"] * 0 + 99.0
        w2[f"{l}.wv"] = w[f"{l}.wv"] * 0 - 99.0
    assert np.array_equal(D.logits_all_positions(w2, route, tok, hq, hkv, d, cos, sin), base)
    # ... and sharing changes the function: the same weights under the identity route differ
    ident = D.logits_all_positions(w, [0, 1, 2, 3], tok, hq, hkv, d, cos, sin)
    assert not np.allclose(ident, base)
    # the first position attends to itself only: its attention output is its own value row,
    # whatever the query is -- so scaling wq leaves the first position's logits unchanged
    w3 = dict(w)
    for l in range(L):
        w3[f"{l}.wq"] = 3.0 * w[f"{l}.wq"]
    scaled = D.logits_all_positions(w3, route, tok, hq, hkv, d, cos, sin)
    assert np.allclose(scaled[:, 0], base[:, 0]) and not np.allclose(scaled[:, 1:], base[:, 1:])


@pytest.mark.parametrize("qk_norm", [False, True])
def test_identity_route_is_a_standard_decoder_built_from_library_routines(qk_norm):
    """With every layer its own source (no sharing) the decoder is the standard pre-norm block of
    the Llama / Qwen families (with qk_norm: Qwen3's, whose q and k heads pass an RMS normalisation
    of their own before the rotation).  Here it is put together from torch's routines (rms_norm,
    silu, scaled_dot_product_attention with its own causal mask and its own grouping of the heads,
    linear) in float64; only the rotary rotation is written out, in the rotate-half form."""
    import torch
    import torch.nn.functional as F

    L, hidden, hq, hkv, d, mlp, vocab = 3, 16, 4, 2, 8, 24, 13
    route = list(range(L))
    B, T = 2, 7
    cos, sin = _tables(T, d)
    w = _weights(L, hidden, hq, hkv, d, mlp, vocab, route, seed=5, qk_norm=qk_norm)
    tok = np.random.default_rng(6).integers(0, vocab, (B, T))
    got = D.logits_all_positions(w, route, tok, hq, hkv, d, cos, sin)

    t = {k: torch.from_numpy(np.ascontiguousarray(v)) for k, v in w.items()}
    tc, ts = torch.from_numpy(cos), torch.from_numpy(sin)                 # [T][d/2]

    def rope(x):                                                          # x: [B][H][T][d]
        lo, hi = x[..., : d // 2], x[..., d // 2:]
        return torch.cat([lo * tc - hi * ts, hi * tc + lo * ts], dim=-1)

    x = F.embedding(torch.from_numpy(tok), t["emb"])
    for l in range(L):
        h = F.rms_norm(x, (hidden,), t[f"{l}.norm1"], eps=1e-6)
        q = F.linear(h, t[f"{l}.wq"]).view(B, T, hq, d).transpose(1, 2)
        k = F.linear(h, t[f"{l}.wk"]).view(B, T, hkv, d).transpose(1, 2)
        v = F.linear(h, t[f"{l}.wv"]).view(B, T, hkv, d).transpose(1, 2)
        if qk_norm:
            q = F.rms_norm(q, (d,), t[f"{l}.q_norm"], eps=1e-6)
            k = F.rms_norm(k, (d,), t[f"{l}.k_norm"], eps=1e-6)
        o = F.scaled_dot_product_attention(rope(q), rope(k), v, is_causal=True, enable_gqa=True)
        x = x + F.linear(o.transpose(1, 2).reshape(B, T, hq * d), t[f"{l}.wo"])
        h2 = F.rms_norm(x, (hidden,), t[f"{l}.norm2"], eps=1e-6)
        x = x + F.linear(F.silu(F.linear(h2, t[f"{l}.wg"])) * F.linear(h2, t[f"{l}.wu"]), t[f"{l}.wd"])
    want = F.linear(F.rms_norm(x, (hidden,), t["final_norm"], eps=1e-6), t["emb"]).numpy()
    assert np.abs(got - want).max() < 1e-10


def test_a_layer_reads_the_layer_its_route_names_not_the_latest_cache():
    """Eq. (3.1) allows any earlier source.  Route [0, 1, 0]: layer 2 reads layer 0's K, V although
    layer 1 has its own.  Layer 1 is made the identity on the residual stream (zero output and
    down projections), so its K/V weights can matter only to a reader of its cache."""
    L, hidden, hq, hkv, d, mlp, vocab = 3, 16, 2, 1, 8, 24, 11
    cos, sin = _tables(8, d)
    w = _weights(L, hidden, hq, hkv, d, mlp, vocab, [0, 1, 2], seed=3)
    w["1.wo"] = w["1.wo"] * 0.0
    w["1.wd"] = w["1.wd"] * 0.0
    tok = np.random.default_rng(4).integers(0, vocab, (1, 6))
    w2 = dict(w)
    w2["1.wk"], w2["1.wv"] = -2.0 * w["1.wk"], 3.0 * w["1.wv"]
    run = lambda ww, route: D.logits_all_positions(ww, route, tok, hq, hkv, d, cos, sin)
    assert np.array_equal(run(w, [0, 1, 0]), run(w2, [0, 1, 0]))        # nobody reads layer 1's cache
    assert not np.allclose(run(w, [0, 1, 1]), run(w2, [0, 1, 1]))       # layer 2 does
    assert not np.allclose(run(w, [0, 1, 0]), run(w, [0, 1, 1]))
