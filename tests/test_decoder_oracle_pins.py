"""Pins of the end-to-end decoder oracle (oracle/decoder_oracle.py): properties the paper's
inference scheme fixes, checked without any cache."""
import numpy as np

from oracle import decoder_oracle as D


def _weights(L, hidden, hq, hkv, d, mlp, vocab, route, seed=0, all_kv=False):
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
