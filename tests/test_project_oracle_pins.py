"""Pins of oracle/project_oracle.py to things other than itself."""
import numpy as np

from oracle import project_oracle as P


def _tables(n_pos, d, base=10000.0):
    inv = base ** (-np.arange(d // 2) * 2.0 / d)
    ang = np.arange(n_pos)[:, None] * inv[None, :]
    return np.cos(ang), np.sin(ang)


def test_identity_weights_and_linearity():
    rng = np.random.default_rng(1)
    B, T, Hkv, D = 2, 3, 2, 8
    hidden = Hkv * D
    x = rng.standard_normal((B, T, hidden))
    eye = np.eye(hidden)
    k, v = P.project_kv(x, eye, 2 * eye, Hkv, D)
    assert np.array_equal(k.reshape(B, T, hidden), x) and np.array_equal(v.reshape(B, T, hidden), 2 * x)
    # a weight row picks out one input feature
    w = np.zeros((hidden, hidden))
    w[5, 11] = 3.0
    k, _ = P.project_kv(x, w, w, Hkv, D)
    assert np.allclose(k.reshape(B, T, hidden)[..., 5], 3.0 * x[..., 11]) and np.count_nonzero(k) == B * T
    # linear in x and in w
    wk, wv = rng.standard_normal((hidden, hidden)), rng.standard_normal((hidden, hidden))
    y = rng.standard_normal((B, T, hidden))
    k1, v1 = P.project_kv(x, wk, wv, Hkv, D)
    k2, v2 = P.project_kv(y, wk, wv, Hkv, D)
    k3, v3 = P.project_kv(2 * x - y, wk, wv, Hkv, D)
    assert np.allclose(k3, 2 * k1 - k2) and np.allclose(v3, 2 * v1 - v2)
    # one token, one feature, by hand
    assert np.isclose(k1[1, 2, 1, 3], float(np.dot(x[1, 2], wk[D + 3])))


def test_rotation_properties():
    rng = np.random.default_rng(2)
    B, T, Hkv, D = 1, 6, 1, 8
    cos, sin = _tables(64, D)
    x = rng.standard_normal((B, T, D))
    eye = np.eye(D)
    pos = np.array([[0, 1, 5, 17, 40, 63]])
    k, v = P.project_kv(x, eye, eye, Hkv, D, pos, cos, sin)
    assert np.array_equal(v[:, :, 0], x)                                    # V is never rotated
    assert np.allclose(k[0, 0, 0], x[0, 0])                                 # position 0: no rotation
    # every (i, i + d/2) pair is rotated: norms of the pairs are kept
    pair_norm = lambda a: a[..., : D // 2] ** 2 + a[..., D // 2:] ** 2
    assert np.allclose(pair_norm(k[:, :, 0]), pair_norm(x))
    # the defining property of the rotary encoding: <R_m a, R_n b> depends on m - n only
    a, b = rng.standard_normal(D), rng.standard_normal(D)
    def rot(vec, p):
        return P.project_kv(vec[None, None, :], eye, eye, 1, D, np.array([[p]]), cos, sin)[0][0, 0, 0]
    assert np.isclose(rot(a, 30) @ rot(b, 10), rot(a, 25) @ rot(b, 5))
    assert np.isclose(rot(a, 30) @ rot(b, 10), rot(a, 20) @ b)
    assert not np.isclose(rot(a, 30) @ rot(b, 10), rot(a, 31) @ rot(b, 10))
    # a quarter turn maps the pair (lo, hi) to (-hi, lo)
    c90, s90 = np.zeros((1, D // 2)), np.ones((1, D // 2))
    k90, _ = P.project_kv(a[None, None, :], eye, eye, 1, D, np.array([[0]]), c90, s90)
    assert np.allclose(k90[0, 0, 0], np.concatenate([-a[D // 2:], a[: D // 2]]))
    # heads are rotated independently, each over its own d/2 pairs
    x2 = rng.standard_normal((1, 1, 2 * D))
    k2, _ = P.project_kv(x2, np.eye(2 * D), np.eye(2 * D), 2, D, np.array([[9]]), cos, sin)
    assert np.allclose(k2[0, 0, 1], rot(x2[0, 0, D:], 9)) and np.allclose(k2[0, 0, 0], rot(x2[0, 0, :D], 9))


def test_key_normalisation():
    rng = np.random.default_rng(3)
    B, T, Hkv, D = 2, 4, 3, 8
    hidden = Hkv * D
    x = rng.standard_normal((B, T, hidden))
    wk, wv = rng.standard_normal((hidden, hidden)), rng.standard_normal((hidden, hidden))
    cos, sin = _tables(16, D)
    pos = np.array([[0, 3, 7, 15], [1, 2, 4, 8]])
    ones = np.ones(D)
    k, v = P.project_kv(x, wk, wv, Hkv, D, pos, cos, sin, k_norm_weight=ones, k_norm_eps=0.0)
    k_plain, v_plain = P.project_kv(x, wk, wv, Hkv, D, pos, cos, sin)
    assert np.allclose((k * k).mean(axis=-1), 1.0)               # every head's key has unit root-mean-square (the rotation keeps it)
    assert np.array_equal(v, v_plain)                            # V is not normalised
    # the direction is kept: normalised key = plain key / its rms, head by head
    rms = np.sqrt((k_plain * k_plain).mean(axis=-1, keepdims=True))
    assert np.allclose(k, k_plain / rms)
    # scaling the input leaves the normalised keys alone; the weight scales feature d before the rotation
    k2, _ = P.project_kv(5.0 * x, wk, wv, Hkv, D, pos, cos, sin, k_norm_weight=ones, k_norm_eps=0.0)
    assert np.allclose(k2, k)
    w = rng.uniform(0.5, 2.0, D)
    kw, _ = P.project_kv(x, wk, wv, Hkv, D, k_norm_weight=w, k_norm_eps=0.0)        # no rotation
    k1, _ = P.project_kv(x, wk, wv, Hkv, D, k_norm_weight=ones, k_norm_eps=0.0)
    assert np.allclose(kw, k1 * w)
    # eps enters under the root
    ke, _ = P.project_kv(x, wk, wv, Hkv, D, k_norm_weight=ones, k_norm_eps=0.5)
    kp, _ = P.project_kv(x, wk, wv, Hkv, D)
    assert np.allclose(ke, kp / np.sqrt((kp * kp).mean(axis=-1, keepdims=True) + 0.5))
    # the normalisation (weight included) comes BEFORE the rotation: rotating the normalised,
    # unrotated keys (identity weights, no normalisation) gives the same result
    kn, _ = P.project_kv(x, wk, wv, Hkv, D, k_norm_weight=w, k_norm_eps=1e-3)
    eye = np.eye(hidden)
    want, _ = P.project_kv(kn.reshape(B, T, hidden), eye, eye, Hkv, D, pos, cos, sin)
    got, _ = P.project_kv(x, wk, wv, Hkv, D, pos, cos, sin, k_norm_weight=w, k_norm_eps=1e-3)
    assert np.allclose(got, want) and not np.allclose(got, kn)
