"""Pins of the training-time oracle (oracle/rcla_train_oracle.py) to things other than itself:
published SplitMix64 outputs, the sampling rule of Sec. 3.2 as frequencies, closed forms of the
attention, finite differences of the forward for the backward, invariants of softmax gradients."""
import math

import numpy as np
import pytest

from oracle import rcla_train_oracle as T


def test_mix_reproduces_the_published_splitmix64_sequence():
    # first three outputs of SplitMix64 seeded with 0 (the reference implementation's test vector):
    # the state advances by the golden-ratio increment, mix(state before the step) is the output
    inc = 0x9E3779B97F4A7C15
    want = [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    assert [T.mix((i * inc) & (2 ** 64 - 1)) for i in range(3)] == want


def test_rcla_sampling_rule_of_sec_3_2():
    L, p, steps = 12, 0.6, 4000
    self_count = np.zeros(L)
    src_hist = [np.zeros(max(l, 1)) for l in range(L)]
    for step in range(steps):
        r = T.sample_route(T.RCLA, L, 0, p, seed=42, step=step)
        assert r[0] == 0                                    # nothing precedes the first layer
        assert all(0 <= r[l] <= l for l in range(L))        # l' <= l, Eq. (3.1)
        for l in range(1, L):
            if r[l] == l:
                self_count[l] += 1
            else:
                src_hist[l][r[l]] += 1
        assert r == T.sample_route(T.RCLA, L, 0, p, seed=42, step=step)   # a pure function of its arguments
    for l in range(1, L):
        # d ~ Bernoulli(p): four standard deviations of a binomial proportion
        assert abs(self_count[l] / steps - p) < 4 * math.sqrt(p * (1 - p) / steps)
        # l' uniform over the l earlier layers
        n = src_hist[l].sum()
        for c in src_hist[l]:
            q = 1.0 / l
            assert abs(c / n - q) < 4 * math.sqrt(q * (1 - q) / n) + 1e-12
    assert T.sample_route(T.RCLA, L, 0, 1.0, 1, 1) == list(range(L))              # p = 1: standard self-attention
    assert all(r < l for l, r in enumerate(T.sample_route(T.RCLA, L, 0, 0.0, 1, 1)) if l)  # p = 0: never self
    # different passes see different strategies
    assert len({tuple(T.sample_route(T.RCLA, L, 0, 0.5, 7, s)) for s in range(50)}) > 40
    assert T.sample_route(T.RCLA, L, 0, 0.5, 7, 3) != T.sample_route(T.RCLA, L, 0, 0.5, 8, 3)


def test_ablation_schemes_of_sec_4_2_3():
    # CLA@k: "layers 0 to k-1 share one KV", and so on
    assert T.sample_route(T.CLA_K, 8, 4, 0.5, 0, 0) == [0, 0, 0, 0, 4, 4, 4, 4]
    assert T.sample_route(T.CLA_K, 7, 3, 0.5, 0, 0) == [0, 0, 0, 3, 3, 3, 6]
    # RD-CLA@k: per layer and step either the fixed shared layer or the local K, V
    fixed = T.sample_route(T.CLA_K, 8, 4, 0.5, 0, 0)
    local = 0
    for step in range(2000):
        r = T.sample_route(T.RDCLA_K, 8, 4, 0.5, 5, step)
        for l in range(8):
            assert r[l] in (l, fixed[l])
        local += sum(r[l] == l for l in (1, 2, 3, 5, 6, 7))
    assert abs(local / (6 * 2000) - 0.5) < 4 * math.sqrt(0.25 / (6 * 2000))
    assert T.sample_route(T.RDCLA_K, 8, 4, 0.0, 5, 1) == fixed
    assert T.sample_route(T.RDCLA_K, 8, 4, 1.0, 5, 1) == list(range(8))


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def test_forward_closed_forms():
    B, S, Hq, Hkv, D = 2, 6, 4, 2, 8
    q, k, v = _rand((B, S, Hq, D), 1), _rand((B, S, Hkv, D), 2), _rand((B, S, Hkv, D), 3)
    scale = 0.37
    out, lse = T.attn_fwd(q, k, v, scale)
    # the first row sees one key: out = that value row, lse = the one score
    for h in range(Hq):
        assert np.allclose(out[:, 0, h], v[:, 0, h // 2])
        assert np.allclose(lse[:, h, 0], scale * np.einsum("bd,bd->b", q[:, 0, h], k[:, 0, h // 2]))
    # equal keys: uniform weights over the visible prefix, lse = score + log(count)
    k_eq = np.broadcast_to(k[:, :1], k.shape).copy()
    out, lse = T.attn_fwd(q, k_eq, v, scale)
    for i in range(S):
        assert np.allclose(out[:, i, 0], v[:, : i + 1, 0].mean(axis=1))
        s = scale * np.einsum("bd,bd->b", q[:, i, 0], k[:, 0, 0])
        assert np.allclose(lse[:, 0, i], s + math.log(i + 1))
    # a row never depends on later keys or values (causal mask)
    k2, v2 = k.copy(), v.copy()
    k2[:, 4:], v2[:, 4:] = 9.0, -9.0
    o1, _ = T.attn_fwd(q, k, v, scale)
    o2, _ = T.attn_fwd(q, k2, v2, scale)
    assert np.array_equal(o1[:, :4], o2[:, :4]) and not np.allclose(o1[:, 4:], o2[:, 4:])
    # ragged: rows beyond a sequence's length are zero, the others ignore the padding
    o3, l3 = T.attn_fwd(q, k2, v2, scale, seq_lens=[4, 6])
    assert np.array_equal(o3[0, :4], o1[0, :4]) and not o3[0, 4:].any() and not l3[0, :, 4:].any()
    assert np.array_equal(o3[1], o2[1])


@pytest.mark.parametrize("lens", [None, [5, 3]])
def test_backward_against_finite_differences_of_the_forward(lens):
    B, S, Hq, Hkv, D = 2, 5, 4, 2, 4
    q, k, v = _rand((B, S, Hq, D), 4), _rand((B, S, Hkv, D), 5), _rand((B, S, Hkv, D), 6)
    d_out = _rand((B, S, Hq, D), 7)
    scale = 0.61
    dq, dk, dv = T.attn_bwd(q, k, v, d_out, scale, lens)

    def loss(q_, k_, v_):
        return float((T.attn_fwd(q_, k_, v_, scale, lens)[0] * d_out).sum())

    eps = 1e-6
    rng = np.random.default_rng(8)
    for name, x, g in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        for _ in range(25):
            idx = tuple(int(rng.integers(n)) for n in x.shape)
            xp, xm = x.copy(), x.copy()
            xp[idx] += eps
            xm[idx] -= eps
            args_p = {"q": (xp, k, v), "k": (q, xp, v), "v": (q, k, xp)}[name]
            args_m = {"q": (xm, k, v), "k": (q, xm, v), "v": (q, k, xm)}[name]
            fd = (loss(*args_p) - loss(*args_m)) / (2 * eps)
            assert abs(fd - g[idx]) < 1e-7 * max(1.0, abs(fd)), (name, idx, fd, g[idx])


def test_backward_invariants():
    B, S, Hq, Hkv, D = 1, 7, 2, 1, 8
    q, k, v = _rand((B, S, Hq, D), 9), _rand((B, S, Hkv, D), 10), _rand((B, S, Hkv, D), 11)
    d_out = _rand((B, S, Hq, D), 12)
    dq, dk, dv = T.attn_bwd(q, k, v, d_out, 0.3)
    # weights of a row sum to one: the value gradients sum to the output gradients
    assert np.allclose(dv.sum(axis=1)[:, 0], d_out.sum(axis=(1, 2)))
    # softmax ignores a constant added to all scores of a row, so moving every key by the same
    # vector changes nothing: the key gradients sum to zero
    assert np.allclose(dk.sum(axis=1), 0.0, atol=1e-12)
    # one visible key: the weight is 1 whatever q is, so the first row's dq vanishes
    assert np.allclose(dq[:, 0], 0.0, atol=1e-14)
    # the last key is seen by the last row only: dv = its weight times that row's d_out
    _, lse = T.attn_fwd(q, k, v, 0.3)
    w = np.exp(0.3 * np.einsum("hd,d->h", q[0, -1], k[0, -1, 0]) - lse[0, :, -1])
    assert np.allclose(dv[0, -1, 0], (w[:, None] * d_out[0, -1]).sum(axis=0))


def test_layer_stack_accumulates_the_gradients_of_all_readers():
    L, B, S, H, D = 4, 1, 4, 1, 4
    qs = [_rand((B, S, H, D), 20 + l) for l in range(L)]
    ks = [_rand((B, S, H, D), 30 + l) for l in range(L)]
    vs = [_rand((B, S, H, D), 40 + l) for l in range(L)]
    dos = [_rand((B, S, H, D), 50 + l) for l in range(L)]
    route = [0, 0, 2, 0]
    outs, dqs, dks, dvs = T.layer_stack_fwd_bwd(qs, ks, vs, dos, route, 0.5)
    # layer 1 is read by nobody: no gradient; layer 0 collects layers 0, 1, 3
    assert not dks[1].any() and not dvs[1].any() and not dks[3].any()
    want = sum(T.attn_bwd(qs[l], ks[0], vs[0], dos[l], 0.5)[1] for l in (0, 1, 3))
    assert np.allclose(dks[0], want)
    # finite difference through the whole stack for one element of layer 0's keys
    def loss(k0):
        tot = 0.0
        for l in range(L):
            src = ks[route[l]] if route[l] else k0
            tot += float((T.attn_fwd(qs[l], src, vs[route[l]], 0.5)[0] * dos[l]).sum())
        return tot
    kp, km = ks[0].copy(), ks[0].copy()
    kp[0, 1, 0, 2] += 1e-6
    km[0, 1, 0, 2] -= 1e-6
    fd = (loss(kp) - loss(km)) / 2e-6
    assert abs(fd - dks[0][0, 1, 0, 2]) < 1e-7 * max(1.0, abs(fd))
