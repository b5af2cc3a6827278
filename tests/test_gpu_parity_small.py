"""GPU parity, exhaustive on small workloads: every output element of the HIP path is compared
with the float64 oracle, and the cache image is compared bit for bit."""
import numpy as np
import pytest
import torch

import paper_2604_22782_amd as skv
from oracle import skv_oracle as O
from tests import harness as H
from workloads import configs, gen

pytestmark = pytest.mark.gpu


def _small(dtype, n_q_heads, n_kv_heads, head_dim, batch, lens, route, paged=False, seed=77):
    lens = np.asarray(lens, dtype=np.int32)
    w = configs.Workload(f"small_{dtype}", dtype, len(route), n_q_heads, n_kv_heads, head_dim, batch,
                         list(route), lens, 1.0, 1.0 if dtype == "f32" else 0.5, seed=seed)
    if paged:
        rng = np.random.default_rng(seed)
        table, n_blocks = configs._paged(lens, 16, rng)
        w.block_size, w.block_table, w.n_blocks = 16, table, n_blocks
        w.max_ctx = table.shape[1] * 16
    return w


def _check_cache_image(cache, w, oc, lens):
    """Physical K/V pools == the oracle's logical image laid out as the header documents."""
    k_pool, v_pool = H.pool_tensors(cache, w)
    for pool, logical in ((k_pool, oc.bits_k), (v_pool, oc.bits_v)):
        got = pool.numpy().view(logical.dtype)
        if w.block_size:
            want = O.paged_image(logical, w.block_table, w.block_size, w.n_blocks, lens)
            want = want.reshape(got.shape)
        else:
            want = logical.reshape(got.shape)
        assert np.array_equal(got, want)


def test_config1_tiny_routed_gqa_f32_prefill_then_decode():
    """4 layers, route [0,0,2,2]: causal prefill of 128 tokens on every layer (append on the two
    owners only), then one decode step per layer (owners append position 128 first)."""
    w = configs.tiny_f32()
    cache, _ = H.alloc_cache(w)
    assert skv.skv_cache_info(cache)[0] == 2
    oc = O.Cache(w.route, w.batch, w.max_ctx, w.n_kv_heads, w.head_dim, np.uint32)
    T = 128
    lens_p = np.full(w.batch, T, dtype=np.int32)
    d_lens_p = torch.from_numpy(lens_p).cuda()
    zeros = torch.zeros(w.batch, dtype=torch.int32, device="cuda")
    for layer in range(w.n_layers):
        if layer in w.owner_layers:
            k = w.kv_rows("k", layer, 0, w.batch, 0, T, "cuda")
            v = w.kv_rows("v", layer, 0, w.batch, 0, T, "cuda")
            skv.skv_kv_append(cache, layer, k, v, zeros, d_lens_p, T)
            oc.append(layer, gen.to_f64(k), gen.to_f64(v), gen.to_bits(k), gen.to_bits(v), np.zeros(2, int), lens_p)
        q = w.q_prefill(layer, 0, w.batch, 0, T, "cuda")
        out = torch.empty_like(q)
        skv.skv_attn_prefill(cache, layer, q, out, d_lens_p, d_lens_p, T, T, w.scale)
        want = O.prefill(oc, layer, gen.to_f64(q), lens_p, lens_p, w.scale)
        assert H.max_abs_err(out, want) <= H.TOL["f32"], layer
    # one decode step
    lens_d = np.full(w.batch, T + 1, dtype=np.int32)
    d_lens_d = torch.from_numpy(lens_d).cuda()
    ws = H.workspace_for(cache, T + 1)
    ones = torch.ones(w.batch, dtype=torch.int32, device="cuda")
    outs = []
    for layer in range(w.n_layers):
        if layer in w.owner_layers:
            k = w.kv_rows("k", layer, 0, w.batch, T, T + 1, "cuda")
            v = w.kv_rows("v", layer, 0, w.batch, T, T + 1, "cuda")
            skv.skv_kv_append(cache, layer, k, v, d_lens_p, ones, 1)
            oc.append(layer, gen.to_f64(k), gen.to_f64(v), gen.to_bits(k), gen.to_bits(v), lens_p, np.ones(2, int))
        q = w.q_decode(layer, "cuda")
        out = H.decode_layer(cache, w, layer, q, d_lens_d, T + 1, ws)
        want = O.decode(oc, layer, gen.to_f64(q), lens_d, w.scale)
        assert H.max_abs_err(out, want) <= H.TOL["f32"], layer
        outs.append(out)
    _check_cache_image(cache, w, oc, lens_d)
    assert skv.skv_cache_device_faults(cache) == 0
    # layers that share a slot give identical outputs for identical queries
    q = w.q_decode(0, "cuda")
    same = [H.decode_layer(cache, w, l, q, d_lens_d, T + 1, ws).clone() for l in range(4)]
    assert torch.equal(same[0], same[1]) and torch.equal(same[2], same[3]) and not torch.equal(same[0], same[2])


CASES = [
    # dtype, Hq, Hkv, D, lens, route, paged
    ("f32", 4, 2, 64, [1, 2, 65, 300], [0, 0, 2, 2], False),
    ("f32", 8, 1, 128, [257, 33], [0, 1, 1], True),
    ("f32", 2, 2, 256, [70, 5, 131], [0, 0], False),
    ("bf16", 32, 8, 128, [1, 17, 640, 1500], [0, 0, 2, 0], False),
    ("bf16", 8, 2, 128, [513, 31, 1100], [0, 1, 1, 1], True),
    ("f16", 4, 4, 128, [1200, 64, 1], [0, 0, 0], False),
    ("f16", 16, 2, 64, [100, 777], [0, 1], True),
    ("bf16", 16, 1, 64, [2049, 3], [0, 0], False),
    ("bf16", 4, 2, 256, [300, 45], [0, 0, 2], True),
]


@pytest.mark.parametrize("dtype,hq,hkv,d,lens,route,paged", CASES)
def test_decode_matches_oracle_exhaustively(dtype, hq, hkv, d, lens, route, paged):
    w = _small(dtype, hq, hkv, d, len(lens), lens, route, paged)
    cache, _ = H.alloc_cache(w, caller_pools=True)
    H.fill_by_append(cache, w, chunk_tokens=w.batch * 500)     # several append chunks
    oc = H.oracle_cache(w)
    _check_cache_image(cache, w, oc, w.kv_lens)
    d_lens = torch.from_numpy(w.kv_lens).cuda()
    max_len = int(w.kv_lens.max())
    ws = H.workspace_for(cache, max_len)
    for layer in range(w.n_layers):
        q = w.q_decode(layer, "cuda")
        out = H.decode_layer(cache, w, layer, q, d_lens, max_len, ws)
        want = O.decode(oc, layer, gen.to_f64(q), w.kv_lens, w.scale)
        err = H.max_abs_err(out, want)
        assert err <= H.TOL[dtype], (layer, err)
    # a single cached position returns its V row exactly
    for b, n in enumerate(lens):
        if n == 1:
            src_slot = oc.slot[w.n_layers - 1]
            want = np.repeat(oc.vals_v[src_slot, b, 0], w.group, axis=0)
            assert np.array_equal(gen.to_f64(out[b]), want)
    assert skv.skv_cache_device_faults(cache) == 0


PREFILL_CASES = [
    # dtype, Hq, Hkv, D, kv_lens, q_lens, route, paged
    ("f32", 4, 2, 64, [200, 77, 5], [200, 30, 1], [0, 0, 2, 2], False),
    ("f32", 2, 1, 128, [130, 64], [130, 0], [0, 1], True),
    ("bf16", 8, 2, 128, [300, 129, 256, 7], [300, 129, 100, 7], [0, 0, 2], False),
    ("bf16", 32, 8, 128, [260, 515], [260, 131], [0, 0], True),
    ("f16", 4, 4, 128, [333, 128], [333, 1], [0, 1, 1], False),
    ("bf16", 4, 1, 64, [400, 63], [400, 63], [0, 0], True),
    ("f16", 16, 2, 64, [257], [200], [0], False),
    # several 256-row work groups, rows that end inside a 64-row wave block, chunk offsets
    # (kv > q), an empty and a one-row sequence, MHA and 8-head groups: the pipelined kernel
    ("bf16", 4, 1, 128, [700, 900, 64, 300], [700, 333, 0, 1], [0, 0, 2, 2], False),
    ("f16", 2, 2, 128, [513, 1025], [513, 257], [0, 1], False),
    ("bf16", 8, 1, 128, [320, 65], [129, 65], [0], False),
    # the same through a block table: the pipelined kernel's paged variant (one block id per wave
    # and tile), lengths that end inside a block, a tile, a 256-row group; chunk offsets; MHA
    ("bf16", 4, 1, 128, [700, 900, 64, 300], [700, 333, 0, 1], [0, 0, 2, 2], True),
    ("f16", 2, 2, 128, [513, 1025, 17], [513, 257, 17], [0, 1], True),
    ("bf16", 8, 1, 128, [320, 65, 1], [129, 65, 1], [0], True),
]


@pytest.mark.parametrize("dtype,hq,hkv,d,kv_lens,q_lens,route,paged", PREFILL_CASES)
def test_prefill_matches_oracle_exhaustively(dtype, hq, hkv, d, kv_lens, q_lens, route, paged):
    w = _small(dtype, hq, hkv, d, len(kv_lens), kv_lens, route, paged, seed=99)
    cache, _ = H.alloc_cache(w)
    H.fill_by_append(cache, w)
    oc = H.oracle_cache(w)
    max_q, max_kv = max(max(q_lens), 1), int(max(kv_lens))
    d_q = torch.tensor(q_lens, dtype=torch.int32, device="cuda")
    d_kv = torch.from_numpy(w.kv_lens).cuda()
    for layer in range(w.n_layers):
        q = w.q_prefill(layer, 0, w.batch, 0, max_q, "cuda")
        out = torch.full_like(q, 7.0)
        skv.skv_attn_prefill(cache, layer, q, out, d_q, d_kv, max_q, max_kv, w.scale)
        want = O.prefill(oc, layer, gen.to_f64(q), q_lens, kv_lens, w.scale)
        got = gen.to_f64(out)
        for b, nq in enumerate(q_lens):
            err = float(np.max(np.abs(got[b, :nq] - want[b, :nq]))) if nq else 0.0
            assert err <= H.TOL[dtype], (layer, b, err)
            assert (got[b, nq:] == 7.0).all()           # padding rows are not written
    assert skv.skv_cache_device_faults(cache) == 0


def test_decode_equals_last_prefill_row_and_chunked_prefill():
    w = _small("bf16", 8, 2, 128, 2, [384, 200], [0, 0])
    cache, _ = H.alloc_cache(w)
    H.fill_by_append(cache, w)
    d_kv = torch.from_numpy(w.kv_lens).cuda()
    q = w.q_prefill(1, 0, 2, 0, 200, "cuda")
    full = torch.zeros_like(q)
    d_q = torch.tensor([200, 200], dtype=torch.int32, device="cuda")
    skv.skv_attn_prefill(cache, 1, q, full, d_q, d_kv, 200, 384, w.scale)
    ws = H.workspace_for(cache, 384)
    dec = H.decode_layer(cache, w, 1, q[:, -1].contiguous(), d_kv, 384, ws)
    assert (dec.float() - full[:, -1].float()).abs().max().item() <= 2e-2
    # second chunk alone: rows 100..199 are the last 100 positions
    part = torch.zeros_like(q[:, 100:])
    d_q2 = torch.tensor([100, 100], dtype=torch.int32, device="cuda")
    skv.skv_attn_prefill(cache, 1, q[:, 100:].contiguous(), part, d_q2, d_kv, 100, 384, w.scale)
    assert (part.float() - full[:, 100:].float()).abs().max().item() <= 2e-2


def test_decode_work_queue_mode_ragged_batch():
    """A ragged batch with many splits per sequence runs the decode kernel in its persistent mode
    (work groups pull (sequence, kv head, split) items from a counter).  Every output element is
    checked, twice in a row (the counters must be back at rest after a launch), and a sequence with
    an impossible length is contained."""
    rng = np.random.default_rng(5)
    lens = np.clip(np.rint(rng.lognormal(np.log(600), 1.0, size=24)), 1, 4000).astype(np.int32)
    lens[3], lens[7] = 4000, 1
    w = _small("bf16", 32, 8, 128, len(lens), lens, [0, 0], paged=True, seed=123)
    cache, _ = H.alloc_cache(w)
    H.fill_by_append(cache, w)
    oc = H.oracle_cache(w)
    d_lens = torch.from_numpy(w.kv_lens).cuda()
    max_len = int(w.kv_lens.max())
    ws = H.workspace_for(cache, max_len)
    # 24 sequences x 8 kv heads x ceil(4000 / 256) splits: far more grid slots than items with keys
    q = w.q_decode(1, "cuda")
    want = O.decode(oc, 1, gen.to_f64(q), w.kv_lens, w.scale)
    for _ in range(2):
        out = H.decode_layer(cache, w, 1, q, d_lens, max_len, ws)
        assert H.max_abs_err(out, want) <= H.TOL["bf16"]
    assert skv.skv_cache_device_faults(cache) == 0
    bad = w.kv_lens.copy()
    bad[5] = 0
    bad[9] = max_len + 1
    out = H.decode_layer(cache, w, 1, q, torch.from_numpy(bad).cuda(), max_len, ws)
    assert skv.skv_cache_device_faults(cache) & 4
    got = gen.to_f64(out)
    ok = [b for b in range(len(lens)) if b not in (5, 9)]
    assert np.abs(got[ok] - want[ok]).max() <= H.TOL["bf16"]
    assert not got[5].any() and not got[9].any()
    out = H.decode_layer(cache, w, 1, q, d_lens, max_len, ws)      # and the queue still works afterwards
    assert H.max_abs_err(out, want) <= H.TOL["bf16"]


def test_scale_must_be_positive():
    w = _small("bf16", 8, 2, 128, 2, [64, 64], [0])
    cache, _ = H.alloc_cache(w)
    q = w.q_decode(0, "cuda")
    lens = torch.from_numpy(w.kv_lens).cuda()
    ws = H.workspace_for(cache, 64)
    for bad in (0.0, -1.0, float("nan")):
        with pytest.raises(skv.SkvError) as e:
            skv.skv_attn_decode(cache, 0, q, torch.empty_like(q), lens, 64, bad, ws)
        assert e.value.status == 1
        with pytest.raises(skv.SkvError) as e:
            skv.skv_attn_prefill(cache, 0, q, torch.empty_like(q), lens, lens, 1, 64, bad)
        assert e.value.status == 1


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_prefill_with_growing_scores_rescales_often(dtype):
    """Keys whose norm grows with the position: the running row maximum keeps jumping by far more
    than the lazy-rescale threshold, so the rescale path of the prefill kernels (new maximum,
    deferred O and row-sum rescale) runs on most tiles instead of once."""
    tdt = {"bf16": torch.bfloat16, "f16": torch.float16}[dtype]
    B, S, Hq, Hkv, D = 2, 700, 2, 1, 128
    route = [0, 0]
    w = _small(dtype, Hq, Hkv, D, B, [S, 450], route, False, seed=123)
    g = torch.Generator().manual_seed(7)
    grow = (0.1 + 0.012 * torch.arange(S, dtype=torch.float32)).view(1, S, 1, 1)
    k = (torch.randn(B, S, Hkv, D, generator=g) * grow).to(tdt)
    v = torch.randn(B, S, Hkv, D, generator=g).to(tdt)
    q = torch.randn(B, S, Hq, D, generator=g).to(tdt)
    lens = np.array([S, 450], dtype=np.int32)
    cache, _ = H.alloc_cache(w)
    d_lens = torch.from_numpy(lens).cuda()
    zeros = torch.zeros(B, dtype=torch.int32, device="cuda")
    skv.skv_kv_append(cache, 0, k.cuda(), v.cuda(), zeros, d_lens, S)
    oc = O.Cache(route, B, w.max_ctx, Hkv, D, np.uint16)
    oc.append(0, gen.to_f64(k), gen.to_f64(v), gen.to_bits(k), gen.to_bits(v), np.zeros(B, dtype=np.int64), lens)
    for layer in (0, 1):
        out = torch.full_like(q, 7.0, device="cuda")
        skv.skv_attn_prefill(cache, layer, q.cuda(), out, d_lens, d_lens, S, S, w.scale)
        want = O.prefill(oc, layer, gen.to_f64(q), lens, lens, w.scale)
        got = gen.to_f64(out)
        for b in range(B):
            err = float(np.abs(got[b, : lens[b]] - want[b, : lens[b]]).max())
            assert err <= H.TOL[dtype], (layer, b, err)
    assert skv.skv_cache_device_faults(cache) == 0
    cache.free()


@pytest.mark.gpu
@pytest.mark.parametrize("block", [32, 128])
def test_paged_prefill_with_larger_blocks(block):
    """Blocks of 32 and 128 positions (the pipelined kernel's paged variant takes any power of two
    from 16 on: a wave's rows of a tile lie inside one block, at an offset that now varies)."""
    lens = np.array([700, 333, 129], dtype=np.int32)
    w = configs.Workload("blk", "bf16", 2, 4, 2, 128, 3, [0, 0], lens, 1.0, 0.5, seed=61)
    table, n_blocks = configs._paged(lens, block, np.random.default_rng(block))
    w.block_size, w.block_table, w.n_blocks, w.max_ctx = block, table, n_blocks, table.shape[1] * block
    cache, _ = H.alloc_cache(w)
    H.fill_by_append(cache, w)
    oc = H.oracle_cache(w)
    q_lens = [700, 100, 129]
    d_q = torch.tensor(q_lens, dtype=torch.int32, device="cuda")
    d_kv = torch.from_numpy(lens).cuda()
    for layer in (0, 1):
        q = w.q_prefill(layer, 0, 3, 0, 700, "cuda")
        out = torch.full_like(q, 7.0)
        skv.skv_attn_prefill(cache, layer, q, out, d_q, d_kv, 700, 700, w.scale)
        assert skv.skv_last_kernel_name() == "prefill_pipe_kernel"
        want = O.prefill(oc, layer, gen.to_f64(q), q_lens, lens, w.scale)
        got = gen.to_f64(out)
        for b, nq in enumerate(q_lens):
            assert np.abs(got[b, :nq] - want[b, :nq]).max() <= H.TOL["bf16"], (layer, b)
            assert (got[b, nq:] == 7.0).all()
    assert skv.skv_cache_device_faults(cache) == 0
    cache.free()


@pytest.mark.gpu
@pytest.mark.parametrize("kind", ["high", "low", "jump_even_half_tile", "jump_odd_half_tile", "sink_then_low"])
def test_prefill_fast_stream_hands_over_on_extreme_scores(kind):
    """The bf16 pre-fill kernel computes the weights of tiles below the diagonal without a running
    maximum as long as the row sums stay inside [2^-64, 2^64], and otherwise redoes the half tile
    with one and continues in the general stream.  Scores far above that range from the first tile
    on, far below it, jumping up in the first or in the second half of a tile (the two ways out), and
    a row whose weight sits in the first key while everything after it is far below."""
    B, S, Hq, Hkv, D = 2, 900, 2, 1, 128
    route = [0, 0]
    w = _small("bf16", Hq, Hkv, D, B, [S, 600], route, False, seed=321)
    g = torch.Generator().manual_seed(17)
    q = torch.randn(B, S, Hq, D, generator=g)
    k = torch.randn(B, S, Hkv, D, generator=g)
    v = torch.randn(B, S, Hkv, D, generator=g)
    pos = torch.arange(S).view(1, S, 1, 1)
    if kind == "high":
        k = k * 20.0                                    # scores of +-100 in log2 units
    elif kind == "low":
        u = torch.randn(D, generator=g)
        q = u.expand(B, S, Hq, D) + 0.05 * q            # every score is about -8 |u|^2 / sqrt(D)
        k = -8.0 * u.expand(B, S, Hkv, D) + 0.05 * k
    elif kind.startswith("jump"):
        at = 320 if kind == "jump_even_half_tile" else 352
        k = torch.where(pos >= at, k * 30.0, k)
    else:
        u = torch.randn(D, generator=g)
        q = u.expand(B, S, Hq, D) + 0.05 * q
        k = torch.where(pos == 0, 0.0 * k, -8.0 * u.expand(B, S, Hkv, D) + 0.05 * k)
    q, k, v = q.to(torch.bfloat16), k.to(torch.bfloat16), v.to(torch.bfloat16)
    lens = np.array([S, 600], dtype=np.int32)
    cache, _ = H.alloc_cache(w)
    d_lens = torch.from_numpy(lens).cuda()
    zeros = torch.zeros(B, dtype=torch.int32, device="cuda")
    skv.skv_kv_append(cache, 0, k.cuda(), v.cuda(), zeros, d_lens, S)
    oc = O.Cache(route, B, w.max_ctx, Hkv, D, np.uint16)
    oc.append(0, gen.to_f64(k), gen.to_f64(v), gen.to_bits(k), gen.to_bits(v), np.zeros(B, dtype=np.int64), lens)
    out = torch.full_like(q, 7.0, device="cuda")
    skv.skv_attn_prefill(cache, 1, q.cuda(), out, d_lens, d_lens, S, S, w.scale)
    assert skv.skv_last_kernel_name() == "prefill_pipe_kernel"
    want = O.prefill(oc, 1, gen.to_f64(q), lens, lens, w.scale)
    got = gen.to_f64(out)
    for b in range(B):
        err = float(np.abs(got[b, : lens[b]] - want[b, : lens[b]]).max())
        assert np.isfinite(got[b, : lens[b]]).all() and err <= H.TOL["bf16"], (kind, b, err)
    assert skv.skv_cache_device_faults(cache) == 0
    cache.free()
