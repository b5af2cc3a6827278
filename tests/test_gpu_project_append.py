"""GPU parity of the fused owner-layer K/V projection + cache update against the fp64 oracle:
every written cache row element by element, everything else untouched."""
import numpy as np
import pytest
import torch

import paper_2604_22782_amd as skv
from oracle import project_oracle as P
from tests import harness as H
from tests.test_gpu_parity_small import _small
from workloads import gen

pytestmark = pytest.mark.gpu

TDT = {"bf16": torch.bfloat16, "f16": torch.float16}


def _tables(n_pos, d, base=10000.0):
    inv = base ** (-np.arange(d // 2) * 2.0 / d)
    ang = np.arange(n_pos)[:, None] * inv[None, :]
    return np.cos(ang), np.sin(ang)


def _logical_rows(pool, w, slot, b, n):
    """float64 [n][Hkv][D] of positions 0..n-1 of sequence b in `slot` of a pool read back from the device."""
    bits = pool[slot]
    if w.block_size:
        pos = np.arange(n)
        rows = w.block_table[b][pos >> 4].astype(np.int64) * 16 + (pos & 15)
    else:
        rows = b * w.max_ctx + np.arange(n)
    return gen.to_f64(bits[torch.from_numpy(rows)].view(TDT[w.dtype]))


CASES = [
    # dtype, Hkv, D, hidden, lens (capacity), start_pos, new_lens, max_new, paged, rope
    ("bf16", 2, 128, 256, [100, 60], [0, 5], [70, 33], 70, False, True),
    ("f16", 2, 64, 128, [40, 64, 17], [3, 0, 16], [20, 64, 1], 64, True, False),
    ("bf16", 1, 128, 512, [400, 400], [10, 0], [300, 257], 300, True, True),
    ("f16", 4, 128, 192, [9, 9, 9], [0, 8, 3], [9, 1, 0], 9, False, True),
    ("bf16", 2, 64, 64, [300], [0], [300], 300, False, True),
    # few tokens and a long hidden axis: the launch splits the hidden axis and sums fp32 partials
    ("bf16", 2, 128, 2048, [50, 50, 50], [49, 0, 7], [1, 1, 1], 1, True, True),
    ("f16", 1, 64, 1024, [40], [2], [33], 33, False, True),
    # prompt-sized launches (one split, 256 x 256 tiles straight into LDS): ragged last tile whose
    # upper waves stage no token at all, 2 to 10 ring slots, tile order by XCD (8 | token tiles) and plain
    ("bf16", 4, 128, 64, [4200], [0], [4111], 4111, False, True),
    ("f16", 8, 64, 128, [1100, 1100, 1100, 1100], [0, 5, 0, 76], [1024, 1024, 1024, 1024], 1024, True, True),
    ("bf16", 8, 128, 192, [2100], [17], [2048], 2048, True, False),
    ("f16", 2, 128, 320, [8300, 8300], [0, 0], [8192, 7000], 8192, False, True),
    # mid-sized prompts: the 256 x 256 tiles alone would leave most of the chip idle, so the hidden axis
    # is split over them as well (2 and 4 splits), partial sums finished by the second kernel
    ("bf16", 8, 128, 1024, [2100], [17], [2048], 2048, True, True),
    ("f16", 8, 128, 2048, [1100, 1100], [0, 3], [1024, 1000], 1024, False, True),
]


@pytest.mark.parametrize("dtype,Hkv,D,hidden,lens,start,new,max_new,paged,rope", CASES)
def test_projected_rows_match_oracle(dtype, Hkv, D, hidden, lens, start, new, max_new, paged, rope):
    print(f"\nproject+append {dtype} Hkv={Hkv} D={D} hidden={hidden} new={new} paged={paged} rope={rope}", flush=True)
    B = len(lens)
    route = [0, 0, 2]
    w = _small(dtype, 2 * Hkv, Hkv, D, B, lens, route, paged, seed=41)
    cache, _ = H.alloc_cache(w)
    g = torch.Generator().manual_seed(3)
    x = torch.randn(B, max_new, hidden, generator=g).to(TDT[dtype])
    wk = (torch.randn(Hkv * D, hidden, generator=g) / np.sqrt(hidden)).to(TDT[dtype])
    wv = (torch.randn(Hkv * D, hidden, generator=g) / np.sqrt(hidden)).to(TDT[dtype])
    cos = sin = d_cos = d_sin = None
    if rope:
        cos, sin = _tables(int(max(lens)), D)
        d_cos = torch.from_numpy(cos.astype(np.float32)).cuda()
        d_sin = torch.from_numpy(sin.astype(np.float32)).cuda()
        cos, sin = d_cos.cpu().double().numpy(), d_sin.cpu().double().numpy()   # the tables as the kernel sees them
    d_start = torch.tensor(start, dtype=torch.int32, device="cuda")
    d_new = torch.tensor(new, dtype=torch.int32, device="cuda")
    norm_w = d_norm = None
    if hidden % 128 == 0:          # half of the cases also normalise the keys per head
        d_norm = (1.0 + 0.2 * torch.randn(D, generator=g)).float().cuda()
        norm_w = d_norm.cpu().double().numpy()
    ws_bytes = skv.skv_kv_project_workspace_bytes(cache, max_new, hidden)
    ws = torch.empty(max(ws_bytes, 4) // 4, dtype=torch.float32, device="cuda")
    print(f"workspace {ws_bytes} bytes", flush=True)
    for layer in (0, 2):
        skv.skv_kv_project_append(cache, layer, x.cuda(), wk.cuda(), wv.cuda(), d_cos, d_sin, d_start, d_new, max_new, ws,
                                  k_norm_weight=d_norm, k_norm_eps=1e-5)
    with pytest.raises(skv.SkvError) as e:          # layer 1 owns no slot: nothing to project, nothing to store
        skv.skv_kv_project_append(cache, 1, x.cuda(), wk.cuda(), wv.cuda(), d_cos, d_sin, d_start, d_new, max_new)
    assert e.value.status == 3
    assert skv.skv_cache_device_faults(cache) == 0

    positions = np.array(start)[:, None] + np.arange(max_new)[None, :]
    positions = np.minimum(positions, (cos.shape[0] - 1) if rope else positions)   # rows beyond new_lens are not compared
    want_k, want_v = P.project_kv(gen.to_f64(x), gen.to_f64(wk), gen.to_f64(wv), Hkv, D, positions, cos, sin,
                                  k_norm_weight=norm_w, k_norm_eps=1e-5)
    k_pool, v_pool = H.pool_tensors(cache, w)
    for slot in (0, 1):
        for b in range(B):
            cap = int(lens[b])
            got_k = _logical_rows(k_pool, w, slot, b, cap)
            got_v = _logical_rows(v_pool, w, slot, b, cap)
            s0, n = start[b], new[b]
            if n:       # a sequence may have no new token at all: then only "untouched" is checked below
                assert np.abs(got_k[s0:s0 + n] - want_k[b, :n]).max() <= H.TOL[dtype], (slot, b)
                assert np.abs(got_v[s0:s0 + n] - want_v[b, :n]).max() <= H.TOL[dtype], (slot, b)
            # within one rounding of the exact value, relative to its size
            rel = 2.0 ** -8 if dtype == "bf16" else 2.0 ** -10
            assert (np.abs(got_k[s0:s0 + n] - want_k[b, :n]) <= rel * np.abs(want_k[b, :n]) + 2e-3).all()
            # positions outside the update keep the zeros the pool was allocated with
            assert not got_k[:s0].any() and not got_k[s0 + n:].any() and not got_v[:s0].any() and not got_v[s0 + n:].any()
    cache.free()


def test_position_beyond_the_table_or_capacity_is_dropped_and_reported():
    w = _small("bf16", 2, 1, 128, 1, [32], [0], False, seed=1)
    cache, _ = H.alloc_cache(w)
    g = torch.Generator().manual_seed(4)
    x = torch.randn(1, 8, 64, generator=g).to(torch.bfloat16).cuda()
    wk = torch.randn(128, 64, generator=g).to(torch.bfloat16).cuda()
    cos, sin = _tables(4, 128)
    d_cos, d_sin = torch.from_numpy(cos.astype(np.float32)).cuda(), torch.from_numpy(sin.astype(np.float32)).cuda()
    zero = torch.zeros(1, dtype=torch.int32, device="cuda")
    eight = torch.full((1,), 8, dtype=torch.int32, device="cuda")
    ws = torch.empty(max(skv.skv_kv_project_workspace_bytes(cache, 8, 64), 4) // 4, dtype=torch.float32, device="cuda")
    skv.skv_kv_project_append(cache, 0, x, wk, wk, d_cos, d_sin, zero, eight, 8, ws)  # table has 4 positions
    assert skv.skv_cache_device_faults(cache) == 1                                    # SKV_FAULT_APPEND_RANGE
    k_pool, v_pool = H.pool_tensors(cache, w)
    assert k_pool[0, :4].any() and not k_pool[0, 4:].any()                            # K rows 4..7 dropped
    skv.skv_kv_project_append(cache, 0, x, wk, wk, None, None, torch.full((1,), 28, dtype=torch.int32, device="cuda"), eight, 8, ws)
    assert skv.skv_cache_device_faults(cache) == 1                                    # positions 32..35 exceed the capacity
    with pytest.raises(skv.SkvError) as e:
        skv.skv_kv_project_append(cache, 0, x[:, :, :48].contiguous(), wk[:, :48].contiguous(), wk[:, :48].contiguous(),
                                  None, None, zero, eight, 8)
    assert e.value.status == 6                                                        # hidden not a multiple of 64
    cache.free()


def test_projection_at_the_size_the_benchmark_times_sampled_rows():
    """The prompt of the prefill workload (4 x 8192 tokens, hidden 4096, 8 kv heads of 128, bf16:
    the launch bench.py times, tile kernel, one split) and one decode token of the decode workload
    (64 tokens: hidden axis split 16 ways): sampled token rows against the fp64 oracle, every other
    row of the pools untouched where the update does not reach."""
    from workloads import configs
    hidden, rng = 4096, np.random.default_rng(8)
    for w, new in ((configs.llama3_prefill(), None), (configs.llama3_decode(n_layers=2), 1)):
        S = int(w.kv_lens.max())
        new = S if new is None else new
        B, Hkv, D = w.batch, w.n_kv_heads, w.head_dim
        print(f"\nprojection at bench size: {B} x {new} tokens, hidden {hidden}", flush=True)
        cache, _ = H.alloc_cache(w)
        g = torch.Generator(device="cuda").manual_seed(7)
        x = torch.randn(B, new, hidden, generator=g, device="cuda").to(torch.bfloat16)
        wk = (torch.randn(Hkv * D, hidden, generator=g, device="cuda") / hidden ** 0.5).to(torch.bfloat16)
        wv = (torch.randn(Hkv * D, hidden, generator=g, device="cuda") / hidden ** 0.5).to(torch.bfloat16)
        cos, sin = _tables(S, D)
        d_cos, d_sin = torch.from_numpy(cos.astype(np.float32)).cuda(), torch.from_numpy(sin.astype(np.float32)).cuda()
        cos, sin = d_cos.cpu().double().numpy(), d_sin.cpu().double().numpy()
        start = torch.full((B,), S - new, dtype=torch.int32, device="cuda")
        lens = torch.full((B,), new, dtype=torch.int32, device="cuda")
        ws = torch.empty(max(skv.skv_kv_project_workspace_bytes(cache, new, hidden), 4) // 4, dtype=torch.float32, device="cuda")
        layer = w.owner_layers[0]
        skv.skv_kv_project_append(cache, layer, x, wk, wv, d_cos, d_sin, start, lens, new, ws)
        assert skv.skv_cache_device_faults(cache) == 0
        k_pool, v_pool = H.pool_tensors(cache, w)
        slot = 0
        wk64, wv64 = gen.to_f64(wk.cpu()), gen.to_f64(wv.cpu())
        worst = 0.0
        for b in range(B) if new > 1 else rng.choice(B, 8, replace=False):
            rows = np.unique(np.concatenate([[0, new - 1], rng.integers(0, new, 14)])) if new > 1 else np.array([0])
            xs = gen.to_f64(x[b, torch.from_numpy(rows).cuda()].cpu())[None]            # [1][n][hidden]
            pos = (S - new + rows)[None]
            want_k, want_v = P.project_kv(xs, wk64, wv64, Hkv, D, pos, cos, sin)
            got_k = gen.to_f64(k_pool[slot][torch.from_numpy(b * w.max_ctx + S - new + rows)].view(torch.bfloat16))
            got_v = gen.to_f64(v_pool[slot][torch.from_numpy(b * w.max_ctx + S - new + rows)].view(torch.bfloat16))
            worst = max(worst, np.abs(got_k - want_k[0]).max(), np.abs(got_v - want_v[0]).max())
            assert (np.abs(got_k - want_k[0]) <= 2.0 ** -8 * np.abs(want_k[0]) + 2e-3).all(), b
            assert (np.abs(got_v - want_v[0]) <= 2.0 ** -8 * np.abs(want_v[0]) + 2e-3).all(), b
        print(f"worst |err| {worst:.2e}", flush=True)
        assert worst <= H.TOL["bf16"]
        if new == 1:      # positions before the appended one keep the zeros the pool was allocated with
            assert not k_pool[slot][: S - 1].any()
        cache.free()
        del x, k_pool, v_pool
        torch.cuda.empty_cache()
