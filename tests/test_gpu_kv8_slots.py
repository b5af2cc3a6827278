"""8-bit cache slots (e4m3 codes with a power-of-two scale per (position, kv head); the composition
of depth-wise sharing with KV quantisation that the paper's Sec. 5 leaves open, in this build's
reading): the quantising cache update is compared bit for bit with oracle/kv_quant_oracle.py, and
decode / prefill over such slots element by element with the float64 oracle evaluated on the
dequantised values -- at the same 2e-2 bar as 16-bit slots, because the stored values are exact in
bf16 / fp16 and the kernels compute on them as on a 16-bit cache."""
import numpy as np
import pytest
import torch

import paper_2604_22782_amd as skv
from oracle import kv_quant_oracle as KQ
from oracle import skv_oracle as O
from tests import harness as H
from tests.test_gpu_parity_full import _decode_sampled
from tests.test_gpu_parity_small import CASES, PREFILL_CASES, _small
from workloads import configs, gen

pytestmark = pytest.mark.gpu


def _kv8(w):
    w.kv8 = True
    return w


def _check_kv8_image(cache, w, oc, lens):
    """Codes of K and V and the exponent bytes == the oracle's images, laid out as the header says."""
    k_pool, v_pool, s_pool = H.pool_tensors(cache, w)
    exps = np.concatenate([oc.exps.bits_k, oc.exps.bits_v], axis=-1)          # [slot][b][pos][kvh][2]
    for pool, logical in ((k_pool, oc.bits_k), (v_pool, oc.bits_v), (s_pool, exps)):
        got = pool.numpy()
        if w.block_size:
            want = O.paged_image(logical, w.block_table, w.block_size, w.n_blocks, lens).reshape(got.shape)
        else:
            want = logical.reshape(got.shape)
        if logical is exps:      # rows never written hold exponent byte 127 (scale 1), not 0
            written = np.zeros(logical.shape[:3], dtype=bool)
            for b in range(w.batch):
                written[:, b, : int(lens[b])] = True
            if w.block_size:
                mask = O.paged_image(written[..., None, None].astype(np.uint8), w.block_table, w.block_size,
                                     w.n_blocks, lens).reshape(got.shape[:2] + (1, 1)).astype(bool)
            else:
                mask = written.reshape(got.shape[:2] + (1, 1))
            want = np.where(mask, want, 127)
        assert np.array_equal(got, want)


@pytest.mark.parametrize("dtype,d,paged", [("bf16", 128, False), ("f16", 128, True), ("bf16", 64, True), ("f16", 64, False)])
def test_quantising_append_is_bit_exact(dtype, d, paged):
    """Rows of very different magnitudes (2^-40 .. 2^30 for bf16), rows of zeros, constant rows, rows
    whose scaled values sit exactly half way between two codes."""
    tdt = {"bf16": torch.bfloat16, "f16": torch.float16}[dtype]
    B, S, Hkv = 3, 150, 2
    lens = np.array([150, 77, 1], dtype=np.int32)
    w = _kv8(_small(dtype, 4, Hkv, d, B, lens, [0, 0, 2], paged, seed=5))
    g = torch.Generator().manual_seed(11)
    lo, hi = (-40, 30) if dtype == "bf16" else (-12, 8)
    def rows():
        mag = torch.exp2(torch.empty(B, S, Hkv, 1).uniform_(lo, hi, generator=g))
        x = torch.randn(B, S, Hkv, d, generator=g) * mag
        x[0, 3] = 0.0                                              # all zeros
        x[0, 4] = 1.0                                              # constant
        x[0, 5, :, 1:] = 0.0                                       # one element
        grid = torch.from_numpy(KQ.E4M3_TABLE[:0x7F]).float()
        mid = (grid[:-1] + grid[1:]) / 2                            # exact ties (exact in bf16/fp16: 5 bits)
        x[0, 6, 0] = torch.cat([torch.tensor([448.0]), mid, torch.zeros(1)])[:d]
        x[0, 6, 1] = -torch.cat([torch.tensor([448.0]), mid.flip(0), torch.zeros(1)])[:d]
        x[0, 7] = x[0, 6] * 2.0 ** -9
        return x.to(tdt)
    cache, _ = H.alloc_cache(w, caller_pools=True)
    oc = O.Cache(w.route, B, w.max_ctx, Hkv, d, np.uint8)
    oc.exps = O.Cache(w.route, B, w.max_ctx, Hkv, 1, np.uint8)
    zeros = np.zeros(B, dtype=np.int64)
    for layer in w.owner_layers:
        k, v = rows(), rows()
        skv.skv_kv_append(cache, layer, k.cuda(), v.cuda(), torch.zeros(B, dtype=torch.int32, device="cuda"),
                          torch.from_numpy(lens).cuda(), S)
        (kc, ke), (vc, ve) = KQ.quantise_rows(gen.to_f64(k)), KQ.quantise_rows(gen.to_f64(v))
        oc.append(layer, KQ.dequantise_rows(kc, ke), KQ.dequantise_rows(vc, ve), kc, vc, zeros, lens)
        oc.exps.append(layer, ke[..., None].astype(float), ve[..., None].astype(float), ke[..., None], ve[..., None], zeros, lens)
    _check_kv8_image(cache, w, oc, lens)
    assert skv.skv_cache_device_faults(cache) == 0
    cache.free()


KV8_CASES = [c for c in CASES if c[0] != "f32" and c[3] != 256]


@pytest.mark.parametrize("dtype,hq,hkv,d,lens,route,paged", KV8_CASES)
def test_decode_over_8bit_slots_matches_oracle_exhaustively(dtype, hq, hkv, d, lens, route, paged):
    w = _kv8(_small(dtype, hq, hkv, d, len(lens), lens, route, paged))
    cache, _ = H.alloc_cache(w, caller_pools=paged)
    H.fill_by_append(cache, w, chunk_tokens=w.batch * 500)
    oc = H.oracle_cache(w)
    _check_kv8_image(cache, w, oc, w.kv_lens)
    d_lens = torch.from_numpy(w.kv_lens).cuda()
    max_len = int(w.kv_lens.max())
    ws = H.workspace_for(cache, max_len)
    for layer in range(w.n_layers):
        q = w.q_decode(layer, "cuda")
        out = H.decode_layer(cache, w, layer, q, d_lens, max_len, ws)
        want = O.decode(oc, layer, gen.to_f64(q), w.kv_lens, w.scale)
        err = H.max_abs_err(out, want)
        assert err <= H.TOL[dtype], (layer, err)
    for b, n in enumerate(lens):          # a single cached position returns its (dequantised) V row exactly
        if n == 1:
            want = np.repeat(oc.vals_v[oc.slot[w.n_layers - 1], b, 0], w.group, axis=0)
            assert np.array_equal(gen.to_f64(out[b]), want)
    assert skv.skv_last_kernel_name() == "decode_mfma_kernel"
    assert skv.skv_cache_device_faults(cache) == 0
    cache.free()


KV8_PREFILL = [c for c in PREFILL_CASES if c[0] != "f32"]


@pytest.mark.parametrize("dtype,hq,hkv,d,kv_lens,q_lens,route,paged", KV8_PREFILL)
def test_prefill_over_8bit_slots_matches_oracle_exhaustively(dtype, hq, hkv, d, kv_lens, q_lens, route, paged):
    w = _kv8(_small(dtype, hq, hkv, d, len(kv_lens), kv_lens, route, paged, seed=99))
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
            assert (got[b, nq:] == 7.0).all()
    assert skv.skv_last_kernel_name() == "prefill_mfma_kernel"
    assert skv.skv_cache_device_faults(cache) == 0
    cache.free()


def test_work_queue_decode_over_8bit_slots():
    rng = np.random.default_rng(6)
    lens = np.clip(np.rint(rng.lognormal(np.log(600), 1.0, size=24)), 1, 4000).astype(np.int32)
    lens[3], lens[7] = 4000, 1
    w = _kv8(_small("bf16", 32, 8, 128, len(lens), lens, [0, 0], paged=True, seed=321))
    cache, _ = H.alloc_cache(w)
    H.fill_by_append(cache, w)
    oc = H.oracle_cache(w)
    d_lens = torch.from_numpy(w.kv_lens).cuda()
    max_len = int(w.kv_lens.max())
    ws = H.workspace_for(cache, max_len)
    q = w.q_decode(1, "cuda")
    want = O.decode(oc, 1, gen.to_f64(q), w.kv_lens, w.scale)
    for _ in range(2):
        out = H.decode_layer(cache, w, 1, q, d_lens, max_len, ws)
        assert H.max_abs_err(out, want) <= H.TOL["bf16"]
    got = torch.empty_like(q)
    skv.skv_attn_decode_static(cache, 1, q, got, d_lens, max_len, w.scale)
    assert torch.equal(got, out)
    assert skv.skv_cache_device_faults(cache) == 0
    cache.free()


def test_config2_llama3_decode_8bit_slots_full_size():
    w = _kv8(configs.llama3_decode())
    w.name += "_kv8"
    _decode_sampled(w, seqs_per_layer=1, heads_per_seq=1, all_kv_heads_every=2)


def test_config4_qwen3_paged_ragged_decode_8bit_slots_full_size():
    w = _kv8(configs.qwen3_paged_decode())
    w.name += "_kv8"
    shortest, longest = int(np.argmin(w.kv_lens)), int(np.argmax(w.kv_lens))
    _decode_sampled(w, seqs_per_layer=1, heads_per_seq=1, must_seqs=(shortest, longest), all_kv_heads_every=3)


def test_8bit_slot_descriptor_rules():
    base = dict(n_layers=2, n_q_heads=4, n_kv_heads=2, head_dim=128, batch=2, max_ctx=64, route=[0, 0])
    total = skv.skv_cache_bytes(dtype=skv.SKV_BF16_KV8, **base)
    kvb, scb = skv.skv_cache_pool_bytes(dtype=skv.SKV_BF16_KV8, **base)
    # an 8-bit slot holds whole groups of 128 rows per sequence: 64 positions take 128 rows
    assert kvb == 1 * 2 * 128 * 2 * 128 and scb == 1 * 2 * 128 * 2 * 2 and total == 2 * kvb + scb
    assert skv.skv_cache_pool_bytes(dtype=skv.SKV_BF16, **base) == (2 * 1 * 2 * 64 * 2 * 128, 0)
    paged = dict(base, block_size=16, n_blocks=10)
    assert skv.skv_cache_pool_bytes(dtype=skv.SKV_BF16_KV8, **paged) == (10 * 16 * 2 * 128, 10 * 16 * 2 * 2)
    with pytest.raises(skv.SkvError) as e:                       # a wave-wide load of codes needs blocks of 16 rows
        skv.skv_cache_bytes(dtype=skv.SKV_BF16_KV8, **dict(base, block_size=8, n_blocks=10))
    assert e.value.status == 6
    with pytest.raises(skv.SkvError) as e:                       # head_dim 256 has no 8-bit path
        skv.skv_cache_bytes(dtype=skv.SKV_F16_KV8, **{**base, "head_dim": 256})
    assert e.value.status == 6
    pool = torch.zeros(kvb, dtype=torch.uint8, device="cuda")
    with pytest.raises(skv.SkvError) as e:                       # caller pools need a scale pool too
        skv.skv_cache_alloc(dtype=skv.SKV_BF16_KV8, k_pool=pool, v_pool=pool.clone(), pool_bytes=kvb, **base)
    assert e.value.status == 1
    sc = torch.zeros(scb - 2, dtype=torch.uint8, device="cuda")
    with pytest.raises(skv.SkvError) as e:
        skv.skv_cache_alloc(dtype=skv.SKV_BF16_KV8, k_pool=pool, v_pool=pool.clone(), pool_bytes=kvb,
                            scale_pool=sc, scale_pool_bytes=scb - 2, **base)
    assert e.value.status == 4
    cache = skv.skv_cache_alloc(dtype=skv.SKV_BF16_KV8, **base)
    x = torch.zeros(2, 1, 256, dtype=torch.bfloat16, device="cuda")
    wk = torch.zeros(256, 256, dtype=torch.bfloat16, device="cuda")
    one = torch.ones(2, dtype=torch.int32, device="cuda")
    with pytest.raises(skv.SkvError) as e:                       # the fused projection writes 16-bit slots only
        skv.skv_kv_project_append(cache, 0, x, wk, wk, None, None, one, one, 1)
    assert e.value.status == 6
    cache.free()
