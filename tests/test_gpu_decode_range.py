"""skv_attn_decode_range: sampling-phase attention for a sub-range of the cached sequences (the
building block of the chunk-by-chunk walk over the layers of one sharing group, see the header).
Every range result is compared with the oracle's full-batch decode restricted to those sequences;
rows outside the range must stay untouched."""
import numpy as np
import pytest
import torch

import paper_2604_22782_amd as skv
from oracle import skv_oracle as O
from tests import harness as H
from tests.test_gpu_parity_small import _small
from workloads import gen

pytestmark = pytest.mark.gpu

RANGES = [(0, 5), (1, 3), (4, 1), (2, 2), (0, 1)]


@pytest.mark.parametrize("dtype,hq,hkv,d,paged,kv8", [("bf16", 8, 2, 128, False, False), ("f16", 4, 4, 128, True, False),
                                                      ("f32", 4, 2, 64, False, False), ("bf16", 16, 1, 64, True, False),
                                                      ("bf16", 8, 2, 128, False, True), ("f16", 8, 4, 64, True, True)])
def test_range_decode_matches_oracle(dtype, hq, hkv, d, paged, kv8):
    lens = [700, 33, 1, 2049, 256]
    w = _small(dtype, hq, hkv, d, len(lens), lens, [0, 0, 2, 2], paged, seed=31)
    w.kv8 = kv8      # 8-bit slots: a contiguous slot holds whole row groups per sequence, the range view moves by those
    cache, _ = H.alloc_cache(w)
    H.fill_by_append(cache, w)
    oc = H.oracle_cache(w)
    d_lens = torch.from_numpy(w.kv_lens).cuda()
    max_len = int(w.kv_lens.max())
    for layer in range(w.n_layers):
        q = w.q_decode(layer, "cuda")
        want = O.decode(oc, layer, gen.to_f64(q), w.kv_lens, w.scale)
        for b0, cnt in RANGES:
            nbytes = skv.skv_decode_range_workspace_bytes(cache, cnt, max_len)
            ws = torch.empty(nbytes // 4 + 1, dtype=torch.float32, device="cuda")
            out = torch.full_like(q, 7.0)
            skv.skv_attn_decode_range(cache, layer, b0, cnt, q[b0:], out[b0:], d_lens[b0:], max_len, w.scale, ws)
            got = gen.to_f64(out)
            err = float(np.abs(got[b0:b0 + cnt] - want[b0:b0 + cnt]).max())
            assert err <= H.TOL[dtype], (layer, b0, cnt, err)
            assert (got[:b0] == 7.0).all() and (got[b0 + cnt:] == 7.0).all()
    assert skv.skv_cache_device_faults(cache) == 0
    cache.free()


def test_full_range_is_the_plain_call_bit_for_bit():
    lens = [300, 129, 77]
    w = _small("bf16", 8, 2, 128, 3, lens, [0, 0], False, seed=5)
    cache, _ = H.alloc_cache(w)
    H.fill_by_append(cache, w)
    d_lens = torch.from_numpy(w.kv_lens).cuda()
    ws = H.workspace_for(cache, 300)
    q = w.q_decode(1, "cuda")
    a = H.decode_layer(cache, w, 1, q, d_lens, 300, ws)
    b = torch.empty_like(q)
    skv.skv_attn_decode_range(cache, 1, 0, 3, q, b, d_lens, 300, w.scale, ws)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    cache.free()


def test_range_errors_enqueue_nothing():
    w = _small("bf16", 4, 2, 64, 3, [10, 20, 30], [0, 0], False)
    cache, _ = H.alloc_cache(w)
    H.fill_by_append(cache, w)
    d_lens = torch.from_numpy(w.kv_lens).cuda()
    q = w.q_decode(0, "cuda")
    out = torch.full_like(q, 7.0)
    ws = H.workspace_for(cache, 30)
    for b0, cnt in [(-1, 2), (0, 0), (0, 4), (3, 1), (2, 2)]:
        with pytest.raises(skv.SkvError) as e:
            skv.skv_attn_decode_range(cache, 0, b0, cnt, q, out, d_lens, 30, w.scale, ws)
        assert e.value.status == 1   # SKV_ERR_INVALID_ARG
    with pytest.raises(skv.SkvError):
        skv.skv_decode_range_workspace_bytes(cache, 4, 30)
    with pytest.raises(skv.SkvError):   # workspace of the wrong size class
        skv.skv_attn_decode_range(cache, 0, 0, 2, q, out, d_lens, 30, w.scale, ws[:1])
    torch.cuda.synchronize()
    assert (gen.to_f64(out) == 7.0).all()
    cache.free()
