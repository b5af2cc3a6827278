"""Temporal eviction composed with depth-wise sharing (paper Sec. 5 leaves the composition open;
the reading built here is a sliding window with sinks: positions [sink, first) of a sequence are
dropped from every slot).  Decode over the survivors is compared element by element with the
oracle attending over the surviving positions only; the block-table entries of dropped blocks are
poisoned to prove that nothing reads them."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2604_22782_amd as skv
from oracle import kv_quant_oracle as KQ
from oracle import skv_oracle as O
from tests import harness as H
from tests.test_gpu_parity_small import _small
from workloads import gen

pytestmark = pytest.mark.gpu


def _oracle_decode(oc, w, layer, q64, lens, sink, first):
    out = np.zeros_like(q64)
    s = oc.slot[layer]
    for b in range(w.batch):
        pos = KQ.surviving_positions(int(lens[b]), int(sink[b]), int(first[b]))
        for h in range(w.n_q_heads):
            kvh = h // w.group
            out[b, h] = KQ.attn_over_positions(q64[b, h], oc.vals_k[s, b, :, kvh], oc.vals_v[s, b, :, kvh], pos, w.scale)
    return out


@pytest.mark.parametrize("dtype,paged,kv8,many_splits", [("bf16", True, False, True), ("bf16", True, True, False),
                                                        ("f16", False, False, False), ("bf16", True, False, False),
                                                        ("f16", False, True, False)])
def test_decode_attends_over_surviving_positions_only(dtype, paged, kv8, many_splits):
    rng = np.random.default_rng(9)
    if many_splits:   # ragged batch, work-queue launch shape
        lens = np.clip(np.rint(rng.lognormal(np.log(900), 0.9, size=24)), 40, 4000).astype(np.int32)
        lens[1], lens[2] = 4000, 40
        hq, hkv = 32, 8
    else:
        lens = np.array([3000, 1500, 700, 64, 33, 2047], dtype=np.int32)
        hq, hkv = 8, 2
    B = len(lens)
    w = _small(dtype, hq, hkv, 128, B, lens, [0, 0, 2], paged, seed=41)
    w.kv8 = kv8
    cache, _ = H.alloc_cache(w)
    H.fill_by_append(cache, w)
    oc = H.oracle_cache(w)
    # windows: nothing evicted, sinks of 0 / 32 / 64 positions, windows that start right at the end
    sink = np.array([(0, 32, 64, 0)[b % 4] for b in range(B)], dtype=np.int32)
    first = np.array([min(max(int(sink[b]), (int(lens[b]) * (b % 5) // 5) // 16 * 16), int(lens[b]) // 16 * 16)
                      for b in range(B)], dtype=np.int32)
    sink = np.minimum(sink, first // 32 * 32).astype(np.int32)
    if kv8 and not paged:                            # a contiguous 8-bit slot: the gap is whole groups of 128 rows
        first = (sink + (first - sink) // 128 * 128).astype(np.int32)
    first[3 % B] = sink[3 % B]                       # one sequence with nothing evicted
    assert (sink % 32 == 0).all() and ((first - sink) % 16 == 0).all() and (sink <= first).all() and (first <= lens).all()
    if paged:                                        # dropped blocks: their table entries are poison
        table = w.block_table.copy()
        for b in range(B):
            table[b, sink[b] // 16: first[b] // 16] = -1
        skv.skv_cache_set_block_table(cache, torch.from_numpy(table).cuda())
    d_sink, d_first = torch.from_numpy(sink).cuda(), torch.from_numpy(first).cuda()
    skv.skv_cache_set_eviction(cache, d_sink, d_first)
    survivors = lens - (first - sink)
    max_keys = int(survivors.max())
    d_lens = torch.from_numpy(lens).cuda()
    ws = H.workspace_for(cache, max_keys)
    for layer in (1, 2):
        q = w.q_decode(layer, "cuda")
        want = _oracle_decode(oc, w, layer, gen.to_f64(q), lens, sink, first)
        for _ in range(2):
            out = torch.full_like(q, 7.0)
            skv.skv_attn_decode(cache, layer, q, out, d_lens, max_keys, w.scale, ws)
            assert H.max_abs_err(out, want) <= H.TOL[dtype], layer
        got = torch.full_like(q, 9.0)
        skv.skv_attn_decode_static(cache, layer, q, got, d_lens, max_keys, w.scale)
        assert torch.equal(got, out)
    assert skv.skv_cache_device_faults(cache) == 0
    assert skv.skv_last_kernel_name() == "decode_mfma_kernel"
    # pre-fill over an evicted cache is not built
    with pytest.raises(skv.SkvError) as e:
        skv.skv_attn_prefill(cache, 0, q[:, None].contiguous(), torch.empty_like(q[:, None]),
                             torch.ones(B, dtype=torch.int32, device="cuda"), d_lens, 1, int(lens.max()), w.scale)
    assert e.value.status == 6
    # eviction off again: the full attention (the poisoned table would now be read, so restore it)
    skv.skv_cache_set_eviction(cache, None, None)
    if paged:
        skv.skv_cache_set_block_table(cache, torch.from_numpy(np.ascontiguousarray(w.block_table)).cuda())
    ws = H.workspace_for(cache, int(lens.max()))
    out = H.decode_layer(cache, w, 1, q, d_lens, int(lens.max()), ws)
    assert H.max_abs_err(out, O.decode(oc, 1, gen.to_f64(q), lens, w.scale)) <= H.TOL[dtype]
    assert skv.skv_cache_device_faults(cache) == 0
    cache.free()


def test_impossible_windows_are_contained():
    lens = np.array([500, 500, 500, 500], dtype=np.int32)
    w = _small("bf16", 8, 2, 128, 4, lens, [0, 0], True, seed=43)
    cache, _ = H.alloc_cache(w)
    H.fill_by_append(cache, w)
    oc = H.oracle_cache(w)
    sink = np.array([0, 16, 64, 32], dtype=np.int32)       # 16 is no multiple of the 32-key tile
    first = np.array([128, 128, 32, 512], dtype=np.int32)  # 32 < 64; 512 > 500
    skv.skv_cache_set_eviction(cache, torch.from_numpy(sink).cuda(), torch.from_numpy(first).cuda())
    q = w.q_decode(1, "cuda")
    out = torch.full_like(q, 7.0)
    ws = H.workspace_for(cache, 500)
    skv.skv_attn_decode(cache, 1, q, out, torch.from_numpy(lens).cuda(), 500, w.scale, ws)
    assert skv.skv_cache_device_faults(cache) & 4
    got = gen.to_f64(out)
    assert not got[1:].any()                               # the three impossible ones: zeros
    s_ok, f_ok = sink.copy(), first.copy()
    f_ok[1:] = s_ok[1:] = 0
    want = _oracle_decode(oc, w, 1, gen.to_f64(q), lens, s_ok, f_ok)
    assert np.abs(got[0] - want[0]).max() <= H.TOL["bf16"]
    cache.free()


def test_window_off_the_row_groups_of_an_8bit_slot_is_contained():
    """A contiguous 8-bit slot keeps the rows of a kv head together in groups of 128 rows: a window whose
    gap is not whole groups would put a 32-key tile across two groups, so it is refused like any other
    impossible window (fault word, zero output), while a gap of whole groups is served."""
    lens = np.array([700, 700], dtype=np.int32)
    w = _small("bf16", 8, 2, 128, 2, lens, [0, 0], False, seed=47)
    w.kv8 = True
    cache, _ = H.alloc_cache(w)
    H.fill_by_append(cache, w)
    oc = H.oracle_cache(w)
    sink = np.array([64, 64], dtype=np.int32)
    first = np.array([64 + 256, 64 + 160], dtype=np.int32)     # gaps of 256 (two groups) and 160 (no multiple of 128)
    skv.skv_cache_set_eviction(cache, torch.from_numpy(sink).cuda(), torch.from_numpy(first).cuda())
    q = w.q_decode(1, "cuda")
    out = torch.full_like(q, 7.0)
    ws = H.workspace_for(cache, 700)
    skv.skv_attn_decode(cache, 1, q, out, torch.from_numpy(lens).cuda(), 700, w.scale, ws)
    assert skv.skv_cache_device_faults(cache) & 4
    got = gen.to_f64(out)
    assert not got[1].any()
    want = _oracle_decode(oc, w, 1, gen.to_f64(q), lens, sink, np.array([320, 64]))
    assert np.abs(got[0] - want[0]).max() <= H.TOL["bf16"]
    cache.free()


def test_eviction_is_refused_where_no_kernel_has_it():
    w = _small("f32", 4, 2, 64, 2, [64, 64], [0])
    cache, _ = H.alloc_cache(w)
    z = torch.zeros(2, dtype=torch.int32, device="cuda")
    skv.skv_cache_set_eviction(cache, z, z)
    q = w.q_decode(0, "cuda")
    ws = H.workspace_for(cache, 64)
    with pytest.raises(skv.SkvError) as e:
        skv.skv_attn_decode(cache, 0, q, torch.empty_like(q), torch.from_numpy(w.kv_lens).cuda(), 64, w.scale, ws)
    assert e.value.status == 6
    assert skv.lib().skv_cache_set_eviction(cache.handle, ctypes.c_void_p(z.data_ptr()), None) == 1   # both or neither
    cache.free()
