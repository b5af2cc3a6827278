"""Error behaviour of the compute entry points on a real device: host-detectable problems return
a status and leave the cache untouched; impossible device-side lengths never touch memory outside
the cache and are reported through the fault word."""
import numpy as np
import pytest
import torch

import paper_2604_22782_amd as skv
from tests import harness as H
from workloads import configs

pytestmark = pytest.mark.gpu


def _w(paged=False):
    w = configs.Workload("err", "bf16", 4, 8, 2, 128, 2, [0, 0, 2, 2], np.array([100, 60]), 1.0, 0.5, seed=3)
    if paged:
        table, n_blocks = configs._paged(w.kv_lens, 16, np.random.default_rng(0))
        w.block_size, w.block_table, w.n_blocks, w.max_ctx = 16, table, n_blocks, table.shape[1] * 16
    return w


def test_append_to_non_owner_layer_is_refused_and_cache_untouched():
    w = _w()
    cache, pools = H.alloc_cache(w, caller_pools=True)
    k = w.kv_rows("k", 1, 0, 2, 0, 10, "cuda")
    z = torch.zeros(2, dtype=torch.int32, device="cuda")
    n = torch.full((2,), 10, dtype=torch.int32, device="cuda")
    for layer in (1, 3):
        with pytest.raises(skv.SkvError) as e:
            skv.skv_kv_append(cache, layer, k, k, z, n, 10)
        assert e.value.status == 3
    torch.cuda.synchronize()
    assert not pools[0].any() and not pools[1].any()
    assert skv.skv_cache_slot_of_layer(cache, 3) == (1, False) and skv.skv_cache_slot_of_layer(cache, 2) == (1, True)


def test_host_side_argument_errors():
    w = _w()
    cache, _ = H.alloc_cache(w)
    q = w.q_decode(0, "cuda")
    out = torch.empty_like(q)
    lens = torch.from_numpy(w.kv_lens).cuda()
    ws = H.workspace_for(cache, 100)
    with pytest.raises(skv.SkvError) as e:      # layer out of range
        skv.skv_attn_decode(cache, 4, q, out, lens, 100, w.scale, ws)
    assert e.value.status == 1
    with pytest.raises(skv.SkvError) as e:      # hint above the capacity
        skv.skv_attn_decode(cache, 0, q, out, lens, 101, w.scale, ws)
    assert e.value.status == 4
    with pytest.raises(skv.SkvError) as e:      # workspace too small
        skv.skv_attn_decode(cache, 0, q, out, lens, 100, w.scale, ws[:8])
    assert e.value.status == 1
    with pytest.raises(skv.SkvError) as e:
        skv.skv_attn_prefill(cache, 0, q, out, lens, lens, 1, 1000, w.scale)
    assert e.value.status == 4
    with pytest.raises(skv.SkvError) as e:      # block table on a contiguous cache
        skv.skv_cache_set_block_table(cache, torch.zeros(2, 4, dtype=torch.int32, device="cuda"))
    assert e.value.status == 6
    pw = _w(paged=True)                          # paged cache used before its table is set
    pc = skv.skv_cache_alloc(n_layers=4, n_q_heads=8, n_kv_heads=2, head_dim=128, batch=2, max_ctx=112,
                             dtype=skv.SKV_BF16, route=pw.route, block_size=16, n_blocks=pw.n_blocks)
    with pytest.raises(skv.SkvError) as e:
        skv.skv_attn_decode(pc, 0, q, out, lens, 100, w.scale, ws)
    assert e.value.status == 1


def test_device_side_bad_lengths_and_block_ids_are_contained():
    w = _w(paged=True)
    cache, pools = H.alloc_cache(w, caller_pools=True)
    H.fill_by_append(cache, w)
    assert skv.skv_cache_device_faults(cache) == 0
    snapshot = (pools[0].clone(), pools[1].clone())
    k = w.kv_rows("k", 0, 0, 2, 0, 4, "cuda")
    # rows that would land beyond the capacity are dropped, the rest of the cache is unchanged
    start = torch.tensor([w.max_ctx - 2, w.max_ctx + 5], dtype=torch.int32, device="cuda")
    four = torch.full((2,), 4, dtype=torch.int32, device="cuda")
    skv.skv_kv_append(cache, 0, k, k, start, four, 4)
    assert skv.skv_cache_device_faults(cache) & 1
    # decode with a zero / oversized length: defined (zero) output, fault recorded, no crash
    q = w.q_decode(0, "cuda")
    out = torch.full_like(q, 3.0)
    ws = H.workspace_for(cache, 100)
    bad = torch.tensor([0, 500], dtype=torch.int32, device="cuda")
    skv.skv_attn_decode(cache, 1, q, out, bad, 100, w.scale, ws)
    assert skv.skv_cache_device_faults(cache) & 4
    assert not out.any()
    # a block table entry outside the pool is skipped and reported
    table = torch.from_numpy(w.block_table.copy()).cuda()
    table[0, 1] = w.n_blocks + 7
    table[1, 0] = -3
    skv.skv_cache_set_block_table(cache, table)
    lens = torch.from_numpy(w.kv_lens).cuda()
    skv.skv_attn_decode(cache, 1, q, out, lens, 100, w.scale, ws)
    assert skv.skv_cache_device_faults(cache) & 2
    assert torch.isfinite(out.float()).all()
    qp = w.q_prefill(1, 0, 2, 0, 60, "cuda")
    op = torch.zeros_like(qp)
    ql = torch.tensor([60, 60], dtype=torch.int32, device="cuda")
    skv.skv_attn_prefill(cache, 1, qp, op, ql, lens, 60, 100, w.scale)
    assert skv.skv_last_kernel_name() == "prefill_pipe_kernel"      # its paged variant checks the ids too
    assert skv.skv_cache_device_faults(cache) & 2
    assert torch.isfinite(op.float()).all()
    skv.skv_kv_append(cache, 0, k, k, torch.zeros(2, dtype=torch.int32, device="cuda"), four, 4)
    assert skv.skv_cache_device_faults(cache) & 2
    torch.cuda.synchronize()


@pytest.mark.parametrize("dtype,d,kernel", [("f32", 64, "attn_valu_kernel"), ("bf16", 64, "prefill_mfma_kernel"),
                                            ("bf16", 128, "prefill_pipe_kernel")])
def test_prefill_writes_nothing_for_a_sequence_with_impossible_lengths(dtype, d, kernel):
    """The three pre-fill kernels contain impossible device-side lengths the same way: the fault word
    is raised, the sequence's output stays untouched, the other sequences are computed."""
    from oracle import skv_oracle as O
    from tests.test_gpu_parity_small import _small
    from workloads import gen
    lens = np.array([96, 96, 96], dtype=np.int32)
    w = _small(dtype, 4, 2, d, 3, lens, [0, 0])
    cache, _ = H.alloc_cache(w)
    H.fill_by_append(cache, w)
    oc = H.oracle_cache(w)
    q = w.q_prefill(1, 0, 3, 0, 96, "cuda")
    for bad_q, bad_kv in (([96, 97, 96], [96, 96, 96]), ([96, 50, 96], [96, 40, 96]), ([96, 96, 96], [96, 0, 96])):
        out = torch.full_like(q, 7.0)
        skv.skv_attn_prefill(cache, 1, q, out, torch.tensor(bad_q, dtype=torch.int32, device="cuda"),
                             torch.tensor(bad_kv, dtype=torch.int32, device="cuda"), 96, 96, w.scale)
        assert skv.skv_last_kernel_name() == kernel
        assert skv.skv_cache_device_faults(cache) & 4
        assert (out[1] == 7.0).all()
        want = O.prefill(oc, 1, gen.to_f64(q), [96, 0, 96], [96, 1, 96], w.scale)
        got = gen.to_f64(out)
        assert np.abs(got[[0, 2]] - want[[0, 2]]).max() <= H.TOL[dtype]
    cache.free()


@pytest.mark.parametrize("kv8,paged", [(False, False), (True, False), (False, True)])
def test_library_pools_are_one_allocation_with_the_documented_distance(kv8, paged):
    """skv_cache_alloc places the V pool 384 bytes past a multiple of 1 KiB behind the start of the K pool
    (the decode call streams both at once; pools a multiple of 1 KiB apart meet in the same memory channels)
    and right behind it; appended rows still land where the documented layout says (the pool images
    of the exhaustive tests are read through these pointers)."""
    w = configs.Workload("placement", "bf16", 2, 8, 2, 128, 3, [0, 0], np.array([37, 5, 129], dtype=np.int32), 1.0, 0.5, seed=3)
    w.kv8 = kv8
    if paged:
        table, n_blocks = configs._paged(w.kv_lens, 16, np.random.default_rng(1))
        w.block_size, w.block_table, w.n_blocks, w.max_ctx = 16, table, n_blocks, table.shape[1] * 16
    cache, _ = H.alloc_cache(w)
    n_slots, kp, vp, each = skv.skv_cache_info(cache)
    assert n_slots == 1 and kp % 256 == 0
    assert (vp - kp) % 1024 == 384 and each <= vp - kp < each + 1024 + 384
    cache.free()
