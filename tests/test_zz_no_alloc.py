"""skv_attn_decode_static: the decode entry point that allocates nothing (its split partials and
work counter live in a scratch array of the library's device image).  Through the C ABI, against
skv_attn_decode on the same inputs (same kernels, same split: equal bits) and against the oracle,
on two calls in a row, the second with a smaller input, in both launch shapes of the kernel."""
import numpy as np
import pytest
import torch

import paper_2604_22782_amd as skv
from oracle import skv_oracle as O
from tests import harness as H
from tests.test_gpu_parity_small import _small
from workloads import gen

pytestmark = pytest.mark.gpu


def test_static_scratch_decode_matches_workspace_decode_and_oracle():
    rng = np.random.default_rng(11)
    lens = np.clip(np.rint(rng.lognormal(np.log(700), 0.9, size=24)), 1, 4000).astype(np.int32)
    lens[2], lens[5] = 4000, 3
    w = _small("bf16", 32, 8, 128, len(lens), lens, [0, 0], paged=True, seed=77)
    cache, _ = H.alloc_cache(w)
    H.fill_by_append(cache, w)
    oc = H.oracle_cache(w)
    q = w.q_decode(1, "cuda")
    assert skv.skv_static_scratch_bytes() == 64 << 20
    # first call: ragged batch, many splits per sequence (persistent launch shape, merge launch);
    # second call: the same cache read up to 900 positions only (plain grid, fewer splits)
    for cap in (4000, 900):
        cur = np.minimum(w.kv_lens, cap).astype(np.int32)
        d_lens = torch.from_numpy(cur).cuda()
        max_len = int(cur.max())
        assert skv.skv_decode_workspace_bytes(cache, max_len) <= skv.skv_static_scratch_bytes()
        ws = H.workspace_for(cache, max_len)
        ref = torch.full_like(q, 7.0)
        skv.skv_attn_decode(cache, 1, q, ref, d_lens, max_len, w.scale, ws)
        got = torch.full_like(q, 9.0)
        skv.skv_attn_decode_static(cache, 1, q, got, d_lens, max_len, w.scale)
        torch.cuda.synchronize()
        assert torch.equal(got, ref), cap
        want = O.decode(oc, 1, gen.to_f64(q), cur, w.scale)
        assert H.max_abs_err(got, want) <= H.TOL["bf16"], cap
    assert skv.skv_cache_device_faults(cache) == 0
    cache.free()


def test_static_scratch_decode_rejects_what_does_not_fit():
    """A launch whose split partials exceed the scratch array is refused with SKV_ERR_CAPACITY and
    nothing is enqueued (1024 sequences of up to 8192 positions: 65 MiB of partials; the paged pool
    behind it is tiny, the call fails on the host before anything reads it)."""
    desc = dict(n_layers=1, n_q_heads=32, n_kv_heads=8, head_dim=128, batch=1024, max_ctx=8192,
                dtype=skv.SKV_BF16, route=[0], block_size=16, n_blocks=64)
    cache = skv.skv_cache_alloc(**desc)
    skv.skv_cache_set_block_table(cache, torch.zeros(1024, 512, dtype=torch.int32, device="cuda"))
    q = torch.zeros(1024, 32, 128, dtype=torch.bfloat16, device="cuda")
    out = torch.full_like(q, 5.0)
    d_lens = torch.full((1024,), 16, dtype=torch.int32, device="cuda")
    assert skv.skv_decode_workspace_bytes(cache, 8192) > skv.skv_static_scratch_bytes()
    with pytest.raises(skv.SkvError) as e:
        skv.skv_attn_decode_static(cache, 0, q, out, d_lens, 8192, 1.0)
    assert e.value.status == 4
    torch.cuda.synchronize()
    assert (out == 5.0).all()
    # a shorter hint fits and runs
    skv.skv_attn_decode_static(cache, 0, q, out, d_lens, 16, 1.0)
    torch.cuda.synchronize()
    assert (out == 0.0).all()          # zero V rows
    assert skv.skv_cache_device_faults(cache) == 0
    cache.free()
