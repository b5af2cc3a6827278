"""GPU parity of the pipelined pre-fill kernel's work-group mapping at sizes where a work group walks
several pairs of query tiles (Sec. 3.1.1 pre-fill phase: causal attention of a prompt over the layer's
routed slot).  The exhaustive small cases stay below that launch shape and the full-size case samples a few
rows, so here the oracle recomputes one row of EVERY 64-row block of a sequence (plus its first and last
row), for all query heads that share a work group and one other head, on ragged batches: odd and even
tile counts, groups of 1, 2, 4 and 8 query heads per kv head, a chunk offset (kv > q), a one-row and an
empty sequence, contiguous and paged slots."""
import numpy as np
import pytest
import torch

import paper_2604_22782_amd as skv
from oracle import skv_oracle as O
from tests import harness as H
from workloads import configs, gen

pytestmark = pytest.mark.gpu

CASES = [
    # dtype, Hq, Hkv, q_lens, kv offset of sequence 1, paged
    ("bf16", 32, 8, [8100, 5000, 8037, 1, 0, 4097, 6400, 64], 500, False),    # 127 tiles of 64 rows, four pairs
    ("bf16", 16, 8, [8000, 3000, 7999, 1, 0, 4160, 129, 7000], 300, False),   # 63 tiles of 128 rows, two pairs
    ("f16", 32, 32, [7800, 2049, 7700, 255], 77, False),                      # 31 tiles of 256 rows, two pairs
    ("bf16", 32, 4, [4096, 4000, 1000, 0, 2048, 4095, 65, 3333], 1024, True), # 64 tiles, two head sets per kv head
]


@pytest.mark.parametrize("dtype,hq,hkv,q_lens,offset,paged", CASES)
def test_every_query_tile_of_a_long_ragged_prefill_matches_the_oracle(dtype, hq, hkv, q_lens, offset, paged):
    q_lens = np.asarray(q_lens, dtype=np.int32)
    kv_lens = q_lens.copy()
    kv_lens[1] += offset
    kv_lens[kv_lens == 0] = 1          # an empty prompt over a cache that holds one position
    B = len(q_lens)
    w = configs.Workload(f"tiles_{dtype}_{hq}_{hkv}", dtype, 2, hq, hkv, 128, B, [0, 0], kv_lens, 1.0, 0.5, seed=4242)
    if paged:
        table, n_blocks = configs._paged(kv_lens, 16, np.random.default_rng(5))
        w.block_size, w.block_table, w.n_blocks, w.max_ctx = 16, table, n_blocks, table.shape[1] * 16
    print(f"\n{w.name}: q_lens={q_lens.tolist()} kv_lens={kv_lens.tolist()} paged={paged}", flush=True)
    cache, _ = H.alloc_cache(w)
    H.fill_by_append(cache, w)
    max_q, max_kv = int(q_lens.max()), int(kv_lens.max())
    d_q = torch.from_numpy(q_lens).cuda()
    d_kv = torch.from_numpy(kv_lens).cuda()
    layer = 1                           # the reader of layer 0's slot
    q = w.q_prefill(layer, 0, B, 0, max_q, "cuda")
    out = torch.full_like(q, 7.0)
    skv.skv_attn_prefill(cache, layer, q, out, d_q, d_kv, max_q, max_kv, w.scale)
    torch.cuda.synchronize()
    assert skv.skv_last_kernel_name() == "prefill_pipe_kernel"
    assert skv.skv_cache_device_faults(cache) == 0

    rng = np.random.default_rng(99)
    G = hq // hkv
    gh = 4 if G % 4 == 0 else 2 if G % 2 == 0 else 1
    worst = 0.0
    for b in (0, 1, 2):                 # the longest, the one with a chunk offset, one more ragged one
        nq, nkv = int(q_lens[b]), int(kv_lens[b])
        kvh = int(rng.integers(hkv))
        hset = int(rng.integers(G // gh))
        heads = [kvh * G + hset * gh + i for i in range(gh)]
        other = int(rng.integers(hq))
        rows = sorted({0, nq - 1} | {min(nq - 1, r0 + int(rng.integers(64))) for r0 in range(0, nq, 64)})
        for h in heads + [other]:
            K, V = H.oracle_kv_rows(w, layer, b, h // G, nkv)
            qh, oh = gen.to_f64(q[b, rows, h]), gen.to_f64(out[b, rows, h])
            for i, r in enumerate(rows):
                n = nkv - nq + r + 1    # causal with the chunk offset: row r sees the first kv - q + r + 1 keys
                worst = max(worst, float(np.abs(oh[i] - O.attn_one(qh[i], K[:n], V[:n], w.scale)).max()))
        print(f"sequence {b}: {len(rows)} rows x {gh + 1} heads, worst so far {worst:.3e}", flush=True)
    assert worst <= H.TOL[dtype]
    for b in range(B):                  # rows past a sequence's length are not written
        assert (out[b, int(q_lens[b]):] == 7.0).all()
    cache.free()
