"""Seeded random shapes for the operators added around the hot path (training attention, fused
projection): lengths around every tile boundary, odd batch sizes, every head grouping, both dtypes
and head sizes, each case against the fp64 oracle."""
import numpy as np
import pytest
import torch

import paper_2604_22782_amd as skv
from oracle import project_oracle as P
from oracle import rcla_train_oracle as T
from tests import harness as H
from tests.test_gpu_parity_small import _small
from tests.test_gpu_project_append import _logical_rows, _tables
from tests.test_gpu_train_attention import _grad_tol, _run_fwd
from workloads import gen

pytestmark = pytest.mark.gpu
TDT = {"bf16": torch.bfloat16, "f16": torch.float16}


def test_training_attention_random_shapes():
    rng = np.random.default_rng(2604)
    for case in range(14):
        dtype = ["bf16", "f16"][case % 2]
        D = [64, 128][(case // 2) % 2]
        Hkv = int(rng.choice([1, 2, 3]))
        Hq = Hkv * int(rng.choice([1, 2, 4, 5]))
        B = int(rng.integers(1, 4))
        S = int(rng.choice([1, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, 300, 385]))
        lens = [int(rng.integers(1, S + 1)) for _ in range(B)]
        lens[int(rng.integers(B))] = S
        print(f"\ncase {case}: {dtype} D={D} Hq={Hq} Hkv={Hkv} B={B} S={S} lens={lens}", flush=True)
        g = torch.Generator().manual_seed(case)
        mk = lambda h: torch.randn(B, S, h, D, generator=g).to(TDT[dtype])
        q, k, v, do = mk(Hq), mk(Hkv), mk(Hkv), mk(Hq)
        scale = float(rng.uniform(0.5, 1.5)) / np.sqrt(D)
        d_lens = torch.tensor(lens, dtype=torch.int32, device="cuda")
        out, lse = _run_fwd(q, k, v, d_lens, scale)
        dq = torch.full_like(q, 7.0, device="cuda")
        dk = torch.zeros(B, S, Hkv, D, dtype=torch.float32, device="cuda")
        dv = torch.zeros_like(dk)
        ws = torch.empty(skv.skv_train_bwd_workspace_bytes(B, S, Hq) // 4, dtype=torch.float32, device="cuda")
        skv.skv_train_attn_bwd(q.cuda(), k.cuda(), v.cuda(), out, lse, do.cuda(), dq, dk, dv, d_lens, scale, ws)
        f = gen.to_f64
        w_out, w_lse = T.attn_fwd(f(q), f(k), f(v), scale, lens)
        w_dq, w_dk, w_dv = T.attn_bwd(f(q), f(k), f(v), f(do), scale, lens)
        for b, n in enumerate(lens):
            assert np.abs(f(out)[b, :n] - w_out[b, :n]).max() <= H.TOL[dtype], (case, b)
            assert np.abs(lse.cpu().double().numpy()[b, :, :n] - w_lse[b, :, :n]).max() <= 2e-3, (case, b)
            for name, got, want in (("dq", f(dq), w_dq), ("dk", dk.cpu().double().numpy(), w_dk),
                                    ("dv", dv.cpu().double().numpy(), w_dv)):
                assert np.abs(got[b, :n] - want[b, :n]).max() <= _grad_tol(dtype, want[b, :n]), (case, name, b)
            assert (f(dq)[b, n:] == 7.0).all() and not dk[b, n:].any() and not dv[b, n:].any()
    assert skv.skv_train_device_faults() == 0


def test_fused_projection_random_shapes():
    rng = np.random.default_rng(22782)
    for case in range(12):
        dtype = ["bf16", "f16"][case % 2]
        D = [64, 128][(case // 2) % 2]
        Hkv = int(rng.choice([1, 2, 3, 4]))
        hidden = 64 * int(rng.integers(1, 9))
        B = int(rng.integers(1, 4))
        max_new = int(rng.choice([1, 2, 31, 32, 33, 64, 100, 255, 256, 257, 290]))
        new = [int(rng.integers(0, max_new + 1)) for _ in range(B)]
        new[int(rng.integers(B))] = max_new
        start = [int(rng.integers(0, 40)) for _ in range(B)]
        lens = [s + n + int(rng.integers(0, 5)) for s, n in zip(start, new)]      # capacities
        paged = bool(case % 3 == 0)
        rope = bool(case % 4 != 3)
        print(f"\ncase {case}: {dtype} D={D} Hkv={Hkv} hidden={hidden} B={B} new={new} start={start} paged={paged} rope={rope}", flush=True)
        w = _small(dtype, 2 * Hkv, Hkv, D, B, [max(n, 1) for n in lens], [0, 0], paged, seed=case)
        cache, _ = H.alloc_cache(w)
        g = torch.Generator().manual_seed(100 + case)
        x = torch.randn(B, max_new, hidden, generator=g).to(TDT[dtype])
        wk = (torch.randn(Hkv * D, hidden, generator=g) / np.sqrt(hidden)).to(TDT[dtype])
        wv = (torch.randn(Hkv * D, hidden, generator=g) / np.sqrt(hidden)).to(TDT[dtype])
        cos = sin = d_cos = d_sin = None
        if rope:
            cos, sin = _tables(int(max(lens)) + 1, D)
            d_cos, d_sin = torch.from_numpy(cos.astype(np.float32)).cuda(), torch.from_numpy(sin.astype(np.float32)).cuda()
            cos, sin = d_cos.cpu().double().numpy(), d_sin.cpu().double().numpy()
        ws = torch.empty(max(skv.skv_kv_project_workspace_bytes(cache, max_new, hidden), 4) // 4, dtype=torch.float32, device="cuda")
        skv.skv_kv_project_append(cache, 0, x.cuda(), wk.cuda(), wv.cuda(), d_cos, d_sin,
                                  torch.tensor(start, dtype=torch.int32, device="cuda"),
                                  torch.tensor(new, dtype=torch.int32, device="cuda"), max_new, ws)
        assert skv.skv_cache_device_faults(cache) == 0
        positions = np.array(start)[:, None] + np.arange(max_new)[None, :]
        if rope:
            positions = np.minimum(positions, cos.shape[0] - 1)
        want_k, want_v = P.project_kv(gen.to_f64(x), gen.to_f64(wk), gen.to_f64(wv), Hkv, D, positions, cos, sin)
        k_pool, v_pool = H.pool_tensors(cache, w)
        for b in range(B):
            cap = int(w.kv_lens[b])
            got_k, got_v = _logical_rows(k_pool, w, 0, b, cap), _logical_rows(v_pool, w, 0, b, cap)
            s0, n = start[b], new[b]
            if n:
                assert np.abs(got_k[s0:s0 + n] - want_k[b, :n]).max() <= H.TOL[dtype], (case, b)
                assert np.abs(got_v[s0:s0 + n] - want_v[b, :n]).max() <= H.TOL[dtype], (case, b)
            assert not got_k[:s0].any() and not got_k[s0 + n:].any() and not got_v[:s0].any() and not got_v[s0 + n:].any()
        cache.free()
