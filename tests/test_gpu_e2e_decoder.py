"""The end-to-end harness against the fp64 decoder oracle on tiny shapes: cached serving
(pre-fill, then teacher-forced decode steps; owner layers project + append, the others skip) must
give the logits of the cache-free whole-sequence evaluation, and the cache must have the size the
paper's KV-MB columns imply."""
import numpy as np
import pytest
import torch

from oracle import decoder_oracle as D
from workloads import gen
from workloads.e2e_decoder import SyntheticDecoder

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("hq,hkv,d,group,qk_norm", [(4, 2, 64, 2, False), (2, 1, 128, 3, False), (2, 2, 128, 1, False),
                                                    (4, 2, 128, 2, True), (2, 1, 64, 4, True)])
def test_cached_serving_matches_whole_sequence_oracle(hq, hkv, d, group, qk_norm):
    L, hidden, mlp, vocab, B, T, steps = 4, 128, 256, 96, 2, 70, 3
    m = SyntheticDecoder(L, hidden, hq, hkv, d, mlp, vocab, group=group, seed=5, sigma=0.09, qk_norm=qk_norm)
    print(f"\nroute {m.route}", flush=True)
    m.start(B, T + steps)
    rng = np.random.default_rng(3)
    tok = torch.from_numpy(rng.integers(0, vocab, (B, T + steps))).cuda()
    got = [m.prefill(tok[:, :T])]
    for s in range(steps):                                   # teacher forcing: the oracle sees the same tokens
        got.append(m.decode_step(tok[:, T + s]))
    got = torch.stack(got, dim=1).float().cpu().double().numpy()          # [B][1 + steps][V]
    w = {k: gen.to_f64(v) for k, v in m.w.items()}
    cos, sin = m.cos.cpu().double().numpy(), m.sin.cpu().double().numpy()
    want = D.logits_all_positions(w, m.route, tok.cpu().numpy(), hq, hkv, d, cos, sin)[:, T - 1:]
    err = np.abs(got - want).max()
    print(f"logits: max |err| {err:.3e}, max |want| {np.abs(want).max():.3e}", flush=True)
    assert err <= 0.03 * np.abs(want).max()                  # a chain of bf16 roundings through four blocks
    assert (got.argmax(-1) == want.argmax(-1)).mean() >= 0.75
    m.close()


def test_kv_cache_size_is_the_papers_column():
    """Tab. 4: 8192 input + 128 generated tokens, Qwen3-8B-scale -> 1170 MB without sharing, 293 with groups of 4."""
    for g, mb in ((1, 1170.0), (4, 292.5)):
        m = SyntheticDecoder.__new__(SyntheticDecoder)
        m.L, m.hq, m.hkv, m.d, m.dtype, m.B = 36, 32, 8, 128, torch.bfloat16, 1
        m.route = [g * (l // g) for l in range(36)]
        assert m.kv_cache_bytes(8192 + 128) / 2 ** 20 == mb


def test_decode_workspace_sized_for_the_capacity_serves_every_shorter_hint():
    """A serving loop sizes its scratch once, for the longest context, and passes a growing length
    hint: the size query must cover every hint up to its argument (split counts are not monotone)."""
    import paper_2604_22782_amd as skv
    cache = skv.skv_cache_alloc(n_layers=1, n_q_heads=32, n_kv_heads=8, head_dim=128, batch=1, max_ctx=8320,
                                dtype=skv.SKV_BF16, route=[0], block_size=0, n_blocks=0)
    top = skv.skv_decode_workspace_bytes(cache, 8320)
    assert all(skv.skv_decode_workspace_bytes(cache, n) <= top for n in range(1, 8321, 37))
    ws = torch.empty(top, dtype=torch.uint8, device="cuda")
    q = torch.randn(1, 32, 128, device="cuda").to(torch.bfloat16)
    out = torch.empty_like(q)
    for n in (1, 255, 257, 4096, 4097, 8193, 8320):
        lens = torch.tensor([n], dtype=torch.int32, device="cuda")
        skv.skv_attn_decode(cache, 0, q, out, lens, n, 0.1, ws)          # raised SKV_ERR_INVALID_ARG at 8193 before
    torch.cuda.synchronize()
    assert skv.skv_cache_device_faults(cache) == 0
    cache.free()


def test_captured_decode_step_replays_like_the_eager_one():
    """The decode step as a HIP graph: every replay, with eager work and synchronisations in between,
    gives bit for bit the logits of the eager step run with the same launch sizes."""
    L, hidden, hq, hkv, d, mlp, vocab, B, T, steps = 4, 128, 4, 2, 64, 256, 96, 2, 40, 6
    rng = np.random.default_rng(9)
    tok = torch.from_numpy(rng.integers(0, vocab, (B, T + steps))).cuda()
    results = {}
    for mode in ("eager", "graph"):
        m = SyntheticDecoder(L, hidden, hq, hkv, d, mlp, vocab, group=2, seed=5, sigma=0.09)
        m.start(B, T + steps)
        m.prefill(tok[:, :T])
        if mode == "graph":
            m.capture_decode()
        outs = []
        for s_ in range(steps):
            if mode == "graph":
                outs.append(m.decode_step_graph(tok[:, T + s_]).clone())
                junk = torch.randn(64, 64, device="cuda") @ torch.randn(64, 64, device="cuda")   # eager work between replays
                torch.cuda.synchronize()
            else:
                outs.append(m.decode_step(tok[:, T + s_], hint=T + steps).clone())
        results[mode] = torch.stack(outs)
        assert int(m.lens[0]) == T + steps
        m.close()
    assert torch.equal(results["eager"], results["graph"])
