"""Host-side checks of the seeded input generators and the five workload descriptions."""
import numpy as np
import pytest
import torch

from workloads import configs, gen


def test_generator_is_deterministic_and_normal_like():
    idx = torch.arange(1 << 20, dtype=torch.int64)
    a = gen.normal(idx, 7, 1, 1.0, torch.float32)
    b = gen.normal(idx, 7, 1, 1.0, torch.float32)
    assert torch.equal(a, b)
    assert not torch.equal(a, gen.normal(idx, 8, 1, 1.0, torch.float32))
    assert not torch.equal(a, gen.normal(idx, 7, 2, 1.0, torch.float32))
    assert abs(a.mean().item()) < 5e-3 and abs(a.std().item() - 1.0) < 5e-3
    assert abs((a.abs() < 1.0).float().mean().item() - 0.6827) < 5e-3
    h = gen.normal(idx + (1 << 40), 7, 1, 0.5, torch.bfloat16).float()
    assert abs(h.std().item() - 0.5) < 5e-3
    # element i does not depend on which chunk it is generated in
    assert torch.equal(gen.normal(idx[1000:2000], 7, 1, 1.0, torch.float32), a[1000:2000])


def test_rows_do_not_depend_on_chunking():
    w = configs.llama3_decode(batch=4, ctx=64, n_layers=2)
    whole = w.kv_rows("k", 0, 0, 4, 0, 64, "cpu")
    part = w.kv_rows("k", 0, 1, 3, 16, 48, "cpu")
    assert torch.equal(whole[1:3, 16:48], part)
    assert not torch.equal(whole, w.kv_rows("v", 0, 0, 4, 0, 64, "cpu"))


def test_workload_shapes_and_sizes():
    w1 = configs.tiny_f32()
    assert w1.route == [0, 0, 2, 2] and w1.owner_layers == [0, 2]
    w2 = configs.llama3_decode()
    assert len(w2.owner_layers) == 16 and w2.route[5] == 4
    assert w2.decode_bytes_per_layer() == (1 << 30) + (1 << 20)
    w3 = configs.llama3_prefill()
    assert w3.owner_layers == list(range(0, 32, 4))
    assert abs(w3.prefill_flops_per_layer() / 2.199e12 - 1) < 1e-3
    w5 = configs.llama2_mha_decode()
    assert w5.owner_layers == [0, 8, 16, 24] and w5.decode_bytes_per_layer() == (8 << 30) + (512 << 10)


def test_paged_workload_table_is_a_permutation_and_fits_hbm():
    w = configs.qwen3_paged_decode()
    assert w.kv_lens.min() >= 512 and w.kv_lens.max() <= 32768 and len(w.kv_lens) == 128
    need = (w.kv_lens + 15) // 16
    used = np.concatenate([w.block_table[b, :n] for b, n in enumerate(need)])
    assert sorted(used.tolist()) == list(range(w.n_blocks))
    assert w.route[0] == 0 and all(r in (l, w.route[l - 1]) for l, r in enumerate(w.route) if l)
    n_slots = len(w.owner_layers)
    cache = 2 * n_slots * w.n_blocks * 16 * w.n_kv_heads * w.head_dim * 2
    assert cache < 200e9, cache


@pytest.mark.gpu
def test_generator_bits_match_between_host_and_device():
    w = configs.llama3_decode(batch=3, ctx=100, n_layers=2)
    for dt_w in (w, configs.tiny_f32(), configs.llama2_mha_decode(batch=2, ctx=50, n_layers=1)):
        a = dt_w.kv_rows("v", 0, 0, 2, 3, 40, "cpu")
        b = dt_w.kv_rows("v", 0, 0, 2, 3, 40, "cuda").cpu()
        assert np.array_equal(gen.to_bits(a), gen.to_bits(b))
        assert np.array_equal(gen.to_bits(dt_w.q_decode(0, "cpu")), gen.to_bits(dt_w.q_decode(0, "cuda")))
