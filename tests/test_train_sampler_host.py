"""Host-side checks of the training-time route sampler of the library (no GPU): it draws, decision
by decision, what the oracle draws from the same counters, and rejects bad arguments."""
import ctypes

import pytest

import paper_2604_22782_amd as skv
from oracle import rcla_train_oracle as T


@pytest.mark.parametrize("scheme,k,p", [
    (skv.SKV_TRAIN_RCLA, 0, 0.25), (skv.SKV_TRAIN_RCLA, 0, 0.5), (skv.SKV_TRAIN_RCLA, 0, 0.75),
    (skv.SKV_TRAIN_RCLA, 0, 0.0), (skv.SKV_TRAIN_RCLA, 0, 1.0),
    (skv.SKV_TRAIN_CLA_K, 2, 0.0), (skv.SKV_TRAIN_CLA_K, 4, 0.0), (skv.SKV_TRAIN_CLA_K, 5, 0.0),
    (skv.SKV_TRAIN_RDCLA_K, 2, 0.5), (skv.SKV_TRAIN_RDCLA_K, 4, 0.3),
])
def test_library_sampler_draws_what_the_oracle_draws(scheme, k, p):
    assert (skv.SKV_TRAIN_RCLA, skv.SKV_TRAIN_CLA_K, skv.SKV_TRAIN_RDCLA_K) == (T.RCLA, T.CLA_K, T.RDCLA_K)
    for n_layers in (1, 2, 28, 36):
        for seed in (0, 1, 2 ** 63 + 12345, 2 ** 64 - 1):
            for step in (0, 1, 999, 2 ** 40 + 7):
                got = skv.skv_train_sample_route(scheme, n_layers, k, p, seed, step)
                assert got == T.sample_route(scheme, n_layers, k, p, seed, step), (n_layers, seed, step)


def test_sampler_rejects_bad_arguments():
    lib = skv.lib()
    r = (ctypes.c_int32 * 4)()
    u64, f64 = ctypes.c_uint64, ctypes.c_double
    assert lib.skv_train_sample_route(0, 4, 0, f64(0.5), u64(1), u64(1), None) == 1
    assert lib.skv_train_sample_route(0, 0, 0, f64(0.5), u64(1), u64(1), r) == 1
    assert lib.skv_train_sample_route(3, 4, 2, f64(0.5), u64(1), u64(1), r) == 1     # unknown scheme
    assert lib.skv_train_sample_route(0, 4, 0, f64(1.5), u64(1), u64(1), r) == 1     # p outside [0, 1]
    assert lib.skv_train_sample_route(0, 4, 0, f64(float("nan")), u64(1), u64(1), r) == 1
    assert lib.skv_train_sample_route(1, 4, 0, f64(0.5), u64(1), u64(1), r) == 1     # k < 1
    assert lib.skv_train_sample_route(2, 4, 0, f64(0.5), u64(1), u64(1), r) == 1
    assert lib.skv_train_sample_route(1, 4, 2, f64(7.0), u64(1), u64(1), r) == 0     # CLA@k ignores p
    assert list(r) == [0, 0, 2, 2]


def test_training_calls_reject_bad_arguments_before_touching_the_device():
    lib = skv.lib()
    f = ctypes.c_float
    one = ctypes.c_void_p(16)   # never dereferenced: the checks come first
    n = ctypes.c_size_t(0)
    assert lib.skv_train_bwd_workspace_bytes(2, 100, 8, ctypes.byref(n)) == 0 and n.value == 2 * 100 * 8 * 4
    assert lib.skv_train_bwd_workspace_bytes(0, 100, 8, ctypes.byref(n)) == 1
    assert lib.skv_train_attn_fwd(None, one, one, one, one, one, 1, 8, 2, 1, 128, skv.SKV_BF16, f(1.0), None) == 1
    assert lib.skv_train_attn_fwd(one, one, one, one, one, one, 1, 8, 3, 2, 128, skv.SKV_BF16, f(1.0), None) == 1
    assert lib.skv_train_attn_fwd(one, one, one, one, one, one, 1, 8, 2, 1, 128, skv.SKV_BF16, f(0.0), None) == 1
    assert lib.skv_train_attn_fwd(one, one, one, one, one, one, 1, 8, 2, 1, 96, skv.SKV_BF16, f(1.0), None) == 6
    assert lib.skv_train_attn_fwd(one, one, one, one, one, one, 1, 8, 2, 1, 128, skv.SKV_F32, f(1.0), None) == 6
    args = [one] * 9 + [one, 1, 8, 2, 1, 128, skv.SKV_BF16, f(1.0), one, ctypes.c_size_t(1 << 20), None]
    bad = list(args); bad[6] = None
    assert lib.skv_train_attn_bwd(*bad) == 1
    small = list(args); small[18] = ctypes.c_size_t(8)
    assert lib.skv_train_attn_bwd(*small) == 1                                       # workspace too small
    unsup = list(args); unsup[14] = 80
    assert lib.skv_train_attn_bwd(*unsup) == 6
    assert lib.skv_train_device_faults(None) == 1
