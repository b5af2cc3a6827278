"""The pins of the oracles must fail when a plausible mistake is planted in the oracle:
each case edits one line of the oracle's source (a dropped term, a sign, a transposition, a wrong
index), loads the edited copy as a module and runs the pin tests against it.  Everything here is
CPU-only and touches no GPU code."""
import importlib.util
import os
import sys
import types

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _mutant(name, old, new):
    path = os.path.join(ROOT, "oracle", name + ".py")
    src = open(path).read()
    assert src.count(old) == 1, (name, old)          # the edit must hit exactly one place
    if old.startswith("    if k_norm_weight is not None:"):    # the normalisation moves behind the rotation
        src = src.replace("    return k, v", "    if k_norm_weight is not None:\n        k = k / np.sqrt((k * k).mean(axis=-1, keepdims=True) + k_norm_eps) * k_norm_weight\n    return k, v")
    import oracle  # noqa: F401  (the edited copy keeps the package's relative imports)
    mod = types.ModuleType(f"oracle.{name}_mutant")
    mod.__package__ = "oracle"
    mod.__file__ = path
    exec(compile(src.replace(old, new), path, "exec"), mod.__dict__)
    return mod


def _pins_fail(test_module, attr, mutant, tests, monkeypatch):
    monkeypatch.setattr(test_module, attr, mutant)
    failed = []
    for t in tests:
        try:
            t()
        except (Exception, pytest.fail.Exception):    # AssertionError, an error the mistake provokes, "did not raise"
            failed.append(getattr(t, "__name__", "case"))
    return failed


TRAIN_MISTAKES = [
    ("0xBF58476D1CE4E5B9", "0xBF58476D1CE4E5B7"),                                  # a digit of the generator
    ("< p else 0", "> p else 0"),                                                    # decision inverted
    ("route.append(((draw(seed, step, l, 1) >> 32) * l) >> 32)",
     "route.append(((draw(seed, step, l, 1) >> 32) * (l + 1)) >> 32)"),              # source may be the layer itself
    ("route.append(l if bernoulli(seed, step, l, p) else k * (l // k))",
     "route.append(k * (l // k) if bernoulli(seed, step, l, p) else l)"),            # RD-CLA coin swapped
    ("route.append(k * (l // k))\n        elif scheme == RDCLA_K", "route.append(k * (l // k) + k - 1)\n        elif scheme == RDCLA_K"),  # last layer of the group
    ("lse[b, h, :n] = (m + np.log(z))[:, 0]", "lse[b, h, :n] = np.log(z)[:, 0]"),  # maximum dropped
    ("out[b, :n, h] = (e / z) @ v[b, :n, h // G]", "out[b, :n, h] = (e / z) @ v[b, :n, h % (Hq // G)]"),   # wrong kv head
    ("dv[b, :n, g] += p.T @ do", "dv[b, :n, g] = p.T @ do"),                         # heads of a group not added
    ("ds = p * (dp - (p * dp).sum(axis=1, keepdims=True))", "ds = p * dp"),          # softmax Jacobian: term dropped
    ("dq[b, :n, h] = scale * (ds @ k[b, :n, g])", "dq[b, :n, h] = ds @ k[b, :n, g]"),   # scale dropped
    ("dk[b, :n, g] += scale * (ds.T @ q[b, :n, h])", "dk[b, :n, g] += -scale * (ds.T @ q[b, :n, h])"),  # sign
    ("dp = do @ v[b, :n, g].T", "dp = do @ k[b, :n, g].T"),                           # wrong operand
    ("dks[src] += dk", "dks[l] += dk"),                                               # gradient sent to the reader
]


@pytest.mark.parametrize("old,new", TRAIN_MISTAKES)
def test_training_oracle_pins_catch(old, new, monkeypatch):
    from tests import test_rcla_train_oracle_pins as pins
    tests = [pins.test_mix_reproduces_the_published_splitmix64_sequence, pins.test_rcla_sampling_rule_of_sec_3_2,
             pins.test_ablation_schemes_of_sec_4_2_3, pins.test_forward_closed_forms,
             lambda: pins.test_backward_against_finite_differences_of_the_forward(None),
             lambda: pins.test_backward_against_finite_differences_of_the_forward([5, 3]),
             pins.test_backward_invariants, pins.test_layer_stack_accumulates_the_gradients_of_all_readers]
    for t in tests:
        if not hasattr(t, "__name__") or t.__name__ == "<lambda>":
            t.__name__ = "finite_differences"
    assert _pins_fail(pins, "T", _mutant("rcla_train_oracle", old, new), tests, monkeypatch), (old, new)


PROJECT_MISTAKES = [
    ('k = np.einsum("bth,fh->btf", x, w_k)', 'k = np.einsum("bth,hf->btf", x, w_k)'),   # weights transposed
    ('v = np.einsum("bth,fh->btf", x, w_v)', 'v = np.einsum("bth,fh->btf", x, w_k)'),   # V from the K weights
    ("k[..., :half] = lo * c - hi * s", "k[..., :half] = lo * c + hi * s"),             # rotation sign
    ("k[..., half:] = hi * c + lo * s", "k[..., half:] = hi * c"),                      # term dropped
    ("c = rope_cos[positions][:, :, None, :]", "c = rope_cos[positions * 0][:, :, None, :]"),   # position ignored
    ("lo, hi = k[..., :half].copy(), k[..., half:].copy()", "lo, hi = k[..., 0::2].copy(), k[..., 1::2].copy()"),  # interleaved pairs
    # the optional per-head normalisation of K
    ("(k * k).mean(axis=-1, keepdims=True) + k_norm_eps", "(k * k).sum(axis=-1, keepdims=True) + k_norm_eps"),   # sum for mean
    ("(k * k).mean(axis=-1, keepdims=True) + k_norm_eps", "(k * k).mean(axis=-1, keepdims=True)"),               # eps dropped
    ("(k * k).mean(axis=-1, keepdims=True) + k_norm_eps", "(k * k).mean(axis=(-2, -1), keepdims=True) + k_norm_eps"),   # over all heads
    ("+ k_norm_eps) * k_norm_weight", "+ k_norm_eps) * k_norm_weight[::-1]"),                                     # weight reversed
    ("k = k / np.sqrt((k * k).mean(", "v = v / np.sqrt((k * k).mean("),                                          # V normalised, K not
    ("    if k_norm_weight is not None:\n        k = k / np.sqrt((k * k).mean(axis=-1, keepdims=True) + k_norm_eps) * k_norm_weight\n    if rope_cos is not None:",
     "    if rope_cos is not None:"),                                                                             # (first half of moving the normalisation behind the rotation)
]


@pytest.mark.parametrize("old,new", PROJECT_MISTAKES)
def test_projection_oracle_pins_catch(old, new, monkeypatch):
    from tests import test_project_oracle_pins as pins
    tests = [pins.test_identity_weights_and_linearity, pins.test_rotation_properties, pins.test_key_normalisation]
    assert _pins_fail(pins, "P", _mutant("project_oracle", old, new), tests, monkeypatch), (old, new)


def test_the_unedited_oracles_pass_through_the_same_harness(monkeypatch):
    from tests import test_project_oracle_pins as pp
    from tests import test_rcla_train_oracle_pins as tp
    same_t = _mutant("rcla_train_oracle", "RCLA, CLA_K, RDCLA_K = 0, 1, 2", "RCLA, CLA_K, RDCLA_K = 0, 1, 2")
    same_p = _mutant("project_oracle", "half = head_dim // 2", "half = head_dim // 2")
    assert _pins_fail(tp, "T", same_t, [tp.test_forward_closed_forms, tp.test_backward_invariants,
                                        tp.test_ablation_schemes_of_sec_4_2_3], monkeypatch) == []
    assert _pins_fail(pp, "P", same_p, [pp.test_identity_weights_and_linearity, pp.test_rotation_properties], monkeypatch) == []

MAIN_MISTAKES = [
    ("route.append(max(earlier))", "route.append(min(earlier))"),                          # farthest instead of nearest owner
    ("        if route[r] != r:\n", "        if False:\n"),                                # a source that owns no slot is accepted
    ("if not 0 <= r <= l:", "if not 0 <= r:"),                                              # a later layer as source is accepted
    ("rank = {l: i for i, l in enumerate(own)}", "rank = {l: l for i, l in enumerate(own)}"),   # slot = layer number, not its rank
    ("return 2 * n_cached_layers * n_kv_heads * head_dim * elem_bytes", "return n_cached_layers * n_kv_heads * head_dim * elem_bytes"),   # K only
    ("    scores = scale * (K @ q)\n", "    scores = K @ q\n"),                             # scale dropped
    ("    return w / np.sum(w)\n", "    return w / np.max(w)\n"),                           # normalised by the maximum
    ("K = cache.vals_k[s, b, : pos_q + 1, h // G, :]", "K = cache.vals_k[s, b, : pos_q, h // G, :]"),        # the token does not see its own key
    ("V = cache.vals_v[s, b, : pos_q + 1, h // G, :]", "V = cache.vals_v[s, b, : pos_q + 1, h % hkv, :]"),   # interleaved instead of contiguous head groups
    ("    s = cache.slot[layer]\n    K =", "    s = cache.slot[max(layer - 1, 0)]\n    K ="),  # the neighbour's slot
    ("Hq, n - nq + i, q[b, i, h], scale)", "Hq, i, q[b, i, h], scale)"),                   # rows aligned to the start of the cache
    ("Hq, n - 1, q[b, h], scale)", "Hq, n - 2, q[b, h], scale)"),                           # decode one position early
    ("l = sum(s[1] * np.exp(s[0] - m) for s in states)", "l = sum(s[1] for s in states)"),  # merge: sums not rescaled
    ("        if self.route[layer] != layer:\n", "        if False:\n"),                    # a non-owner may append
    ("self.vals_v[s, b, p0 + i] = v_vals[b, i]", "self.vals_v[s, b, p0 + i] = k_vals[b, i]"),   # V rows from K
    ("blk = int(block_table[b][pos // block_size])", "blk = int(block_table[b][pos % block_size])"),   # block index from the offset
]


@pytest.mark.parametrize("old,new", MAIN_MISTAKES)
def test_main_oracle_pins_catch(old, new, monkeypatch):
    from tests import test_oracle_pins as pins
    tests = []
    for name in dir(pins):
        if not name.startswith("test_"):
            continue
        fn = getattr(pins, name)
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        if not marks:
            tests.append(fn)
            continue
        assert len(marks) == 1                         # one parametrize per pin: expand it by hand
        names = [a.strip() for a in marks[0].args[0].split(",")]
        for values in marks[0].args[1]:
            values = values if len(names) > 1 else (values,)
            tests.append((lambda f, kw: (lambda: f(**kw)))(fn, dict(zip(names, values))))
    assert len(tests) >= 30
    failed = _pins_fail(pins, "O", _mutant("skv_oracle", old, new), tests, monkeypatch)
    assert failed, (old, new)

DECODER_MISTAKES = [
    ("return x / np.sqrt((x * x).mean(axis=-1, keepdims=True) + eps) * w", "return x / np.sqrt((x * x).sum(axis=-1, keepdims=True) + eps) * w"),   # sum for mean
    ("return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)", "return np.concatenate([lo * c + hi * s, hi * c - lo * s], axis=-1)"),    # rotation the other way
    ("        k, v = kv[src]\n", "        k, v = kv[max(s for s in kv)]\n"),                       # the latest cache instead of the routed one
    ("k[b, : t + 1, hd // G], v[b, : t + 1, hd // G], scale)", "k[b, : t + 1, hd % n_kv_heads], v[b, : t + 1, hd % n_kv_heads], scale)"),   # head grouping
    ("k[b, : t + 1, hd // G], v[b, : t + 1, hd // G], scale)", "k[b, :, hd // G], v[b, :, hd // G], scale)"),                                 # no causal mask
    ('        x = x + np.einsum("btf,hf->bth", attn.reshape(B, T, -1), w[f"{l}.wo"])', '        x = np.einsum("btf,hf->bth", attn.reshape(B, T, -1), w[f"{l}.wo"])'),   # residual dropped
    ("gate / (1.0 + np.exp(-gate)) * up", "1.0 / (1.0 + np.exp(-gate)) * up"),                       # sigmoid for silu
    ('h2 = rmsnorm(x, w[f"{l}.norm2"])', 'h2 = rmsnorm(x, w[f"{l}.norm1"])'),                          # wrong norm weights
    ('return np.einsum("bth,vh->btv", rmsnorm(x, w["final_norm"]), w["emb"])', 'return np.einsum("bth,vh->btv", x, w["emb"])'),   # final norm dropped
    ("scale = 1.0 / np.sqrt(head_dim)", "scale = 1.0 / head_dim"),                                    # softmax scale
    ('        if f"{l}.q_norm" in w:\n            q = rmsnorm(q, w[f"{l}.q_norm"])\n        q = rope_heads(q, pos, cos, sin)',
     '        q = rope_heads(q, pos, cos, sin)\n        if f"{l}.q_norm" in w:\n            q = rmsnorm(q, w[f"{l}.q_norm"])'),   # q normalised after the rotation
    ('k_norm_weight=w.get(f"{l}.k_norm"), k_norm_eps=1e-6)', 'k_norm_weight=w.get(f"{l}.q_norm"), k_norm_eps=1e-6)'),   # k with q's weights
]


@pytest.mark.parametrize("old,new", DECODER_MISTAKES)
def test_decoder_oracle_pins_catch(old, new, monkeypatch):
    from tests import test_decoder_oracle_pins as pins
    tests = [pins.test_rmsnorm_and_causality_and_skipped_projections,
             lambda: pins.test_identity_route_is_a_standard_decoder_built_from_library_routines(False),
             lambda: pins.test_identity_route_is_a_standard_decoder_built_from_library_routines(True),
             pins.test_a_layer_reads_the_layer_its_route_names_not_the_latest_cache]
    assert _pins_fail(pins, "D", _mutant("decoder_oracle", old, new), tests, monkeypatch), (old, new)


QUANT_MISTAKES = [
    ("return s * (1.0 + m / 8.0) * 2.0 ** (e - 7)", "return s * (1.0 + m / 8.0) * 2.0 ** (e - 8)"),     # exponent bias of the other 8-bit format
    ("return s * (m / 8.0) * 2.0 ** -6", "return s * (m / 8.0) * 2.0 ** -7"),                            # subnormal scale
    ("if e == 0xF and m == 0x7:", "if e == 0xF:"),                                                        # a whole binade lost to NaN
    ("e = k - 9 if f <= 0.875 else k - 8", "e = k - 9 if f < 0.875 else k - 8"),                          # 448 itself gets the larger scale
    ("e = k - 9 if f <= 0.875 else k - 8", "e = k - 8"),                                                  # always the larger scale
    ("e = np.where(f <= 0.875, k - 9, k - 8)", "e = np.where(f <= 0.875, k - 8, k - 7)"),                 # the array form disagrees with the rule
    ("np.where(lo % 2 == 0, lo, hi)", "hi"),                                                              # ties away from zero
    ("codes = round_to_e4m3(np.ldexp(flat, -e[:, None]))", "codes = round_to_e4m3(np.ldexp(flat, -e[:, None] - 1))"),   # scaled once too often
    ("return np.ldexp(E4M3_TABLE[codes], e[..., None])", "return np.ldexp(E4M3_TABLE[codes], e[..., None] + 1)"),       # dequantised with the wrong exponent
    ("np.concatenate([np.arange(0, sink), np.arange(first, n)])", "np.concatenate([np.arange(0, sink), np.arange(first + 1, n)])"),   # window starts late
    ("    Ks, Vs = K[positions], V[positions]\n", "    Ks, Vs = K, V\n"),                                  # eviction ignored
    ("    s = scale * (Ks @ q)\n", "    s = Ks @ q\n"),                                                     # scale dropped
]


@pytest.mark.parametrize("old,new", QUANT_MISTAKES)
def test_quantisation_and_eviction_oracle_pins_catch(old, new, monkeypatch):
    from tests import test_kv_quant_oracle_pins as pins
    tests = [pins.test_e4m3_table_matches_the_format, pins.test_e4m3_table_and_rounding_match_torch_float8,
             pins.test_ties_go_to_the_even_code, pins.test_scale_exponent_closed_forms,
             lambda: pins.test_round_trip_error_bounds(0.5), lambda: pins.test_round_trip_error_bounds(300.0),
             pins.test_identity_on_representable_rows, pins.test_dequantised_values_are_exact_in_bfloat16,
             pins.test_eviction_reading]
    assert _pins_fail(pins, "Q", _mutant("kv_quant_oracle", old, new), tests, monkeypatch), (old, new)
