"""Shared plumbing of the GPU parity tests: regenerates on the host exactly the rows a check
needs and builds the oracle's view of a workload.  The expected values always come from oracle/
(never from the HIP path); the library is driven through workloads/driver.py."""
from __future__ import annotations

import numpy as np
import torch

from oracle import kv_quant_oracle as KQ
from oracle import skv_oracle as O
from workloads import gen
from workloads.driver import (alloc_cache, decode_layer, fill_by_append, pool_tensors,  # noqa: F401
                              workspace_for)

TOL = {"f32": 1e-5, "f16": 2e-2, "bf16": 2e-2}   # max-abs error bounds of the parity bar


def oracle_cache(w, lens=None):
    """Full logical float64 + raw-bits cache of a SMALL workload, built by the oracle's append.
    8-bit slots: the values are the dequantised ones, the bits the codes, and `c.exps` is a second
    logical cache (head_dim 1) holding the exponent bytes."""
    lens = w.kv_lens if lens is None else np.asarray(lens)
    kv8 = getattr(w, "kv8", False)
    bits_dtype = np.uint8 if kv8 else np.uint32 if w.dtype == "f32" else np.uint16
    c = O.Cache(w.route, w.batch, w.max_ctx, w.n_kv_heads, w.head_dim, bits_dtype)
    if kv8:
        c.exps = O.Cache(w.route, w.batch, w.max_ctx, w.n_kv_heads, 1, np.uint8)
    n = int(lens.max())
    zeros = np.zeros(w.batch, dtype=np.int64)
    for layer in w.owner_layers:
        k = w.kv_rows("k", layer, 0, w.batch, 0, n, "cpu")
        v = w.kv_rows("v", layer, 0, w.batch, 0, n, "cpu")
        if kv8:
            (kc, ke), (vc, ve) = KQ.quantise_rows(gen.to_f64(k)), KQ.quantise_rows(gen.to_f64(v))
            c.append(layer, KQ.dequantise_rows(kc, ke), KQ.dequantise_rows(vc, ve), kc, vc, zeros, lens)
            c.exps.append(layer, ke[..., None].astype(np.float64), ve[..., None].astype(np.float64),
                          ke[..., None], ve[..., None], zeros, lens)
        else:
            c.append(layer, gen.to_f64(k), gen.to_f64(v), gen.to_bits(k), gen.to_bits(v), zeros, lens)
    return c


def oracle_kv_rows(w, layer, b, kvh, n):
    """float64 K[n][D], V[n][D] that `layer` reads for sequence b, kv head kvh: the rows its
    source layer (per the oracle's routing) produced."""
    src = O.validate_route(w.route)[layer]
    k = w.kv_rows("k", src, b, b + 1, 0, n, "cpu", kv_head=kvh)[0]
    v = w.kv_rows("v", src, b, b + 1, 0, n, "cpu", kv_head=kvh)[0]
    if getattr(w, "kv8", False):    # what an 8-bit slot holds of these rows
        return (KQ.dequantise_rows(*KQ.quantise_rows(gen.to_f64(k))),
                KQ.dequantise_rows(*KQ.quantise_rows(gen.to_f64(v))))
    return gen.to_f64(k), gen.to_f64(v)


def max_abs_err(got: torch.Tensor, expect: np.ndarray) -> float:
    return float(np.max(np.abs(gen.to_f64(got) - expect))) if expect.size else 0.0
