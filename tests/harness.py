"""Shared plumbing of the GPU parity tests: builds caches through the C ABI, fills them with the
seeded workload tensors via skv_kv_append, and regenerates on the host exactly the rows a check
needs.  The expected values always come from oracle/ (never from the HIP path)."""
from __future__ import annotations

import numpy as np
import torch

import paper_2604_22782_amd as skv
from oracle import skv_oracle as O
from workloads import gen

TOL = {"f32": 1e-5, "f16": 2e-2, "bf16": 2e-2}   # max-abs error bounds of the parity bar


def alloc_cache(w, device="cuda", caller_pools=False):
    desc = dict(n_layers=w.n_layers, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads,
                head_dim=w.head_dim, batch=w.batch, max_ctx=w.max_ctx,
                dtype=skv.dtype_code(w.torch_dtype), route=w.route,
                block_size=w.block_size, n_blocks=w.n_blocks)
    pools = None
    if caller_pools:
        each = skv.skv_cache_bytes(**desc) // 2
        pools = (torch.zeros(each, dtype=torch.uint8, device=device),
                 torch.zeros(each, dtype=torch.uint8, device=device))
        desc.update(k_pool=pools[0], v_pool=pools[1], pool_bytes=each)
    cache = skv.skv_cache_alloc(**desc)
    if w.block_size:
        table = torch.from_numpy(np.ascontiguousarray(w.block_table)).to(device)
        skv.skv_cache_set_block_table(cache, table)
    return cache, pools


def pool_tensors(cache, w):
    """K and V pools as torch views (copied out through a raw-pointer memcpy)."""
    import ctypes
    n_slots, kp, vp, each = skv.skv_cache_info(cache)
    hip = ctypes.CDLL("libamdhip64.so.7")   # the runtime torch already loaded (same soname)
    outs = []
    for p in (kp, vp):
        host = torch.empty(each, dtype=torch.uint8)
        torch.cuda.synchronize()
        rc = hip.hipMemcpy(ctypes.c_void_p(host.data_ptr()), ctypes.c_void_p(p), ctypes.c_size_t(each), 2)
        assert rc == 0, rc
        outs.append(host)
    rows = w.n_blocks * w.block_size if w.block_size else w.batch * w.max_ctx
    shape = (n_slots, rows, w.n_kv_heads, w.head_dim)
    view = {2: torch.int16, 4: torch.int32}[w.elem_bytes]
    return [o.view(view).view(shape) for o in outs]


def fill_by_append(cache, w, lens=None, chunk_tokens=1 << 22, device="cuda"):
    """Append positions [0, lens[b]) of every owner layer, generated on the device in chunks."""
    lens = w.kv_lens if lens is None else np.asarray(lens, dtype=np.int32)
    max_len = int(lens.max())
    d_lens = torch.from_numpy(lens.astype(np.int32)).to(device)
    step = max(1, min(max_len, chunk_tokens // w.batch))
    for layer in w.owner_layers:
        for p0 in range(0, max_len, step):
            p1 = min(max_len, p0 + step)
            k = w.kv_rows("k", layer, 0, w.batch, p0, p1, device)
            v = w.kv_rows("v", layer, 0, w.batch, p0, p1, device)
            start = torch.full((w.batch,), p0, dtype=torch.int32, device=device)
            new = (d_lens - p0).clamp(0, p1 - p0).to(torch.int32)
            skv.skv_kv_append(cache, layer, k, v, start, new, p1 - p0)
    torch.cuda.synchronize()


def oracle_cache(w, lens=None):
    """Full logical float64 + raw-bits cache of a SMALL workload, built by the oracle's append."""
    lens = w.kv_lens if lens is None else np.asarray(lens)
    bits_dtype = np.uint32 if w.dtype == "f32" else np.uint16
    c = O.Cache(w.route, w.batch, w.max_ctx, w.n_kv_heads, w.head_dim, bits_dtype)
    n = int(lens.max())
    for layer in w.owner_layers:
        k = w.kv_rows("k", layer, 0, w.batch, 0, n, "cpu")
        v = w.kv_rows("v", layer, 0, w.batch, 0, n, "cpu")
        c.append(layer, gen.to_f64(k), gen.to_f64(v), gen.to_bits(k), gen.to_bits(v),
                 np.zeros(w.batch, dtype=np.int64), lens)
    return c


def oracle_kv_rows(w, layer, b, kvh, n):
    """float64 K[n][D], V[n][D] that `layer` reads for sequence b, kv head kvh: the rows its
    source layer (per the oracle's routing) produced."""
    src = O.validate_route(w.route)[layer]
    k = w.kv_rows("k", src, b, b + 1, 0, n, "cpu")[0, :, kvh]
    v = w.kv_rows("v", src, b, b + 1, 0, n, "cpu")[0, :, kvh]
    return gen.to_f64(k), gen.to_f64(v)


def decode_layer(cache, w, layer, q, kv_lens_dev, max_kv_len, workspace):
    out = torch.empty_like(q)
    skv.skv_attn_decode(cache, layer, q, out, kv_lens_dev, max_kv_len, w.scale, workspace)
    return out


def workspace_for(cache, max_kv_len, device="cuda"):
    n = skv.skv_decode_workspace_bytes(cache, max_kv_len)
    return torch.empty(max(n, 4) // 4 + 1, dtype=torch.float32, device=device)


def max_abs_err(got: torch.Tensor, expect: np.ndarray) -> float:
    return float(np.max(np.abs(gen.to_f64(got) - expect))) if expect.size else 0.0
