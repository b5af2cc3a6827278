"""Drives the C-ABI library with a Workload: cache allocation, filling through skv_kv_append,
workspace, raw pool readback.  No oracle and no attention arithmetic in here."""
from __future__ import annotations

import numpy as np
import torch

import paper_2604_22782_amd as skv

def alloc_cache(w, device="cuda", caller_pools=False):
    desc = dict(n_layers=w.n_layers, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads,
                head_dim=w.head_dim, batch=w.batch, max_ctx=w.max_ctx,
                dtype=skv.dtype_code(w.torch_dtype, getattr(w, "kv8", False)), route=w.route,
                block_size=w.block_size, n_blocks=w.n_blocks)
    pools = None
    if caller_pools:
        each, sc = skv.skv_cache_pool_bytes(**desc)
        pools = (torch.zeros(each, dtype=torch.uint8, device=device),
                 torch.zeros(each, dtype=torch.uint8, device=device))
        desc.update(k_pool=pools[0], v_pool=pools[1], pool_bytes=each)
        if sc:
            pools += (torch.full((sc,), 127, dtype=torch.uint8, device=device),)
            desc.update(scale_pool=pools[2], scale_pool_bytes=sc)
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
    if getattr(w, "kv8", False):   # codes of K, codes of V, exponent bytes [slot][row][kv head][K, V]
        sp, sb = skv.skv_cache_scale_info(cache)
        host = torch.empty(sb, dtype=torch.uint8)
        rc = hip.hipMemcpy(ctypes.c_void_p(host.data_ptr()), ctypes.c_void_p(sp), ctypes.c_size_t(sb), 2)
        assert rc == 0, rc
        # An 8-bit slot is head-major inside groups of R consecutive rows ([group][kv head][row in group][d],
        # R = 128, or the block size where blocks are smaller; a contiguous slot holds whole groups per
        # sequence): bring the three pools back to row order.
        R = min(w.block_size, 128) if w.block_size else 128
        seq_rows = -(-w.max_ctx // R) * R
        phys = w.n_blocks * w.block_size if w.block_size else w.batch * seq_rows

        def row_order(t, width):
            x = t.view(n_slots, phys // R, w.n_kv_heads, R, width).permute(0, 1, 3, 2, 4).reshape(n_slots, phys, w.n_kv_heads, width)
            if not w.block_size:
                x = x.view(n_slots, w.batch, seq_rows, w.n_kv_heads, width)[:, :, : w.max_ctx]
            return x.reshape(n_slots, rows, w.n_kv_heads, width).contiguous()
        return [row_order(o, w.head_dim) for o in outs] + [row_order(host, 2)]
    view = {2: torch.int16, 4: torch.int32}[w.elem_bytes]
    return [o.view(view).view(shape) for o in outs]


def fill_by_append(cache, w, lens=None, chunk_tokens=1 << 19, device="cuda"):
    """Append positions [0, lens[b]) of every owner layer, generated on the device in chunks of
    positions; sequences that already ended are neither generated nor appended."""
    lens = w.kv_lens if lens is None else np.asarray(lens, dtype=np.int32)
    max_len = int(lens.max())
    d_lens = torch.from_numpy(lens.astype(np.int32)).to(device)
    step = max(1, min(max_len, chunk_tokens // w.batch))
    shape = (w.batch, step, w.n_kv_heads, w.head_dim)
    kbuf = torch.zeros(shape, dtype=w.torch_dtype, device=device)
    vbuf = torch.zeros(shape, dtype=w.torch_dtype, device=device)
    for layer in w.owner_layers:
        for p0 in range(0, max_len, step):
            p1 = min(max_len, p0 + step)
            active = np.nonzero(lens > p0)[0]
            if len(active) == w.batch:
                kbuf[:, : p1 - p0] = w.kv_rows("k", layer, 0, w.batch, p0, p1, device)
                vbuf[:, : p1 - p0] = w.kv_rows("v", layer, 0, w.batch, p0, p1, device)
            else:
                idx = torch.from_numpy(active).to(device)
                kbuf[idx, : p1 - p0] = w.kv_rows("k", layer, 0, 0, p0, p1, device, seqs=active)
                vbuf[idx, : p1 - p0] = w.kv_rows("v", layer, 0, 0, p0, p1, device, seqs=active)
            start = torch.full((w.batch,), p0, dtype=torch.int32, device=device)
            new = (d_lens - p0).clamp(0, p1 - p0).to(torch.int32)
            skv.skv_kv_append(cache, layer, kbuf, vbuf, start, new, step)
    torch.cuda.synchronize()


def decode_layer(cache, w, layer, q, kv_lens_dev, max_kv_len, workspace):
    out = torch.empty_like(q)
    skv.skv_attn_decode(cache, layer, q, out, kv_lens_dev, max_kv_len, w.scale, workspace)
    return out


def workspace_for(cache, max_kv_len, device="cuda"):
    n = skv.skv_decode_workspace_bytes(cache, max_kv_len)
    return torch.empty(max(n, 4) // 4 + 1, dtype=torch.float32, device=device)
