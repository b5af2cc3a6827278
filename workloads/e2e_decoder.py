"""End-to-end harness: a synthetic Qwen3-8B-scale decoder (the paper's inference benchmark,
Sec. 4.3, Tab. 4 / Tab. 5) that serves with the library's depth-shared cache.

The K/V side of every layer is the library: owner layers project and append (skv_kv_project_append),
the other layers of a sharing group skip their K/V projections altogether, all layers attend
through skv_attn_prefill / skv_attn_decode over the slot they are routed to.  Everything else of
the block (norms, query / output / MLP projections, normalisation and rotary encoding of the
queries, the logits) is plain PyTorch: this file is a measurement harness around the path, not part of it.  Weights are
random; tokens are synthetic; decoding is greedy.
"""
from __future__ import annotations

import math

import numpy as np
import torch

import paper_2604_22782_amd as skv


class SyntheticDecoder:
    def __init__(self, n_layers=36, hidden=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, mlp=12288,
                 vocab=151936, group=1, seed=0, dtype=torch.bfloat16, device="cuda", sigma=0.02, qk_norm=False):
        self.L, self.hidden, self.hq, self.hkv, self.d, self.mlp, self.vocab = n_layers, hidden, n_q_heads, n_kv_heads, head_dim, mlp, vocab
        self.route = [group * (l // group) for l in range(n_layers)]       # leader = first layer of each group
        self.dtype, self.device, self.qk_norm = dtype, device, qk_norm
        g = torch.Generator(device=device).manual_seed(seed)
        mk = lambda *shape: (torch.randn(*shape, generator=g, device=device, dtype=torch.float32) * sigma).to(dtype)
        self.w = {"emb": mk(vocab, hidden), "final_norm": torch.ones(hidden, device=device, dtype=dtype)}
        for l in range(n_layers):
            self.w[f"{l}.norm1"] = (1.0 + 0.1 * torch.randn(hidden, generator=g, device=device)).to(dtype)
            self.w[f"{l}.norm2"] = (1.0 + 0.1 * torch.randn(hidden, generator=g, device=device)).to(dtype)
            self.w[f"{l}.wq"] = mk(n_q_heads * head_dim, hidden)
            if qk_norm:                                                    # per-head RMS normalisation of q and k (Qwen3)
                self.w[f"{l}.q_norm"] = (1.0 + 0.1 * torch.randn(head_dim, generator=g, device=device)).to(dtype)
            if self.route[l] == l:                                         # non-owners have no K/V projection
                self.w[f"{l}.wk"] = mk(n_kv_heads * head_dim, hidden)
                self.w[f"{l}.wv"] = mk(n_kv_heads * head_dim, hidden)
                if qk_norm:
                    self.w[f"{l}.k_norm"] = 1.0 + 0.1 * torch.randn(head_dim, generator=g, device=device)
            self.w[f"{l}.wo"] = mk(hidden, n_q_heads * head_dim)
            self.w[f"{l}.wg"] = mk(mlp, hidden)
            self.w[f"{l}.wu"] = mk(mlp, hidden)
            self.w[f"{l}.wd"] = mk(hidden, mlp)
        self.cache = None

    # ---- serving state ---------------------------------------------------------------------------
    def start(self, batch: int, max_ctx: int, rope_base=10000.0):
        self.close()
        self.B, self.max_ctx = batch, max_ctx
        self.cache = skv.skv_cache_alloc(n_layers=self.L, n_q_heads=self.hq, n_kv_heads=self.hkv, head_dim=self.d,
                                         batch=batch, max_ctx=max_ctx, dtype=skv.dtype_code(self.dtype), route=self.route,
                                         block_size=0, n_blocks=0)
        inv = rope_base ** (-torch.arange(self.d // 2, device=self.device, dtype=torch.float64) * 2.0 / self.d)
        ang = torch.arange(max_ctx, device=self.device, dtype=torch.float64)[:, None] * inv[None, :]
        self.cos, self.sin = torch.cos(ang).float().contiguous(), torch.sin(ang).float().contiguous()
        self.lens = torch.zeros(batch, dtype=torch.int32, device=self.device)   # cached positions per sequence
        self.n_host = 0
        self.dec_ws = torch.empty(max(skv.skv_decode_workspace_bytes(self.cache, max_ctx), 4), dtype=torch.uint8, device=self.device)
        self.proj_ws = torch.empty(max(skv.skv_kv_project_workspace_bytes(self.cache, 1, self.hidden), 4), dtype=torch.uint8, device=self.device)

    def close(self):
        if self.cache is not None:
            self.cache.free()
            self.cache = None

    def kv_cache_bytes(self, tokens: int) -> int:
        return skv.skv_cache_bytes(n_layers=self.L, n_q_heads=self.hq, n_kv_heads=self.hkv, head_dim=self.d, batch=self.B,
                                   max_ctx=tokens, dtype=skv.dtype_code(self.dtype), route=self.route, block_size=0, n_blocks=0)

    # ---- the block -------------------------------------------------------------------------------
    @staticmethod
    def _rmsnorm(x, w, eps=1e-6):
        return torch.nn.functional.rms_norm(x, (x.shape[-1],), w, eps)   # one launch

    def _rope_q(self, q, c, s):
        """c, s: [B][new][1][d/2] rows of the tables at the tokens' positions (gathered once per call)."""
        half = self.d // 2
        lo, hi = q[..., :half].float(), q[..., half:].float()
        return torch.cat([lo * c - hi * s, hi * c + lo * s], dim=-1).to(q.dtype)

    def _forward(self, tokens, new: int, hint=None):
        """tokens: int64 [B][new]: the next `new` positions of every sequence.  Returns the logits of
        the last of them, [B][vocab].  hint: host bound on the lengths after this call (default: the
        exact value the host has been counting)."""
        B, w = self.B, self.w
        start = self.lens.clone()
        new_lens = torch.full((B,), new, dtype=torch.int32, device=self.device)
        pos = (start.long()[:, None] + torch.arange(new, device=self.device)[None, :])
        kv_lens = start + new
        n_after = self.n_host + new if hint is None else hint
        x = w["emb"][tokens]
        rope_c, rope_s = self.cos[pos][:, :, None, :], self.sin[pos][:, :, None, :]
        chunk = 16384                                                     # tokens per MLP slice (bounds the temporaries)
        for l in range(self.L):
            h = self._rmsnorm(x, w[f"{l}.norm1"])
            q = (h @ w[f"{l}.wq"].T).view(B, new, self.hq, self.d)
            if self.qk_norm:
                q = self._rmsnorm(q, w[f"{l}.q_norm"])
            q = self._rope_q(q, rope_c, rope_s).contiguous()
            if self.route[l] == l:
                need = skv.skv_kv_project_workspace_bytes(self.cache, new, self.hidden)
                if need > self.proj_ws.numel():                 # prompts only: a captured decode step never gets here
                    self.proj_ws = torch.empty(need, dtype=torch.uint8, device=self.device)
                ws = self.proj_ws
                skv.skv_kv_project_append(self.cache, l, h.contiguous(), w[f"{l}.wk"], w[f"{l}.wv"], self.cos, self.sin,
                                          start, new_lens, new, ws, k_norm_weight=w.get(f"{l}.k_norm"), k_norm_eps=1e-6)
            out = torch.empty_like(q)
            if new == 1:
                skv.skv_attn_decode(self.cache, l, q.view(B, self.hq, self.d), out.view(B, self.hq, self.d), kv_lens,
                                    n_after, 1.0 / math.sqrt(self.d), self.dec_ws)
            else:
                skv.skv_attn_prefill(self.cache, l, q, out, new_lens, kv_lens, new, n_after, 1.0 / math.sqrt(self.d))
            x = x + out.view(B, new, -1) @ w[f"{l}.wo"].T
            h2 = self._rmsnorm(x, w[f"{l}.norm2"]).view(B * new, -1)
            xf = x.view(B * new, -1)
            for i in range(0, B * new, chunk):
                hs = h2[i:i + chunk]
                xf[i:i + chunk] += (torch.nn.functional.silu(hs @ w[f"{l}.wg"].T) * (hs @ w[f"{l}.wu"].T)) @ w[f"{l}.wd"].T
        self.lens.copy_(kv_lens)          # in place: a captured graph keeps reading and advancing this tensor
        self.n_host += new
        return self._rmsnorm(x[:, -1], w["final_norm"]) @ w["emb"].T

    def prefill(self, tokens):
        return self._forward(tokens, tokens.shape[1])

    def decode_step(self, tokens, hint=None):
        return self._forward(tokens.view(self.B, 1), 1, hint)

    # ---- the decode step as one HIP graph ----------------------------------------------------------
    def capture_decode(self):
        """Records one decode step (about 20 launches per layer, each far shorter than the time the
        host needs to issue it) into a HIP graph.  The graph reads its token from a fixed buffer,
        reads and advances the device-side lengths, and sizes its launches for the full capacity."""
        self._tok = torch.zeros(self.B, dtype=torch.int64, device=self.device)
        keep_lens, keep_host = self.lens.clone(), self.n_host
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):                       # warm-up outside the capture (lazy set-up, allocator)
            for _ in range(2):
                self._forward(self._tok.view(self.B, 1), 1, hint=self.max_ctx)
                self.lens.copy_(keep_lens)                  # the rows it wrote are overwritten by the real steps
        torch.cuda.current_stream().wait_stream(side)
        self._graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self._graph):
            self._logits = self._forward(self._tok.view(self.B, 1), 1, hint=self.max_ctx)
        self.n_host = keep_host

    def decode_step_graph(self, tokens):
        self._tok.copy_(tokens.view(self.B))
        self._graph.replay()
        self.n_host += 1
        return self._logits
