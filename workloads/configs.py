"""The five synthetic workloads (shapes, routes, lengths, block tables) and their seeded tensors.

Shapes follow the model families the paper evaluates (Llama-2-7B, Llama-3-8B and Qwen3-8B
style attention); values are synthetic and stand in for the paper's QA / benchmark inputs, which
an attention kernel never looks at beyond shape, length and scale.  Holds no attention
arithmetic: route tables here are plain data handed to the library and to the oracle alike.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np
import torch

from . import gen

STREAM_K, STREAM_V, STREAM_Q_DECODE, STREAM_Q_PREFILL = 1, 2, 3, 4

DTYPES = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


@dataclasses.dataclass
class Workload:
    name: str
    dtype: str                 # "f32" | "f16" | "bf16"
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    batch: int
    route: list                # route[l] = source layer of layer l (0-based)
    kv_lens: np.ndarray        # int32[batch]: cached positions per sequence, new token included
    sigma_q: float
    sigma_kv: float
    seed: int
    block_size: int = 0        # 0 = contiguous cache, else tokens per physical block
    block_table: np.ndarray | None = None   # int32[batch][max_blocks_per_seq]
    n_blocks: int = 0
    max_ctx: int = 0           # capacity per sequence (contiguous) / index stride of positions
    kv8: bool = False          # the cache slots hold 8-bit codes with a power-of-two scale per (position, kv head)

    def __post_init__(self):
        self.kv_lens = np.asarray(self.kv_lens, dtype=np.int32)
        if self.max_ctx == 0:
            self.max_ctx = int(self.kv_lens.max())
        self.scale = 1.0 / math.sqrt(self.head_dim)

    # ---- derived ---------------------------------------------------------------------------
    @property
    def torch_dtype(self):
        return DTYPES[self.dtype]

    @property
    def elem_bytes(self):
        return 4 if self.dtype == "f32" else 2

    @property
    def owner_layers(self):
        return [l for l, r in enumerate(self.route) if r == l]

    @property
    def group(self):
        return self.n_q_heads // self.n_kv_heads

    def decode_bytes_per_layer(self) -> int:
        """Algorithmic bytes of one decode launch: K and V rows of every cached position of
        every sequence once, plus Q in and O out."""
        row = self.n_kv_heads * (self.head_dim + 1) if self.kv8 else self.n_kv_heads * self.head_dim * self.elem_bytes
        qo = 2 * self.batch * self.n_q_heads * self.head_dim * self.elem_bytes
        return int(self.kv_lens.astype(np.int64).sum()) * 2 * row + qo

    def prefill_flops_per_layer(self, q_lens=None) -> int:
        """4 * Hq * D * (number of visible (query, key) pairs); masked pairs are not counted."""
        q_lens = self.kv_lens if q_lens is None else np.asarray(q_lens)
        pairs = 0
        for nq, n in zip(q_lens.tolist(), self.kv_lens.tolist()):
            pairs += nq * (n - nq) + nq * (nq + 1) // 2
        return 4 * self.n_q_heads * self.head_dim * pairs

    # ---- seeded tensors --------------------------------------------------------------------
    def kv_rows(self, which: str, layer: int, b0: int, b1: int, p0: int, p1: int, device,
                kv_head: int | None = None, seqs=None) -> torch.Tensor:
        """K or V rows that layer `layer` produces for sequences [b0,b1) (or the explicit list
        `seqs`), positions [p0,p1): tensor [n_seq][p1-p0][kv_heads][head_dim], or
        [n_seq][p1-p0][head_dim] for one kv head."""
        stream = STREAM_K if which == "k" else STREAM_V
        hd = self.n_kv_heads * self.head_dim
        if seqs is None:
            b = torch.arange(b0, b1, dtype=torch.int64, device=device)[:, None, None]
        else:
            b = torch.as_tensor(seqs, dtype=torch.int64, device=device)[:, None, None]
        p = torch.arange(p0, p1, dtype=torch.int64, device=device)[None, :, None]
        if kv_head is None:
            r = torch.arange(hd, dtype=torch.int64, device=device)[None, None, :]
        else:
            r = kv_head * self.head_dim + torch.arange(self.head_dim, dtype=torch.int64, device=device)[None, None, :]
        idx = ((layer * self.batch + b) * self.max_ctx + p) * hd + r
        x = gen.normal(idx, self.seed, stream, self.sigma_kv, self.torch_dtype)
        if kv_head is not None:
            return x
        return x.view(b.shape[0], p1 - p0, self.n_kv_heads, self.head_dim)

    def q_decode(self, layer: int, device) -> torch.Tensor:
        """[batch][q_heads][head_dim] query of the newest token at layer `layer`."""
        n = self.batch * self.n_q_heads * self.head_dim
        idx = layer * n + torch.arange(n, dtype=torch.int64, device=device)
        x = gen.normal(idx, self.seed, STREAM_Q_DECODE, self.sigma_q, self.torch_dtype)
        return x.view(self.batch, self.n_q_heads, self.head_dim)

    def q_prefill(self, layer: int, b0: int, b1: int, s0: int, s1: int, device) -> torch.Tensor:
        """[b1-b0][s1-s0][q_heads][head_dim] queries of rows [s0,s1) of sequences [b0,b1)."""
        hd = self.n_q_heads * self.head_dim
        b = torch.arange(b0, b1, dtype=torch.int64, device=device)[:, None, None]
        s = torch.arange(s0, s1, dtype=torch.int64, device=device)[None, :, None]
        r = torch.arange(hd, dtype=torch.int64, device=device)[None, None, :]
        idx = ((layer * self.batch + b) * self.max_ctx + s) * hd + r
        x = gen.normal(idx, self.seed, STREAM_Q_PREFILL, self.sigma_q, self.torch_dtype)
        return x.view(b1 - b0, s1 - s0, self.n_q_heads, self.head_dim)


def _paged(kv_lens: np.ndarray, block_size: int, rng: np.random.Generator):
    """Seeded random-permutation block table: physical ids 0..n_blocks-1 shuffled, then dealt to
    the sequences in order.  Unused trailing entries hold 0 (a valid id, never dereferenced)."""
    need = (kv_lens.astype(np.int64) + block_size - 1) // block_size
    n_blocks = int(need.sum())
    perm = rng.permutation(n_blocks).astype(np.int32)
    table = np.zeros((len(kv_lens), int(need.max())), dtype=np.int32)
    at = 0
    for b, n in enumerate(need.tolist()):
        table[b, :n] = perm[at:at + n]
        at += n
    return table, n_blocks


def grouped_route(n_layers: int, g: int) -> list:
    """Leader scheme of the paper's inference benchmark: every g consecutive layers read the
    cache of the first layer of their group."""
    return [l - (l % g) for l in range(n_layers)]


def tiny_f32() -> Workload:
    """Config 1: 4 layers, route [0,0,2,2], 4 q heads / 2 kv heads, d 64, batch 2, context 128
    prefilled + 1 decoded token."""
    return Workload("tiny_routed_gqa_f32", "f32", 4, 4, 2, 64, 2, [0, 0, 2, 2],
                    np.array([129, 129]), 1.0, 1.0, seed=1001, max_ctx=129)


def llama3_decode(batch: int = 64, ctx: int = 4096, n_layers: int = 32) -> Workload:
    """Config 2: Llama-3-8B-shaped decode, bf16, pairs of layers share a slot."""
    return Workload("llama3_8b_decode_bf16", "bf16", n_layers, 32, 8, 128, batch,
                    grouped_route(n_layers, 2), np.full(batch, ctx), 1.0, 0.5, seed=1002)


def llama3_prefill(batch: int = 4, seq: int = 8192, n_layers: int = 32) -> Workload:
    """Config 3: Llama-3-8B-shaped causal prefill, bf16, every 4th layer owns a slot."""
    return Workload("llama3_8b_prefill_bf16", "bf16", n_layers, 32, 8, 128, batch,
                    grouped_route(n_layers, 4), np.full(batch, seq), 1.0, 1.0, seed=1003)


def qwen3_paged_decode(batch: int = 128, n_layers: int = 36, lo: int = 512, hi: int = 32768,
                       median: int = 4096) -> Workload:
    """Config 4: Qwen3-8B-shaped decode, bf16, lognormal context lengths, random strategy S
    pushed through the nearest-preceding-owner rule, paged cache with 16-token blocks."""
    rng = np.random.default_rng(1004)
    lens = np.clip(np.rint(rng.lognormal(math.log(median), 1.0, size=batch)), lo, hi).astype(np.int32)
    route = [0]
    for l in range(1, n_layers):
        route.append(l if rng.random() < 0.5 else route[l - 1])
    table, n_blocks = _paged(lens, 16, rng)
    return Workload("qwen3_8b_paged_decode_bf16", "bf16", n_layers, 32, 8, 128, batch, route, lens,
                    1.0, 0.5, seed=1004, block_size=16, block_table=table, n_blocks=n_blocks,
                    max_ctx=int(table.shape[1]) * 16)


def llama2_mha_decode(batch: int = 32, ctx: int = 16384, n_layers: int = 32) -> Workload:
    """Config 5: Llama-2-7B-shaped MHA decode, fp16, one slot per 8 layers."""
    return Workload("llama2_7b_mha_decode_f16", "f16", n_layers, 32, 32, 128, batch,
                    grouped_route(n_layers, 8), np.full(batch, ctx), 1.0, 0.5, seed=1005)
