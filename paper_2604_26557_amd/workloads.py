"""Seeded synthetic KV workloads: shapes and random draws only.

This module holds no layout, LBA or attention arithmetic.  It names the five
evaluation shapes (sizes taken from 7-8B class models; the paper's own workload
is OPT-6.7B with uniform batches, Sec. V-A "Configuration") and draws the random
inputs both the CPU checker and the GPU library are fed with: K/V/Q values,
per-sequence lengths, a block-id permutation for the paged source, and raw
16-bit patterns for byte-move fuzzing.

Nothing here imports the GPU binding or the checker, so either side can use it.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import List, Optional, Tuple

import torch

F16 = "f16"
BF16 = "bf16"
TOKEN_MAJOR = "token_major"
PER_SEQ = "per_seq"
BHSD = "bhsd"
PAGED = "paged"

MiB = 1 << 20
GiB = 1 << 30


@dataclass(frozen=True)
class KVConfig:
    name: str
    index: int                 # position in the evaluation list; seed = 1000 + index
    n_layers: int
    n_kv_heads: int
    n_q_heads: int
    head_dim: int
    batch: int
    dtype: str                 # F16 | BF16
    sector_bytes: int          # 512 | 4096
    chunk_tokens: int
    depth: int
    extent_mode: str           # TOKEN_MAJOR | PER_SEQ
    layout: str                # BHSD | PAGED
    seq_len: int               # uniform length (ignored when len_range is set)
    len_range: Optional[Tuple[int, int]] = None   # inclusive bounds, ragged batches
    block_tokens: int = 16
    pc_budget_bytes: int = 0   # knob X of the residency planner (Alg. 1)
    lba_start: int = 2048      # first direct tensor's start LBA (user-given, Sec. IV-B "LBA Bind")

    @property
    def seed(self) -> int:
        return 1000 + self.index

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float16 if self.dtype == F16 else torch.bfloat16


# The five evaluation shapes.  X (pc_budget_bytes) is the byte count that makes the
# stated share of layers fit the page-cache path: n_layers_pc * 2 * tensor_bytes.
CONFIGS: List[KVConfig] = [
    KVConfig("tiny", 0, 2, 2, 4, 64, 1, F16, 512, 64, 2, TOKEN_MAJOR, BHSD, 256),
    KVConfig("llama8b_4k", 1, 32, 8, 32, 128, 1, F16, 4096, 256, 3, TOKEN_MAJOR, BHSD, 4096),
    KVConfig("llama8b_32k", 2, 32, 8, 32, 128, 1, BF16, 4096, 1024, 4, TOKEN_MAJOR, BHSD, 32768,
             pc_budget_bytes=16 * 2 * 64 * MiB),
    KVConfig("llama8b_ragged_paged", 3, 32, 8, 32, 128, 8, F16, 4096, 512, 3, PER_SEQ, PAGED, 0,
             len_range=(1024, 8192)),
    KVConfig("gemma7b_mha_8k", 4, 28, 16, 16, 256, 4, BF16, 4096, 256, 3, TOKEN_MAJOR, BHSD, 8192,
             pc_budget_bytes=7 * 2 * 256 * MiB),
]


def config(name_or_index) -> KVConfig:
    if isinstance(name_or_index, int):
        return CONFIGS[name_or_index]
    for c in CONFIGS:
        if c.name == name_or_index:
            return c
    raise KeyError(name_or_index)


def shrink(cfg: KVConfig, **kw) -> KVConfig:
    """Same structure, smaller numbers (for cases the CPU checker finishes in seconds)."""
    return replace(cfg, **kw)


def _gen(seed: int, device: str = "cpu") -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def seq_lens(cfg: KVConfig, seed: Optional[int] = None) -> List[int]:
    """Per-sequence token counts: uniform, or integers drawn from the inclusive range."""
    if cfg.len_range is None:
        return [cfg.seq_len] * cfg.batch
    lo, hi = cfg.len_range
    g = _gen((cfg.seed if seed is None else seed) + 7)
    return [int(v) for v in torch.randint(lo, hi + 1, (cfg.batch,), generator=g)]


def normal_tensor(shape, dtype: torch.dtype, seed: int, device: str = "cpu") -> torch.Tensor:
    """N(0,1) drawn in fp32, rounded to the 16-bit dtype (round to nearest even)."""
    g = _gen(seed, device)
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32).to(dtype)


def raw_u16_tensor(shape, dtype: torch.dtype, seed: int, device: str = "cpu") -> torch.Tensor:
    """Uniform raw 16-bit patterns (NaN/Inf/denormal payloads included), viewed as dtype."""
    g = _gen(seed, device)
    bits = torch.randint(-32768, 32768, shape, generator=g, device=device, dtype=torch.int16)
    return bits.view(dtype)


def layer_seed(cfg: KVConfig, layer: int, kind: int, seed: Optional[int] = None) -> int:
    return (cfg.seed if seed is None else seed) * 100003 + layer * 2 + kind


def bhsd_layer(cfg: KVConfig, layer: int, kind: int, device: str = "cpu",
               seed: Optional[int] = None, raw: bool = False,
               s_alloc: Optional[int] = None) -> torch.Tensor:
    """One K (kind 0) or V (kind 1) tensor of one layer, [B, H, S_alloc, D] contiguous."""
    s = max(seq_lens(cfg, seed)) if s_alloc is None else s_alloc
    shape = (cfg.batch, cfg.n_kv_heads, s, cfg.head_dim)
    f = raw_u16_tensor if raw else normal_tensor
    return f(shape, cfg.torch_dtype, layer_seed(cfg, layer, kind, seed), device)


def query(cfg: KVConfig, layer: int, device: str = "cpu", seed: Optional[int] = None) -> torch.Tensor:
    """Decode-step query of one layer, [B, H_q, D]."""
    s = (cfg.seed if seed is None else seed) * 100003 + 50000 + layer
    return normal_tensor((cfg.batch, cfg.n_q_heads, cfg.head_dim), cfg.torch_dtype, s, device)


def paged_blocks_per_seq(cfg: KVConfig, lens: List[int]) -> List[int]:
    bt = cfg.block_tokens
    return [(n + bt - 1) // bt for n in lens]


def block_table(cfg: KVConfig, lens: List[int], seed: Optional[int] = None,
                identity: bool = False) -> Tuple[torch.Tensor, int]:
    """Block table [B, max_blocks] int32 and pool size.

    The pool has exactly sum_b ceil(len_b / block_tokens) blocks; sequence b owns a run of
    entries of a seeded random permutation of all block ids (identity order on request).
    Unused table entries hold -1.
    """
    per = paged_blocks_per_seq(cfg, lens)
    n_pool = sum(per)
    if identity:
        perm = torch.arange(n_pool, dtype=torch.int64)
    else:
        perm = torch.randperm(n_pool, generator=_gen((cfg.seed if seed is None else seed) + 13))
    table = torch.full((cfg.batch, max(per) if per else 0), -1, dtype=torch.int32)
    base = 0
    for b, n in enumerate(per):
        table[b, :n] = perm[base:base + n].to(torch.int32)
        base += n
    return table, n_pool


def paged_layer(cfg: KVConfig, layer: int, kind: int, n_pool: int, device: str = "cpu",
                seed: Optional[int] = None, raw: bool = False) -> torch.Tensor:
    """One K or V block pool of one layer, [n_pool, H, block_tokens, D] contiguous."""
    shape = (n_pool, cfg.n_kv_heads, cfg.block_tokens, cfg.head_dim)
    f = raw_u16_tensor if raw else normal_tensor
    return f(shape, cfg.torch_dtype, layer_seed(cfg, layer, kind, seed), device)
