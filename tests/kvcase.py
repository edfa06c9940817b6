"""Test scaffolding: one synthetic KV workload held three ways -- device tensors + native view + native
plan for the GPU path, CPU copies of the same bits + the checker's plan for the CPU side."""
from __future__ import annotations

from typing import List, Optional

import numpy as np
import torch

from oracle import kv_oracle as o
from paper_2604_26557_amd import binding as kv
from paper_2604_26557_amd import workloads as W


def native_plan(cfg: W.KVConfig, lens, region_blocks=kv.KV_UNBOUNDED, pageable_bytes=kv.KV_UNBOUNDED) -> kv.Plan:
    return kv.kv_layout_plan(cfg.n_layers, cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim, lens,
                             kv.KV_F16 if cfg.dtype == W.F16 else kv.KV_BF16, cfg.sector_bytes, cfg.chunk_tokens,
                             kv.KV_PER_SEQ if cfg.extent_mode == W.PER_SEQ else kv.KV_TOKEN_MAJOR,
                             cfg.lba_start, region_blocks, cfg.pc_budget_bytes, pageable_bytes)


def oracle_plan(cfg: W.KVConfig, lens) -> o.Plan:
    return o.layout_plan(cfg.n_layers, cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim, lens, 2, cfg.sector_bytes,
                         cfg.extent_mode == W.PER_SEQ, cfg.pc_budget_bytes, cfg.lba_start)


class Case:
    """cfg on `device`; the CPU copies (`k_cpu`, `v_cpu`) are taken from the device tensors so both
    sides see the same bits whichever generator produced them."""

    def __init__(self, cfg: W.KVConfig, device: str = "cuda", raw: bool = False, gen_device: Optional[str] = None,
                 keep_cpu: bool = True, s_extra: int = 0, lens: Optional[List[int]] = None, cap_extra: int = 0):
        self.cfg = cfg
        self.device = device
        self.lens = W.seq_lens(cfg) if lens is None else lens
        # extents (and the source buffers) may hold cap_extra more tokens than are valid (decode appends)
        self.caps = [n + cap_extra for n in self.lens]
        self.plan = native_plan(cfg, self.caps)
        self.ref = oracle_plan(cfg, self.caps)
        gd = device if gen_device is None else gen_device
        L = cfg.n_layers
        self.paged = cfg.layout == W.PAGED
        if self.paged:
            table, n_pool = W.block_table(cfg, self.caps)
            self.table_cpu = table
            self.table_dev = table.to(device)
            self.n_pool = n_pool
            mk = lambda l, k: W.paged_layer(cfg, l, k, n_pool, gd, raw=raw).to(device)
        else:
            s_alloc = max(self.caps) + s_extra
            mk = lambda l, k: W.bhsd_layer(cfg, l, k, gd, raw=raw, s_alloc=s_alloc).to(device)
        self.k = [mk(l, 0) for l in range(L)]
        self.v = [mk(l, 1) for l in range(L)]
        self.k_cpu = [t.cpu() for t in self.k] if keep_cpu else None
        self.v_cpu = [t.cpu() for t in self.v] if keep_cpu else None
        self.lens_dev = torch.tensor(self.lens, dtype=torch.int32, device=device)
        self.view = self.make_view(self.k, self.v)

    # ---- native side
    def make_view(self, k, v, lens: Optional[List[int]] = None) -> kv.View:
        lens_dev = self.lens_dev if lens is None else torch.tensor(lens, dtype=torch.int32, device=self.device)
        lens = self.lens if lens is None else lens
        if self.paged:
            return kv.paged_view(k, v, self.table_dev, lens, lens_dev)
        return kv.bhsd_view(k, v, lens, lens_dev)

    def blank_like_source(self, fill: int = 0x7E7E):
        """Fresh device tensors shaped like the source, filled with a 16-bit pattern."""
        def f(t):
            return torch.full(t.shape, fill, dtype=torch.int16, device=t.device).view(t.dtype)
        return [f(t) for t in self.k], [f(t) for t in self.v]

    # ---- checker side
    def source(self, t_cpu: torch.Tensor) -> o.Source:
        cfg = self.cfg
        if self.paged:
            return o.Source(H=cfg.n_kv_heads, D=cfg.head_dim, paged=True, block_table=self.table_cpu.numpy(),
                            block_tokens=cfg.block_tokens)
        st = t_cpu.stride()
        return o.Source(H=cfg.n_kv_heads, D=cfg.head_dim, stride_b=st[0], stride_h=st[1], stride_s=st[2])

    def tensor_cpu(self, layer: int, kind: int) -> torch.Tensor:
        return (self.k_cpu if kind == 0 else self.v_cpu)[layer]

    def expected_extent(self, layer: int, kind: int, t_cpu: Optional[torch.Tensor] = None,
                        lens: Optional[List[int]] = None) -> np.ndarray:
        """The whole extent image of one tensor (payload + zero pad) by the checker."""
        r = self.ref
        t = self.tensor_cpu(layer, kind) if t_cpu is None else t_cpu
        ext = np.full(r.n_blocks_tensor * r.lba_size, 0xEE, dtype=np.uint8)
        o.pack(self.source(t), o.u16(t), r.per_seq, self.lens if lens is None else lens, r.seq_base,
               r.n_blocks_tensor, r.lba_size, ext)
        return ext

    def expected_host(self, layers=None, fill: int = 0xC3, lens: Optional[List[int]] = None):
        """(region, arena) images after offloading `layers` (default all) into buffers pre-filled with `fill`."""
        r = self.ref
        region = np.full(max(r.region_bytes, 1), fill, dtype=np.uint8)
        arena = np.full(max(r.pageable_bytes, 1), fill, dtype=np.uint8)
        for layer in (range(r.L) if layers is None else layers):
            for kind in (0, 1):
                n = 2 * layer + kind
                buf = region if r.path[n] == 0 else arena
                off = r.ext_byte_off(n)
                buf[off:off + r.n_blocks_tensor * r.lba_size] = self.expected_extent(layer, kind, lens=lens)
        return region, arena

    def expected_attention(self, layer: int, q_cpu: torch.Tensor) -> np.ndarray:
        cfg = self.cfg
        K, V = self.k_cpu[layer], self.v_cpu[layer]
        return o.attention(self.source(K), o.u16(K), o.u16(V), o.u16(q_cpu), cfg.dtype == W.BF16, self.lens,
                           cfg.n_q_heads)


def bits(t: torch.Tensor) -> np.ndarray:
    """Raw 16-bit (or byte) content of a tensor on any device, as NumPy."""
    t = t.detach().cpu().contiguous()
    if t.dtype in (torch.float16, torch.bfloat16):
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def pinned_bytes(n: int, fill: int) -> torch.Tensor:
    t = torch.empty(max(n, 1), dtype=torch.uint8, pin_memory=True)
    t.fill_(fill)
    return t
