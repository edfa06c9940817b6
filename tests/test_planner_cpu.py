"""Host-side logic of the native library against the CPU checker (no GPU needed): the extent
planner (Alg. 1, Eq. 3-6), token-range translation (Alg. 2), chunk commands (Eq. 7-11), error
codes, and that the C ABI exports every symbol the header declares."""
import os
import re

import numpy as np
import pytest

from oracle import kv_oracle as o
from paper_2604_26557_amd import binding as kv
from paper_2604_26557_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _plans(cfg, lens=None):
    lens = W.seq_lens(cfg) if lens is None else lens
    per_seq = cfg.extent_mode == W.PER_SEQ
    p = kv.kv_layout_plan(cfg.n_layers, cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim, lens,
                          kv.KV_F16 if cfg.dtype == W.F16 else kv.KV_BF16, cfg.sector_bytes, cfg.chunk_tokens,
                          kv.KV_PER_SEQ if per_seq else kv.KV_TOKEN_MAJOR, cfg.lba_start, kv.KV_UNBOUNDED,
                          cfg.pc_budget_bytes, kv.KV_UNBOUNDED)
    ref = o.layout_plan(cfg.n_layers, cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim, lens, 2, cfg.sector_bytes,
                        per_seq, cfg.pc_budget_bytes, cfg.lba_start)
    return p, ref, lens


def test_header_symbols_exported():
    text = open(os.path.join(ROOT, "include", "kvblade.h")).read()
    declared = set(re.findall(r"\b(kv_[a-z_0-9]+)\s*\(", text))
    declared -= {n for n in declared if n.endswith("_t")}
    assert declared == set(kv.EXPORTS)
    lib = kv.lib()
    for name in declared:
        assert hasattr(lib, name)
    assert lib.kv_abi_version() == 4
    assert lib.kv_abi_sizeof(7) == kv.C.sizeof(kv.kv_pipe_stats_t) and lib.kv_abi_sizeof(99) == 0


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 on its own, with every struct usable by value."""
    import subprocess
    src = tmp_path / "hdr.c"
    src.write_text('#include "kvblade.h"\n'
                   'int main(void) { kv_plan_desc_t d; kv_view_t v; kv_pipe_opts_t o; kv_pipe_stats_t s; kv_chunk_trace_t t;\n'
                   '  (void)d; (void)v; (void)o; (void)s; (void)t; return kv_abi_version() < 0; }\n')
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                           "-c", str(src), "-o", str(tmp_path / "hdr.o")])


@pytest.mark.parametrize("idx", range(5))
def test_plan_matches_oracle_all_configs(idx):
    cfg = W.CONFIGS[idx]
    p, ref, lens = _plans(cfg)
    info = p.info
    assert info.n_pagecache_layers == ref.n1
    assert info.row_bytes == ref.row_bytes
    assert info.tensor_blocks == ref.n_blocks_tensor
    assert info.tensor_payload_bytes == ref.payload_bytes
    assert info.region_bytes_needed == (ref.region_bytes if ref.n1 < ref.L else 0)
    assert info.pageable_bytes_needed == ref.pageable_bytes
    for layer in range(cfg.n_layers):
        for kind in (0, 1):
            n = 2 * layer + kind
            e = kv.kv_plan_tensor(p, layer, kind)
            assert (e.path, e.lba_start, e.n_blocks, e.file_off, e.bytes) == \
                (int(ref.path[n]), int(ref.lba_start[n]), int(ref.n_blocks[n]), int(ref.file_off[n]), ref.payload_bytes)
    for b in range(len(lens)):
        assert kv.kv_plan_seq_base(p, b) == int(ref.seq_base[b])


def _expected_translate(ref, n, b, tok0, ntok):
    rc, slba, req = o.token_range(ref, n, b, tok0, ntok)
    if rc != o.OK:
        return rc, 0, 0
    cap = ref.cap[b]
    sec = ref.lba_size
    if tok0 + ntok == cap:
        req = -(-req // sec) * sec          # tail of the extent: rounded up, pad is zeros
    elif req % sec:
        return o.EALIGN, 0, 0               # a range may only end inside a sector at the tail
    return rc, slba, req


@pytest.mark.parametrize("idx", [0, 1, 3])
def test_translate_and_chunks_match_oracle(idx):
    cfg = W.CONFIGS[idx]
    if idx == 3:
        cfg = W.shrink(cfg, n_layers=3, len_range=(100, 700))
    p, ref, lens = _plans(cfg)
    rng = np.random.default_rng(idx)
    nseq = len(lens) if ref.per_seq else 1
    for layer in sorted({0, cfg.n_layers - 1}):
        for kind in (0, 1):
            n = 2 * layer + kind
            for b in range(nseq):
                cap = lens[b]
                cases = [(0, cap), (0, 1), (cap - 1, 1), (0, cfg.chunk_tokens), (cfg.chunk_tokens, cap - cfg.chunk_tokens)]
                cases += [(int(rng.integers(0, cap)), int(rng.integers(1, cap + 1))) for _ in range(40)]
                cases = [c for c in cases if c[1] >= 1]
                for tok0, ntok in cases:
                    want = _expected_translate(ref, n, b, tok0, ntok)
                    try:
                        got = (0,) + kv.kv_plan_translate(p, layer, kind, b, tok0, ntok)
                    except kv.KVError as e:
                        got = (e.code, 0, 0)
                    assert got == want, (layer, kind, b, tok0, ntok)
                # Eq. 7-11 over the whole (sub-)extent
                rc, slba, req = o.token_range(ref, n, b, 0, cap)
                want_cmds = o.chunk_cmds(slba, req, cfg.chunk_tokens * ref.row_bytes, ref.lba_size)
                got_cmds = kv.kv_plan_chunk_cmds(p, layer, kind, b)
                assert [(c.slba, c.nlb, c.buf_off) for c in got_cmds] == want_cmds
                assert [c.tok0 for c in got_cmds] == [i * cfg.chunk_tokens for i in range(len(got_cmds))]
                assert sum(c.ntok for c in got_cmds) == cap


def test_chunk_cmds_other_chunk_sizes():
    cfg = W.CONFIGS[1]
    p, ref, lens = _plans(cfg)
    for C in (2, 64, 1000, 4096, 8192):   # rows are 2 KiB, sectors 4 KiB: C must be even
        rc, slba, req = o.token_range(ref, 5, 0, 0, lens[0])
        want = o.chunk_cmds(slba, req, C * ref.row_bytes, ref.lba_size)
        got = kv.kv_plan_chunk_cmds(p, 2, 1, 0, C)
        assert [(c.slba, c.nlb, c.buf_off) for c in got] == want
    with pytest.raises(kv.KVError) as e:
        kv.kv_plan_chunk_cmds(p, 2, 1, 0, 3)
    assert e.value.code == kv.KV_EALIGN


@pytest.mark.parametrize("idx", [0, 1, 3])
def test_range_cmds_with_transfer_limit_match_oracle(idx):
    """Alg. 2 on a token range, then Eq. 7-11 with the chunk size drawn from a transfer-size limit."""
    cfg = W.CONFIGS[idx]
    if idx == 3:
        cfg = W.shrink(cfg, n_layers=3, len_range=(100, 700))
    p, ref, lens = _plans(cfg)
    sec, rb = ref.lba_size, ref.row_bytes
    rng = np.random.default_rng(100 + idx)
    nseq = len(lens) if ref.per_seq else 1
    n_ok = 0
    for layer, kind in ((0, 0), (cfg.n_layers - 1, 1)):
        n = 2 * layer + kind
        for b in range(nseq):
            cap = lens[b]
            ranges = [(0, cap), (cap - 1, 1)] + [(int(rng.integers(0, cap)), int(rng.integers(1, cap + 1))) for _ in range(30)]
            for tok0, ntok in ranges:
                want = _expected_translate(ref, n, b, tok0, ntok)
                for mdts in (0, sec, sec + 1, 3 * sec - 1, 5 * rb + 3, 256 * 1024, 1 << 21):
                    if want[0] != o.OK:
                        with pytest.raises(kv.KVError) as e:
                            kv.kv_plan_range_cmds(p, layer, kind, b, tok0, ntok, mdts)
                        assert e.value.code == want[0]
                        continue
                    chunk = o.chunk_size(mdts, sec) if mdts else cfg.chunk_tokens * rb
                    want_cmds = o.chunk_cmds(want[1], want[2], chunk, sec)
                    got = kv.kv_plan_range_cmds(p, layer, kind, b, tok0, ntok, mdts)
                    assert [(c.slba, c.nlb, c.buf_off) for c in got] == want_cmds
                    # rows named by each command: those its payload bytes touch
                    for c in got:
                        lo, hi = c.buf_off, min(c.buf_off + (c.nlb + 1) * sec, ntok * rb)
                        rows = set(range(tok0 + lo // rb, tok0 + -(-hi // rb))) if hi > lo else set()
                        assert set(range(c.tok0, c.tok0 + c.ntok)) == rows
                    n_ok += 1
    assert n_ok > 50
    with pytest.raises(kv.KVError) as e:
        kv.kv_plan_range_cmds(p, 0, 0, 0, 0, lens[0], sec - 1)   # limit below one sector
    assert e.value.code == kv.KV_EINVAL


def test_range_cmds_paper_devices(paper_sizes):
    """The two devices' MDTS and LBA sizes on a 128 MiB request: 512 and 64 commands (Sec. V-A)."""
    for dev, n_max, n_cmds in (("ssd_a", 64, 512), ("ssd_b", 4096, 64)):
        lba, mdts = paper_sizes[dev + "_lba"], paper_sizes[dev + "_mdts"]
        rows = paper_sizes["prefill_write_bytes"] // (32 * 32 * 128 * 2)   # B=32, H=32, D=128, 16-bit: 512 rows
        p = kv.kv_layout_plan(1, 32, 32, 128, [rows] * 32, kv.KV_F16, lba, 2, kv.KV_TOKEN_MAJOR, 2048,
                              kv.KV_UNBOUNDED, 0, kv.KV_UNBOUNDED)
        cmds = kv.kv_plan_range_cmds(p, 0, 0, 0, 0, rows, mdts)
        assert len(cmds) == n_cmds and all(c.nlb == n_max - 1 for c in cmds)
        assert [c.slba for c in cmds] == [2048 + i * n_max for i in range(n_cmds)]


def test_random_plans_match_oracle():
    """Seeded random shapes, sector sizes, extent modes, start LBAs and budgets: every entry of the map, the
    residency split, the sub-extent bases and the whole-extent commands against the checker."""
    rng = np.random.default_rng(77)
    n_checked = 0
    for _ in range(150):
        L, H = int(rng.integers(1, 9)), int(rng.integers(1, 9))
        G, D = int(rng.choice([1, 2, 4, 8])), int(rng.choice([64, 128, 256]))
        B, sec = int(rng.integers(1, 6)), int(rng.choice([512, 4096]))
        per_seq = bool(rng.integers(0, 2))
        lens = [int(x) for x in rng.integers(1, 700, size=B)] if per_seq else [int(rng.integers(1, 700))] * B
        row = (H if per_seq else B * H) * D * 2
        unit = sec // int(np.gcd(sec, row))
        C = unit * int(rng.integers(1, 9))
        lba0 = int(rng.integers(0, 5000))
        nb = o.tensor_blocks(per_seq, lens, H, D, 2, sec)[0]
        X = int(rng.integers(0, 2 * (L + 1))) * nb * sec + int(rng.integers(0, sec))
        p = kv.kv_layout_plan(L, H, H * G, D, lens, kv.KV_F16, sec, C, kv.KV_PER_SEQ if per_seq else kv.KV_TOKEN_MAJOR,
                              lba0, kv.KV_UNBOUNDED, X, kv.KV_UNBOUNDED)
        ref = o.layout_plan(L, H, H * G, D, lens, 2, sec, per_seq, X, lba0)
        info = p.info
        assert info.n_pagecache_layers == ref.n1 == min(X // (2 * nb * sec), L)      # Alg. 1
        assert info.tensor_blocks == nb and info.row_bytes == row
        assert info.pageable_bytes_needed == ref.pageable_bytes
        for n in range(2 * L):
            e = kv.kv_plan_tensor(p, n // 2, n % 2)
            assert (e.path, e.lba_start, e.n_blocks, e.file_off) == \
                (int(ref.path[n]), int(ref.lba_start[n]), int(ref.n_blocks[n]), int(ref.file_off[n]))
        nseq = B if per_seq else 1
        for b in range(nseq):
            assert kv.kv_plan_seq_base(p, b) == int(ref.seq_base[b])
            n = int(rng.integers(0, 2 * L))
            rc, slba, req = o.token_range(ref, n, b, 0, lens[b])
            assert rc == o.OK
            want = o.chunk_cmds(slba, req, C * row, sec)
            got = kv.kv_plan_chunk_cmds(p, n // 2, n % 2, b)
            assert [(c.slba, c.nlb, c.buf_off) for c in got] == want
            n_checked += len(got)
        p.close()
    assert n_checked > 300


def test_pagecache_path_addresses_are_arena_sectors():
    cfg = W.CONFIGS[2]
    p, ref, lens = _plans(cfg)
    e = kv.kv_plan_tensor(p, 3, 1)
    assert e.path == kv.KV_PATH_PAGECACHE and e.file_off == 7 * 64 * W.MiB
    slba, req = kv.kv_plan_translate(p, 3, 1, 0, 1024, 1024)
    assert slba * 4096 == e.file_off + 1024 * 2048 and req == 2 * W.MiB
    e = kv.kv_plan_tensor(p, 16, 0)
    assert e.path == kv.KV_PATH_DIRECT and e.lba_start == 2048   # numbering skips page-cache tensors


def test_error_codes():
    def plan(**kw):
        a = dict(n_layers=2, n_kv_heads=2, n_q_heads=4, head_dim=64, seq_cap=[256], dtype=kv.KV_F16,
                 sector_bytes=512, chunk_tokens=64)
        a.update(kw)
        return kv.kv_layout_plan(**a)

    def code(fn):
        with pytest.raises(kv.KVError) as e:
            fn()
        return e.value.code

    assert code(lambda: plan(sector_bytes=1024)) == kv.KV_EINVAL
    assert code(lambda: plan(dtype=7)) == kv.KV_EINVAL
    assert code(lambda: plan(n_q_heads=5)) == kv.KV_EINVAL
    assert code(lambda: plan(head_dim=12)) == kv.KV_EINVAL
    assert code(lambda: plan(seq_cap=[256, 255])) == kv.KV_EINVAL               # token-major needs a uniform batch
    assert code(lambda: plan(n_kv_heads=1, head_dim=64, sector_bytes=4096, chunk_tokens=3)) == kv.KV_EALIGN
    assert code(lambda: plan(lba_start=100, region_blocks=100 + 4 * 128 - 1)) == kv.KV_ENOSPC
    plan(lba_start=100, region_blocks=100 + 4 * 128).close()
    assert code(lambda: plan(pc_budget_bytes=2 * 65536, pageable_bytes=2 * 65536 - 1)) == kv.KV_ENOSPC
    p = plan()
    assert code(lambda: kv.kv_plan_tensor(p, 2, 0)) == kv.KV_ERANGE
    assert code(lambda: kv.kv_plan_tensor(p, 0, 2)) == kv.KV_EINVAL
    assert code(lambda: kv.kv_plan_translate(p, 0, 0, 0, 1, 2)) == kv.KV_EALIGN  # 256 B rows, 512 B sectors
    assert code(lambda: kv.kv_plan_translate(p, 0, 0, 0, 0, 3)) == kv.KV_EALIGN  # ends inside a sector, not at tail
    assert code(lambda: kv.kv_plan_translate(p, 0, 0, 0, 250, 8)) == kv.KV_ERANGE
    assert code(lambda: kv.kv_plan_translate(p, 0, 0, 0, 0, 0)) == kv.KV_EINVAL
    assert code(lambda: kv.kv_plan_translate(p, 0, 0, 1, 0, 2)) == kv.KV_ERANGE  # no sequence 1 in token-major
    assert kv.kv_plan_translate(p, 0, 0, 0, 254, 2) == (2048 * 0 + 254 * 256 // 512, 512)
    assert kv.lib().kv_strerror(kv.KV_EALIGN).decode().startswith("offset")


def test_odd_tail_rounds_up():
    """8 KV heads, D=128, batch 1 under 4 KiB sectors: 2 KiB rows, an odd capacity pads half a sector."""
    p = kv.kv_layout_plan(1, 8, 32, 128, [4097], kv.KV_F16, 4096, 256, kv.KV_TOKEN_MAJOR, 2048)
    assert p.info.tensor_blocks == 2049
    slba, req = kv.kv_plan_translate(p, 0, 1, 0, 4096, 1)
    assert slba == 2048 + 2049 + 2048 and req == 4096
    cmds = kv.kv_plan_chunk_cmds(p, 0, 0, 0)
    assert len(cmds) == 17 and cmds[-1].nlb == 0 and cmds[-1].ntok == 1


def test_budget_matches_oracle():
    rng = np.random.default_rng(3)
    for _ in range(200):
        a, m, s = (int(x) for x in rng.integers(0, 20 * 10**9, 3))
        t, pin = int(rng.integers(0, 5)), int(rng.integers(0, 10**9))
        assert kv.kv_budget(a, m, s, t, pin) == o.budget(a, m, s, t, pin)
    assert kv.kv_budget(8 * 10**9, 11 * 10**9, 2 * 10**9, 2, 128 * W.MiB) == (8 * 10**9, 8 * 10**9 - 256 * W.MiB)
    with pytest.raises(kv.KVError):
        kv.kv_budget(1, 1, 0, -1, 1)


def test_trim_matches_oracle_and_touches_only_extents():
    cfg = W.shrink(W.CONFIGS[2], n_layers=4, seq_len=100, chunk_tokens=2, pc_budget_bytes=2 * 2 * 100 * 2048)
    p, ref, lens = _plans(cfg)
    region = np.full(ref.region_bytes + 4096, 0x5C, dtype=np.uint8)     # one guard sector behind the last extent
    arena = np.full(ref.pageable_bytes + 4096, 0x5C, dtype=np.uint8)
    want_r, want_a = region.copy(), arena.copy()
    for layer in (1, 2):                                                 # layer 1: page-cache path, layer 2: direct
        for kind in (0, 1):
            n = 2 * layer + kind
            o.trim(want_r if ref.path[n] == 0 else want_a, ref.ext_byte_off(n), int(ref.n_blocks[n]), ref.lba_size)
    assert kv.kv_plan_trim(p, 1, 3, region, arena) == (4, 4 * ref.n_blocks_tensor)
    assert np.array_equal(region, want_r) and np.array_equal(arena, want_a)
    assert (region[:2048 * 4096] == 0x5C).all() and (region[-4096:] == 0x5C).all()
    with pytest.raises(kv.KVError) as e:
        kv.kv_plan_trim(p, 0, 4, region[:ref.region_bytes - 1], arena)
    assert e.value.code == kv.KV_ENOSPC


def test_adaptive_selection_matches_oracle():
    rng = np.random.default_rng(11)
    for trial in range(50):
        a = kv.kv_adapt_init()
        thr = {0: [0.0, 0.0], 1: [0.0, 0.0]}                   # [group][order] as measured
        for it in range(1, 8):                                  # 1-based decode iterations
            orders = [kv.kv_adapt_order(a, g) for g in (0, 1)]
            for g in (0, 1):
                assert orders[g] == o.adapt_order(it, thr[g][kv.KV_ORDER_INTRA], thr[g][kv.KV_ORDER_CROSS]), (trial, it, g)
            st = kv.kv_pipe_stats_t()
            st.bytes_pagecache, st.bytes_direct = 2 * 10**9, 3 * 10**9
            secs = [float(rng.uniform(0.03, 0.06)), float(rng.uniform(0.04, 0.08))] if trial else [0.05, 0.05]
            st.group_seconds[0], st.group_seconds[1] = secs
            if it in (2, 3):                                    # only these two iterations are measured
                thr[0][orders[0]] = 2.0 / secs[0]
                thr[1][orders[1]] = 3.0 / secs[1]
            kv.kv_adapt_update(a, st)
        assert a.iteration == 7


def _fake_root(tmp_path, meminfo, cgroup_line=None, files=None):
    (tmp_path / "proc" / "self").mkdir(parents=True)
    (tmp_path / "proc" / "meminfo").write_text(meminfo)
    if cgroup_line is not None:
        (tmp_path / "proc" / "self" / "cgroup").write_text(cgroup_line + "\n")
    for rel, text in (files or {}).items():
        f = tmp_path / rel
        f.parent.mkdir(parents=True, exist_ok=True)
        f.write_text(text)
    return str(tmp_path)


MEMINFO = "MemTotal:       16000000 kB\nMemFree:         1000000 kB\nMemAvailable:    9000000 kB\nAnonPages:       2000000 kB\nShmem:            500000 kB\n"


def test_budget_sample_system_and_cgroup_limits(tmp_path):
    """Eq. 1's inputs under system and cgroup limits, from fixture files, then through Eq. 1-2."""
    KiB = 1024
    # no cgroup limit: the machine's memory and its anon + shmem
    root = _fake_root(tmp_path / "a", MEMINFO, "0::/", {"sys/fs/cgroup/memory.max": "max\n"})
    assert kv.kv_budget_sample(root) == (9000000 * KiB, 16000000 * KiB, 2500000 * KiB)
    # cgroup v2 limit of 4 GiB in a nested group, its own anon + shmem (bytes)
    root = _fake_root(tmp_path / "b", MEMINFO, "0::/serve/llm", {
        "sys/fs/cgroup/serve/llm/memory.max": str(4 << 30) + "\n",
        "sys/fs/cgroup/serve/llm/memory.stat": "anon 1000000000\nfile 5\nshmem 24000000\n"})
    got = kv.kv_budget_sample(root)
    assert got == (9000000 * KiB, 4 << 30, 1024000000)
    # Eq. 1-2 on the sample: M* = min(M_avail, M_max - M_anon+shmem), B_pc = max(0, M* - N_threads M_pin)
    m_star, b_pc = kv.kv_budget(*got, 2, 128 << 20)
    assert (m_star, b_pc) == o.budget(*got, 2, 128 << 20)
    assert m_star == (4 << 30) - 1024000000 and b_pc == m_star - (256 << 20)
    # cgroup v1 (memory controller line), rss + shmem
    root = _fake_root(tmp_path / "c", MEMINFO, "4:cpu,memory:/box", {
        "sys/fs/cgroup/memory/box/memory.limit_in_bytes": "2147483648\n",
        "sys/fs/cgroup/memory/box/memory.stat": "cache 1\nrss 300000000\nshmem 1000000\n"})
    assert kv.kv_budget_sample(root) == (9000000 * KiB, 2147483648, 301000000)
    # a limit above the machine's memory is no limit
    root = _fake_root(tmp_path / "d", MEMINFO, "0::/", {"sys/fs/cgroup/memory.max": str(1 << 50) + "\n"})
    assert kv.kv_budget_sample(root)[1:] == (16000000 * KiB, 2500000 * KiB)
    # unreadable or incomplete /proc/meminfo
    with pytest.raises(kv.KVError) as e:
        kv.kv_budget_sample(str(tmp_path / "nowhere"))
    assert e.value.code == kv.KV_EINVAL
    root = _fake_root(tmp_path / "e", "MemTotal: 5 kB\n")
    with pytest.raises(kv.KVError):
        kv.kv_budget_sample(root)
    # the real host: plausible figures
    a, m, s_ = kv.kv_budget_sample()
    assert 0 < a <= m * 2 and m > 0 and s_ >= 0


def test_decode_attention_split_planning():
    """Host arithmetic of the split choice (no GPU): the splits of every sequence tile its tokens exactly, split
    lengths are multiples of the kernel's quantum (of one step of the kernel, and at least the quantum, where a ragged
    batch gets per-sequence lengths), a ragged batch is cut so that the longest split is close to the mean load of
    the workgroup budget, and a given split count is honoured."""
    import random
    rnd = random.Random(7)
    for D, q, step in ((64, 128, 32), (128, 64, 16), (256, 64, 16)):
        for trial in range(40):
            B = rnd.choice([1, 2, 3, 8, 17, 64, 70])
            H = rnd.choice([1, 2, 8])
            G = rnd.choice([1, 2, 4, 8])
            uniform = rnd.random() < 0.3
            n0 = rnd.randint(0, 9000)
            lens = [n0] * B if uniform else [rnd.choice([0, 1, rnd.randint(1, 9000)]) for _ in range(B)]
            plan = kv.kv_layout_plan(1, H, H * G, D, [max(max(lens), 1)] * B, kv.KV_F16, 512, 8)
            for n_splits in (0, 1, 5):
                ns, first, tokens = kv.kv_decode_attn_splits(plan, lens, n_splits)
                assert 1 <= ns <= 1024 and first[0] == 0
                if n_splits:
                    assert ns == n_splits
                per_seq = n_splits == 0 and len(set(lens)) > 1 and B <= 64
                for b, n in enumerate(lens):
                    nb, st = first[b + 1] - first[b], tokens[b]
                    assert st % (step if per_seq else q) == 0 and st >= q
                    assert nb <= ns and nb == -(-n // st)              # exactly the splits that hold tokens
                    assert nb * st >= n and (nb == 0 or (nb - 1) * st < n)
                ragged = len(set(lens)) > 1
                if n_splits == 0 and ragged and B <= 64 and sum(lens) > 0:
                    groups = (H * G) // (4 if G % 4 == 0 else 2 if G % 2 == 0 else 1)
                    budget = max(sum(1 for n in lens if n > 0), 256 // groups)   # 256 workgroups when no GPU is present
                    assert first[B] <= budget
                    nbs = [first[b + 1] - first[b] for b in range(B)]
                    longest = max(min(tokens[b], lens[b]) for b in range(B))
                    assert longest >= sum(lens) / budget - q               # cannot beat the mean load
                    # minimax: taking a split away from any sequence would make that sequence's splits at least as
                    # long as the longest split now (up to the rounding of split lengths to the quantum)
                    for b in range(B):
                        if nbs[b] >= 2:
                            assert longest <= lens[b] / (nbs[b] - 1) + q
    with pytest.raises(kv.KVError):
        kv.kv_decode_attn_splits(plan, [-1] * len(lens), 0)
