"""Pins for the CPU checker's planner half: Alg. 1, Eq. 3-6, Alg. 2, Eq. 7-11.

Everything here is checked against numbers the paper prints (tests/golden/paper_sizes.txt),
closed forms, the three bind invariants, or brute-force enumeration on tiny shapes.
"""
import itertools

import numpy as np
import pytest

from oracle import kv_oracle as o

KiB, MiB, GiB = 1 << 10, 1 << 20, 1 << 30


# ------------------------------------------------------------------ Alg. 1
def test_residency_closed_forms():
    L, S = 32, 64 * MiB
    assert o.residency(0, S, L)[0] == 0                      # X = 0: everything direct (Table 3, NVMe-direct-Only)
    assert o.residency(2 * L * S, S, L)[0] == L              # X covers all layers
    assert o.residency(10**15, S, L)[0] == L                 # clamp at L
    assert o.residency(2 * GiB, S, L)[0] == 16               # 32K-context shape: half the layers
    assert o.residency(7 * 2 * 256 * MiB, 256 * MiB, 28)[0] == 7
    assert o.residency(2 * S - 1, S, L)[0] == 0              # floor, a pair must fit whole
    assert o.residency(2 * S, S, L)[0] == 1
    assert o.residency(3 * S, S, L)[0] == 1                  # K alone does not count: pairs only


def test_residency_prefix_and_monotone():
    L, S = 12, 1000
    prev = -1
    for X in range(0, 2 * L * S + 3 * S, 333):
        n1, x = o.residency(X, S, L)
        assert n1 == min(X // (2 * S), L)
        assert list(x) == [1] * n1 + [0] * (L - n1)          # first n1 layers, nothing else
        assert n1 >= prev
        prev = n1


# ------------------------------------------------------------------ Table 2 / Sec. III sizes
@pytest.mark.parametrize("key,H,D", [("opt_1p3b_unit_per_batch", 32, 64),
                                     ("opt_6p7b_unit_per_batch", 32, 128),
                                     ("opt_13b_unit_per_batch", 40, 128)])
def test_min_io_unit_table2(paper_sizes, key, H, D):
    for B in (1, 2, 3, 8, 32):
        rc, _, req = o.translate(0, (1, B * H, D), (600, B * H, D), (0, 0, 0), 2, 512)
        assert rc == o.OK and req == paper_sizes[key] * B


def test_even_batch_rule_opt13b():
    """10 KiB x B is a 4 KiB multiple exactly when B is even (Sec. IV-B precondition); with 512 B
    LBAs every B is aligned."""
    H, D = 40, 128
    for B in range(1, 9):
        d = (600, B * H, D)
        ok4k = [o.translate(0, (1, B * H, D), d, (t, 0, 0), 2, 4096)[0] == o.OK for t in range(8)]
        ok512 = [o.translate(0, (1, B * H, D), d, (t, 0, 0), 2, 512)[0] == o.OK for t in range(8)]
        assert all(ok512)
        assert all(ok4k) == (B % 2 == 0)
        if B % 2:
            assert ok4k == [t % 2 == 0 for t in range(8)]      # odd B: only even token offsets align


def test_request_sizes_opt6p7b(paper_sizes):
    B, H, D = 32, 32, 128
    tgt = (543, B * H, D)
    rc, slba, req = o.translate(2048, (1, B * H, D), tgt, (512, 0, 0), 2, 4096)
    assert rc == o.OK and req == paper_sizes["decode_write_bytes"]
    assert slba == 2048 + 512 * 64                            # 256 KiB rows = 64 blocks per token
    rc, _, req = o.translate(2048, (512, B * H, D), tgt, (0, 0, 0), 2, 4096)
    assert req == paper_sizes["prefill_write_bytes"] == paper_sizes["decode_read_lo_bytes"]
    rc, _, req = o.translate(2048, (543, B * H, D), tgt, (0, 0, 0), 2, 4096)
    assert rc == o.OK and req // MiB == paper_sizes["decode_read_hi_mb_floor"]


def test_kv_totals(paper_sizes):
    for key, rows in (("kv_total_lo_centi_gb", 511), ("kv_total_hi_centi_gb", 543)):
        nb, _, pay = o.tensor_blocks(False, [rows] * 32, 32, 128, 2, 4096)
        assert nb * 4096 == pay                                # precondition holds: no padding
        assert (64 * pay) // 10**7 == paper_sizes[key]


# ------------------------------------------------------------------ Eq. 3-6
def test_bind_example_chain(paper_sizes):
    L = 4
    nb, _, pay = o.tensor_blocks(False, [543] * 32, 32, 128, 2, 4096)
    x = np.zeros(L, dtype=np.int32)
    path, lba, nbs, off = o.bind(L, x, nb, 4096, paper_sizes["example_lba_start"])
    assert lba[0] == 2048
    assert nb == pay // 4096 == 543 * 64                      # Eq. 5 with exact division
    for n in range(1, 2 * L):
        assert lba[n] == lba[n - 1] + nbs[n - 1]               # Eq. 6
    assert list(lba[:3]) == [2048, 2048 + 34752, 2048 + 2 * 34752]


def _check_invariants(p: o.Plan):
    direct = [n for n in range(2 * p.L) if p.path[n] == 0]
    pc = [n for n in range(2 * p.L) if p.path[n] == 1]
    # contiguity + disjointness in tensor order (K then V, ascending layer)
    if direct:
        assert p.lba_start[direct[0]] == p.lba_start_first
    for a, b in zip(direct, direct[1:]):
        assert int(p.lba_start[b]) == int(p.lba_start[a]) + int(p.n_blocks[a])
    if pc:
        assert p.file_off[pc[0]] == 0
    for a, b in zip(pc, pc[1:]):
        assert int(p.file_off[b]) == int(p.file_off[a]) + int(p.n_blocks[a]) * p.lba_size
    for n in pc:
        assert int(p.file_off[n]) % p.lba_size == 0           # alignment
    # brute-force disjointness
    spans = sorted((int(p.lba_start[n]), int(p.lba_start[n]) + int(p.n_blocks[n])) for n in direct)
    for (a0, a1), (b0, b1) in zip(spans, spans[1:]):
        assert a1 <= b0
    # K and V of a layer share a path; the page-cache layers are a prefix
    for layer in range(p.L):
        assert p.path[2 * layer] == p.path[2 * layer + 1] == p.x[layer]
    assert list(p.x) == [1] * p.n1 + [0] * (p.L - p.n1)


def test_bind_invariants_and_totals():
    # (L, H, Hq, D, cap, sec, per_seq, X) -> direct blocks, n1
    cases = [
        ((2, 2, 4, 64, [256], 512, False, 0), 512, 0),
        ((32, 8, 32, 128, [4096], 4096, False, 0), 131072, 0),
        ((32, 8, 32, 128, [32768], 4096, False, 2 * GiB), 524288, 16),
        ((28, 16, 16, 256, [8192] * 4, 4096, False, 7 * 2 * 256 * MiB), 2752512, 7),
    ]
    for (L, H, Hq, D, cap, sec, ps, X), blocks, n1 in cases:
        p = o.layout_plan(L, H, Hq, D, cap, 2, sec, ps, X, 2048)
        _check_invariants(p)
        assert p.direct_blocks == blocks and p.n1 == n1
        assert p.region_bytes == (2048 + blocks) * sec


def test_per_seq_blocks_and_bases():
    caps = [1025, 8192, 1024, 3000]
    H, D, sec = 8, 128, 4096
    nb, base, pay = o.tensor_blocks(True, caps, H, D, 2, sec)
    want = [-(-c * H * D * 2 // sec) for c in caps]           # ceil per sequence
    assert nb == sum(want)
    assert list(base) == [0, want[0], want[0] + want[1], want[0] + want[1] + want[2]]
    assert pay == sum(caps) * H * D * 2
    assert want[0] == 513                                      # 1025 rows of 2 KiB: one pad half-block
    # batch 1: the two extent modes coincide
    assert o.tensor_blocks(True, [777], H, D, 2, sec)[0] == o.tensor_blocks(False, [777], H, D, 2, sec)[0]
    with pytest.raises(ValueError):
        o.tensor_blocks(False, [5, 6], H, D, 2, sec)           # token-major needs a uniform batch


def test_padding_reading_ceil():
    """Token row 2 KiB under 4 KiB sectors (batch 1, 8 KV heads): odd row counts pad half a block."""
    nb, _, pay = o.tensor_blocks(False, [4097], 8, 128, 2, 4096)
    assert pay == 4097 * 2048 and nb == 2049 and nb * 4096 - pay == 2048


# ------------------------------------------------------------------ Alg. 2, brute force
def _sectors_touched(d, e, lba, tok0, ntok):
    """Enumerate every element of rows [tok0, tok0+ntok) of a row-major (d0,d1,d2) array."""
    s = set()
    for i in range(tok0, tok0 + ntok):
        for j in range(d[1]):
            for k in range(d[2]):
                byte = ((i * d[1] + j) * d[2] + k) * e
                s.add(byte // lba)
                s.add((byte + e - 1) // lba)
    return s


@pytest.mark.parametrize("d,lba", [((12, 4, 32), 512), ((9, 2, 64), 512), ((8, 16, 128), 4096), ((10, 3, 64), 128)])
def test_translate_brute_force(d, lba):
    e, lba_start = 2, 77
    row = d[1] * d[2] * e
    for tok0, ntok in itertools.product(range(d[0]), range(1, d[0] + 1)):
        if tok0 + ntok > d[0]:
            continue
        rc, slba, req = o.translate(lba_start, (ntok, d[1], d[2]), d, (tok0, 0, 0), e, lba)
        if (tok0 * row) % lba:
            assert rc == o.EALIGN
            continue
        assert rc == o.OK and req == ntok * row
        if req % lba:
            continue                                           # a shared tail sector is the caller's problem
        want = {lba_start + x for x in _sectors_touched(d, e, lba, tok0, ntok)}
        assert want == set(range(slba, slba + req // lba))


def test_translate_inner_offsets_and_errors():
    d = (16, 8, 128)
    # (i0, j0, k0) general offsets: Alg. 2 row-major formula, checked against np.ravel_multi_index
    for idx in [(0, 0, 0), (3, 4, 0), (15, 7, 0), (2, 0, 64)]:
        rc, slba, req = o.translate(5, (1, 1, 64), d, idx, 2, 128)
        want = int(np.ravel_multi_index(idx, d)) * 2
        assert rc == o.OK and slba == 5 + want // 128 and req == 128
    assert o.translate(0, (1, 8, 128), d, (16, 0, 0), 2, 512)[0] == o.ERANGE
    assert o.translate(0, (2, 8, 128), d, (15, 0, 0), 2, 512)[0] == o.ERANGE
    assert o.translate(0, (1, 8, 128), d, (0, 0, 1), 2, 512)[0] == o.EALIGN
    assert o.translate(0, (1, 8, 128), d, (-1, 0, 0), 2, 512)[0] == o.EINVAL


# ------------------------------------------------------------------ Eq. 7-11
def test_mdts_arithmetic(paper_sizes):
    req = paper_sizes["prefill_write_bytes"]
    for dev, n_max, n_cmds in (("ssd_a", 64, 512), ("ssd_b", 4096, 64)):
        lba, mdts = paper_sizes[dev + "_lba"], paper_sizes[dev + "_mdts"]
        chunk = o.chunk_size(mdts, lba)                        # Eq. 7 align_down
        assert chunk == n_max * lba == mdts                    # both devices' MDTS are LBA multiples
        cmds = o.chunk_cmds(2048, req, chunk, lba)
        assert len(cmds) == n_cmds
        assert all(nlb == n_max - 1 for _, nlb, _ in cmds)     # 0-based block count
        assert [c[0] for c in cmds] == [2048 + i * n_max for i in range(n_cmds)]
        assert [c[2] for c in cmds] == [i * chunk for i in range(n_cmds)]
        assert sum(nlb + 1 for _, nlb, _ in cmds) * lba == req


def test_chunk_size_aligns_down():
    # Eq. 7 on sizes that are not LBA multiples: the largest multiple not above MDTS
    assert o.chunk_size(1000, 512) == 512
    assert o.chunk_size(511, 512) == 0
    assert o.chunk_size(4096 * 7 + 4095, 4096) == 4096 * 7
    for mdts in range(0, 5000, 37):
        c = o.chunk_size(mdts, 512)
        assert c % 512 == 0 and c <= mdts < c + 512


def test_chunk_cmds_ragged_tail():
    lba, chunk = 4096, 16 * 4096
    for req in (1, 4096, 4097, chunk - 1, chunk, chunk + 1, 5 * chunk + 3 * 4096 + 17):
        cmds = o.chunk_cmds(100, req, chunk, lba)
        blocks = -(-req // lba)
        assert len(cmds) == -(-req // chunk)                   # Eq. 8
        assert sum(n + 1 for _, n, _ in cmds) == blocks        # every block moved once
        for i, (slba, nlb, off) in enumerate(cmds):
            assert slba == 100 + i * 16 and off == i * chunk
            assert nlb + 1 == min(16, blocks - i * 16)         # Eq. 10 with n_remains
    with pytest.raises(ValueError):
        o.chunk_cmds(0, 100, 1000, 512)                        # chunk not a multiple of the LBA size


def test_token_range_helper_matches_alg2():
    p = o.layout_plan(4, 2, 4, 64, [300, 100, 257], 2, 512, True, 0, 2048)
    for n in (0, 3, 7):
        for b in range(3):
            rc, slba, req = o.token_range(p, n, b, 4, 8)
            assert rc == o.OK
            assert slba == int(p.lba_start[n]) + int(p.seq_base[b]) + 4 * 256 // 512
            assert req == 8 * 256


def test_token_range_on_the_pagecache_path_is_the_arena_sector():
    """A page-cache-path tensor has no LBA: Alg. 2 is fed the sector index of its arena offset, so the closed form
    is file_off / sector + seq_base + tok0 * row_bytes / sector, with the tensors before it fixing file_off."""
    sec, H, D, caps = 512, 2, 64, [300, 100, 257]
    row = H * D * 2                                            # 256 bytes per token row of a sequence
    blocks = [-(-c * row // sec) for c in caps]                # per-sequence sub-extents, each padded to a sector
    tensor_bytes = sum(blocks) * sec
    X = 2 * 2 * tensor_bytes                                   # room for exactly two layers on the page-cache path
    p = o.layout_plan(4, H, 4, D, caps, 2, sec, True, X, 2048)
    assert p.n1 == 2 and list(p.path) == [1, 1, 1, 1, 0, 0, 0, 0]
    for n in range(4):                                         # arena tensors, in id order from offset 0
        assert int(p.file_off[n]) == n * tensor_bytes and int(p.lba_start[n]) == 0
        for b in range(3):
            rc, sector, req = o.token_range(p, n, b, 4, 8)
            assert rc == o.OK and req == 8 * row
            assert sector == n * tensor_bytes // sec + sum(blocks[:b]) + 4 * row // sec
    for n in range(4, 8):                                      # direct tensors: LBAs from the user's start, arena skipped
        rc, slba, _ = o.token_range(p, n, 1, 2, 2)
        assert rc == o.OK and slba == 2048 + (n - 4) * sum(blocks) + blocks[0] + 2 * row // sec
    # token-major twin: one extent (S_cap, B*H, D)
    q = o.layout_plan(2, 2, 4, 64, [64, 64], 2, 512, False, 2 * 64 * 2 * 2 * 64 * 2, 7)
    assert q.n1 == 1
    assert o.token_range(q, 1, 0, 3, 2) == (o.OK, 64 * 512 // 512 + 3, 2 * 512)     # second arena tensor, row = 512 B
    assert o.token_range(q, 2, 0, 3, 2) == (o.OK, 7 + 3, 2 * 512)                   # first direct tensor


def test_plan_byte_helpers_closed_forms():
    """row_bytes, region_bytes, pageable_bytes and ext_byte_off against sizes worked out by hand."""
    p = o.layout_plan(3, 2, 4, 64, [100, 100], 2, 512, False, 2 * 51200, 10)        # row = 2*2*64*2 = 512 B
    assert p.row_bytes == 512 and p.n_blocks_tensor == 100 and p.n1 == 1
    assert p.pageable_bytes == 2 * 51200                       # K and V of layer 0
    assert p.region_bytes == (10 + 4 * 100) * 512              # hole below LBA 10, then four direct tensors
    assert [p.ext_byte_off(n) for n in range(6)] == [0, 51200, 10 * 512, 110 * 512, 210 * 512, 310 * 512]
    assert p.direct_blocks == 400
    r = o.layout_plan(1, 2, 4, 64, [3, 5], 2, 512, True, 0, 0)                      # per sequence: row = 256 B
    assert r.row_bytes == 256 and list(r.seq_base) == [0, 2] and r.n_blocks_tensor == 2 + 3


# ------------------------------------------------------------------ Eq. 1-2
def test_budget_closed_forms():
    GB = 10**9
    pin = 128 * MiB                                            # one K or V tensor at the paper's shape
    assert o.budget(8 * GB, 11 * GB, 2 * GB, 2, pin) == (8 * GB, 8 * GB - 2 * pin)       # M_avail binds
    assert o.budget(12 * GB, 11 * GB, 2 * GB, 2, pin) == (9 * GB, 9 * GB - 2 * pin)      # the cgroup limit binds
    assert o.budget(1 * GB, 11 * GB, 2 * GB, 2, GB) == (1 * GB, 0)                        # clamp at zero
    assert o.budget(5 * GB, 2 * GB, 3 * GB, 2, pin) == (-1 * GB, 0)                       # over-committed cgroup
    assert o.budget(4 * GB, 4 * GB, 0, 0, pin) == (4 * GB, 4 * GB)                        # no copy threads
    for t in range(5):                                                                    # each thread costs M_pin
        assert o.budget(4 * GB, 9 * GB, 0, t, pin)[1] == 4 * GB - t * pin


def test_trim_zeroes_exactly_the_extent():
    buf = np.full(10 * 512, 0xAB, dtype=np.uint8)
    o.trim(buf, 3 * 512, 4, 512)
    assert (buf[:3 * 512] == 0xAB).all() and not buf[3 * 512:7 * 512].any() and (buf[7 * 512:] == 0xAB).all()


# ------------------------------------------------------------------ Sec. IV-C strategy selection
def test_adapt_order_schedule():
    INTRA, CROSS = 1, 0
    assert [o.adapt_order(i, 0.0, 0.0) for i in (1, 2, 3)] == [INTRA, INTRA, CROSS]   # warm-up, intra, cross
    assert o.adapt_order(4, 11.93, 13.13) == CROSS          # the paper's Group 1 example: cross is faster
    assert o.adapt_order(4, 13.13, 11.93) == INTRA
    assert o.adapt_order(9, 5.0, 5.0) == INTRA              # tie keeps the first strategy
    assert o.adapt_order(1000, 1.0, 2.0) == CROSS           # fixed for all later iterations
