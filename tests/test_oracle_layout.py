"""Pins for the CPU checker's byte order (pack / unpack).

The extent order is the row-major (S, B*H, D) array (Sec. IV-B precondition and the row-major
offset of Alg. 2).  The scalar-loop definition is checked against an independent formulation
(NumPy axis transposes), round trips on raw 16-bit patterns, zero padding, canaries around the
extent, the batch-1 coincidence of the two extent modes, and the identity block table.
"""
import numpy as np
import pytest

from oracle import kv_oracle as o

CANARY = 0xA5


def _raw(shape, seed):
    rng = np.random.default_rng(seed)
    return rng.integers(0, 65536, size=shape, dtype=np.uint16)


def _pack_bhsd(x, sec, per_seq=False, lens=None, guard=64):
    B, H, S, D = x.shape
    lens = [S] * B if lens is None else lens
    nb, base, pay = o.tensor_blocks(per_seq, lens, H, D, 2, sec)
    buf = np.full(guard + nb * sec + guard, CANARY, dtype=np.uint8)
    ext = buf[guard:guard + nb * sec]
    o.pack(o.bhsd_source(x.shape), x, per_seq, lens, base, nb, sec, ext)
    assert (buf[:guard] == CANARY).all() and (buf[guard + nb * sec:] == CANARY).all()
    return ext, nb, base, pay


@pytest.mark.parametrize("B,H,S,D,sec", [(1, 2, 256, 64, 512), (3, 2, 37, 64, 512), (2, 5, 19, 32, 4096),
                                         (1, 8, 33, 128, 4096), (4, 1, 7, 16, 512)])
def test_token_major_equals_numpy_transpose(B, H, S, D, sec):
    x = _raw((B, H, S, D), 11 * B + S)
    ext, nb, _, pay = _pack_bhsd(x, sec)
    want = np.ascontiguousarray(x.transpose(2, 0, 1, 3)).view(np.uint8).ravel()
    assert pay == want.size
    assert np.array_equal(ext[:pay], want)
    assert not ext[pay:].any()                                 # pad bytes are zero
    assert nb * sec - pay < sec


def test_token_major_strided_source():
    """S_alloc larger than the valid length: only rows [0, len) are read."""
    B, H, S_alloc, S, D = 2, 3, 50, 21, 32
    x = _raw((B, H, S_alloc, D), 5)
    nb, base, pay = o.tensor_blocks(False, [S] * B, H, D, 2, 512)
    ext = np.zeros(nb * 512, dtype=np.uint8)
    o.pack(o.bhsd_source(x.shape), x, False, [S] * B, base, nb, 512, ext)
    want = np.ascontiguousarray(x[:, :, :S].transpose(2, 0, 1, 3)).view(np.uint8).ravel()
    assert np.array_equal(ext[:pay], want)


def test_per_seq_equals_numpy():
    B, H, S, D, sec = 3, 2, 40, 64, 512
    lens = [40, 13, 1]
    x = _raw((B, H, S, D), 3)
    ext, nb, base, pay = _pack_bhsd(x, sec, per_seq=True, lens=lens)
    for b in range(B):
        start = int(base[b]) * sec
        end = (int(base[b + 1]) if b + 1 < B else nb) * sec
        want = np.ascontiguousarray(x[b, :, :lens[b]].transpose(1, 0, 2)).view(np.uint8).ravel()
        assert np.array_equal(ext[start:start + want.size], want)
        assert not ext[start + want.size:end].any()
        assert end - start - want.size < sec


def test_batch1_modes_coincide():
    x = _raw((1, 4, 77, 64), 9)
    a, _, _, _ = _pack_bhsd(x, 4096, per_seq=False)
    b, _, _, _ = _pack_bhsd(x, 4096, per_seq=True)
    assert np.array_equal(a, b)


@pytest.mark.parametrize("per_seq", [False, True])
def test_round_trip_raw_patterns(per_seq):
    B, H, S, D = 2, 3, 29, 64
    lens = [29, 17] if per_seq else [29, 29]
    x = _raw((B, H, S, D), 21)
    ext, nb, base, _ = _pack_bhsd(x, 512, per_seq=per_seq, lens=lens)
    y = np.full_like(x, 0x7E7E)
    o.unpack(o.bhsd_source(x.shape), y, per_seq, lens, base, 512, ext)
    for b in range(B):
        assert np.array_equal(y[b, :, :lens[b]], x[b, :, :lens[b]])
        assert (y[b, :, lens[b]:] == 0x7E7E).all()             # invalid tokens untouched


def _paged_case(lens, H, D, bt, seed, identity):
    rng = np.random.default_rng(seed)
    per = [-(-n // bt) for n in lens]
    n_pool = sum(per)
    perm = np.arange(n_pool) if identity else rng.permutation(n_pool)
    table = np.full((len(lens), max(per)), -1, dtype=np.int32)
    k = 0
    for b, n in enumerate(per):
        table[b, :n] = perm[k:k + n]
        k += n
    pool = _raw((n_pool, H, bt, D), seed + 1)
    return pool, table


def test_paged_identity_table_equals_bhsd():
    """One sequence, identity table: the pool [n,H,16,D] holds the same tokens as [1,H,S,D]."""
    H, D, bt, S = 3, 32, 16, 64
    pool, table = _paged_case([S], H, D, bt, 2, identity=True)
    src = o.Source(H=H, D=D, paged=True, block_table=table, block_tokens=bt)
    nb, base, pay = o.tensor_blocks(True, [S], H, D, 2, 512)
    ext = np.zeros(nb * 512, dtype=np.uint8)
    o.pack(src, pool, True, [S], base, nb, 512, ext)
    as_bhsd = np.ascontiguousarray(pool.transpose(1, 0, 2, 3).reshape(1, H, S, D))
    ext2, _, _, _ = _pack_bhsd(as_bhsd, 512, per_seq=True, lens=[S])
    assert np.array_equal(ext, ext2)


def test_paged_permuted_equals_gather():
    H, D, bt = 2, 64, 16
    lens = [50, 16, 33]
    pool, table = _paged_case(lens, H, D, bt, 4, identity=False)
    src = o.Source(H=H, D=D, paged=True, block_table=table, block_tokens=bt)
    nb, base, pay = o.tensor_blocks(True, lens, H, D, 2, 512)
    ext = np.full(nb * 512, CANARY, dtype=np.uint8)
    o.pack(src, pool, True, lens, base, nb, 512, ext)
    for b, n in enumerate(lens):
        rows = np.stack([pool[table[b, s // bt], :, s % bt, :] for s in range(n)])   # [n, H, D]
        start = int(base[b]) * 512
        assert np.array_equal(ext[start:start + rows.size * 2], rows.view(np.uint8).ravel())
    # round trip into a fresh pool: slots past len_b of a last block stay untouched
    out = np.full_like(pool, 0x1234)
    o.unpack(src, out, True, lens, base, 512, ext)
    for b, n in enumerate(lens):
        for s in range(-(-n // bt) * bt):
            got = out[table[b, s // bt], :, s % bt, :]
            if s < n:
                assert np.array_equal(got, pool[table[b, s // bt], :, s % bt, :])
            else:
                assert (got == 0x1234).all()


def test_token_major_paged_source():
    """Token-major extent from a paged pool (uniform lengths): equals the gather, transposed."""
    H, D, bt, B, S = 2, 32, 16, 2, 48
    pool, table = _paged_case([S] * B, H, D, bt, 8, identity=False)
    src = o.Source(H=H, D=D, paged=True, block_table=table, block_tokens=bt)
    nb, base, pay = o.tensor_blocks(False, [S] * B, H, D, 2, 512)
    ext = np.zeros(nb * 512, dtype=np.uint8)
    o.pack(src, pool, False, [S] * B, base, nb, 512, ext)
    want = np.stack([np.stack([pool[table[b, s // bt], :, s % bt, :] for b in range(B)]) for s in range(S)])
    assert np.array_equal(ext[:pay], want.view(np.uint8).ravel())


def test_chunk_slices_tile_the_extent():
    """Alg. 2 + Eq. 7-11 token chunks address disjoint byte ranges that tile the whole extent."""
    B, H, S, D, sec, Ctok = 1, 2, 256, 64, 512, 64
    p = o.layout_plan(2, H, 4, D, [S], 2, sec, False, 0, 2048)
    covered = np.zeros(p.region_bytes, dtype=np.int32)
    for n in range(4):
        rc, slba, req = o.token_range(p, n, 0, 0, S)
        assert rc == o.OK
        for c_slba, nlb, off in o.chunk_cmds(slba, req, Ctok * p.row_bytes, sec):
            covered[c_slba * sec:(c_slba + nlb + 1) * sec] += 1
    assert (covered[:2048 * sec] == 0).all()                   # the hole below lba_start is never addressed
    assert (covered[2048 * sec:] == 1).all()


def test_all_core_build_equals_the_defining_build():
    """The -fopenmp build of the same file (the benchmark's all-core timing variant) must give the same bytes and
    the same doubles as the one-thread build every other test uses."""
    rng = np.random.default_rng(5)
    B, H, S, D, sec = 3, 2, 37, 64, 512
    data = rng.integers(0, 65536, size=(B, H, S, D), dtype=np.uint16)
    src = o.bhsd_source(data.shape)
    for per_seq, lens in ((False, [S] * B), (True, [37, 5, 20])):
        nb, base, _ = o.tensor_blocks(per_seq, lens, H, D, 2, sec)
        a = np.full(nb * sec, 0xEE, dtype=np.uint8)
        b = np.full(nb * sec, 0xEE, dtype=np.uint8)
        o.pack(src, data, per_seq, lens, base, nb, sec, a)
        o.pack(src, data, per_seq, lens, base, nb, sec, b, omp=True)
        assert np.array_equal(a, b)
        back_a = np.zeros_like(data)
        back_b = np.zeros_like(data)
        o.unpack(src, back_a, per_seq, lens, base, sec, a)
        o.unpack(src, back_b, per_seq, lens, base, sec, a, omp=True)
        assert np.array_equal(back_a, back_b)
    import torch
    K = torch.randn((B, H, S, D), generator=torch.Generator().manual_seed(3)).to(torch.bfloat16)
    V = torch.randn((B, H, S, D), generator=torch.Generator().manual_seed(4)).to(torch.bfloat16)
    q = torch.randn((B, 4, D), generator=torch.Generator().manual_seed(5)).to(torch.bfloat16)
    lens = [37, 0, 20]
    one = o.attention(src, o.u16(K), o.u16(V), o.u16(q), True, lens, 4)
    many = o.attention(src, o.u16(K), o.u16(V), o.u16(q), True, lens, 4, omp=True)
    assert np.array_equal(one, many)
    assert o.threads(False) == 1 and o.threads(True) >= 1
