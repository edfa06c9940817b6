"""GPU parity: the HIP path (through the C ABI) against the CPU checker, element by element, on
reduced shapes of the five evaluation configs that still span several tiles and a ragged tail.
Pack / unpack / host-region bytes must be bit-exact; attention within 2e-3 max abs error of the fp64
reference (and 1e-2 of the reference's own max magnitude, so the check is not vacuous)."""
import numpy as np
import pytest
import torch

from oracle import kv_oracle as o
from paper_2604_26557_amd import binding as kv
from paper_2604_26557_amd import workloads as W
from kvcase import Case, bits, pinned_bytes

pytestmark = pytest.mark.gpu

ATTN_ATOL = 2e-3
ATTN_REL_OF_MAX = 1e-2
GUARD = 4096
CANARY = 0xA5


def small_configs():
    c = W.CONFIGS
    return [
        c[0],
        W.shrink(c[1], n_layers=3, seq_len=1001),
        W.shrink(c[2], n_layers=4, seq_len=3000, pc_budget_bytes=2 * 2 * 3000 * 2048),
        W.shrink(c[3], n_layers=3, batch=4, len_range=(100, 1500)),
        W.shrink(c[4], n_layers=3, seq_len=600, pc_budget_bytes=1 * 2 * 600 * 32768),
        # shapes outside the five: odd head count (row of 5*8 vectors), B=3 token-major, 512 B sectors
        W.KVConfig("odd_heads", 7, 2, 5, 10, 64, 3, W.F16, 512, 4, 2, W.TOKEN_MAJOR, W.BHSD, 203),
        # token-major extent from a paged source, G = 8
        W.KVConfig("paged_token_major", 8, 2, 1, 8, 128, 2, W.BF16, 4096, 32, 2, W.TOKEN_MAJOR, W.PAGED, 320),
    ]


SMALL = small_configs()
IDS = [c.name for c in SMALL]


@pytest.fixture(scope="module", params=SMALL, ids=IDS)
def case(request):
    torch.cuda.set_device(0)
    return Case(request.param, "cuda", gen_device="cpu")


def _guarded(nbytes):
    buf = torch.full((nbytes + 2 * GUARD,), CANARY, dtype=torch.uint8, device="cuda")
    return buf, buf[GUARD:GUARD + nbytes]


def _guards_intact(buf, nbytes):
    b = buf.cpu().numpy()
    return (b[:GUARD] == CANARY).all() and (b[GUARD + nbytes:] == CANARY).all()


# ------------------------------------------------------------------------------------------ pack
def test_pack_whole_tensor(case):
    r = case.ref
    nbytes = r.n_blocks_tensor * r.lba_size
    for layer in sorted({0, case.cfg.n_layers - 1}):
        for kind in (0, 1):
            buf, dst = _guarded(nbytes)
            kv.kv_offload_pack(case.plan, layer, kind, case.view, kv.KV_SEQ_ALL, 0, 0, dst)
            torch.cuda.synchronize()
            assert np.array_equal(dst.cpu().numpy(), case.expected_extent(layer, kind)), (layer, kind)
            assert _guards_intact(buf, nbytes)


def test_pack_chunk_ranges(case):
    r = case.ref
    layer, kind = case.cfg.n_layers - 1, 1
    want = case.expected_extent(layer, kind)
    nseq = len(case.lens) if r.per_seq else 1
    for b in range(nseq):
        base = int(r.seq_base[b]) * r.lba_size
        for c in kv.kv_plan_chunk_cmds(case.plan, layer, kind, b):
            nbytes = (c.nlb + 1) * r.lba_size
            buf, dst = _guarded(nbytes)
            kv.kv_offload_pack(case.plan, layer, kind, case.view, b, c.tok0, c.ntok, dst)
            torch.cuda.synchronize()
            got = dst.cpu().numpy()
            assert np.array_equal(got, want[base + c.buf_off: base + c.buf_off + nbytes]), (b, c.tok0)
            assert _guards_intact(buf, nbytes)


def test_pack_unpack_both_tensors_in_one_launch(case):
    """kind = KV_KV: K's image, then V's, from one launch; whole extents and one chunk range."""
    r = case.ref
    ext_bytes = r.n_blocks_tensor * r.lba_size
    layer = case.cfg.n_layers - 1
    buf, dst = _guarded(2 * ext_bytes)
    kv.kv_offload_pack(case.plan, layer, kv.KV_KV, case.view, kv.KV_SEQ_ALL, 0, 0, dst)
    torch.cuda.synchronize()
    want_k, want_v = case.expected_extent(layer, 0), case.expected_extent(layer, 1)
    got = dst.cpu().numpy()
    assert np.array_equal(got[:ext_bytes], want_k) and np.array_equal(got[ext_bytes:], want_v)
    assert _guards_intact(buf, 2 * ext_bytes)

    k_new, v_new = case.blank_like_source()
    view = case.make_view(k_new, v_new)
    kv.kv_reload_unpack(case.plan, layer, kv.KV_KV, dst, view, kv.KV_SEQ_ALL, 0, 0)
    torch.cuda.synchronize()
    _check_restored(case, k_new, v_new, [layer])

    c = kv.kv_plan_chunk_cmds(case.plan, layer, 0, 0)[-1]          # the ragged tail chunk of sequence 0
    nbytes = (c.nlb + 1) * r.lba_size
    buf, dst = _guarded(2 * nbytes)
    kv.kv_offload_pack(case.plan, layer, kv.KV_KV, case.view, 0, c.tok0, c.ntok, dst)
    torch.cuda.synchronize()
    got = dst.cpu().numpy()
    assert np.array_equal(got[:nbytes], want_k[c.buf_off:c.buf_off + nbytes])
    assert np.array_equal(got[nbytes:], want_v[c.buf_off:c.buf_off + nbytes])
    assert _guards_intact(buf, 2 * nbytes)


# ------------------------------------------------------------------------------------------ unpack
def test_pack_unpack_several_layers_in_one_call(case):
    """kv_offload_pack_layers / kv_reload_unpack_layers: the images of K and V of a run of layers, back to back in
    tensor-id order, equal the single-tensor images; the inverse restores every layer of the run and no other."""
    r, L = case.ref, case.cfg.n_layers
    image = r.n_blocks_tensor * r.lba_size
    for lb, le in ((0, L), (L - 1, L), (1, 1)):
        n = le - lb
        buf, dst = _guarded(2 * n * image)
        if n == 0:
            dst = buf                                      # an empty run writes nothing anywhere
        kv.kv_offload_pack_layers(case.plan, lb, le, case.view, dst)
        torch.cuda.synchronize()
        got = dst.cpu().numpy()
        for l in range(lb, le):
            for kind in (0, 1):
                j = (l - lb) * 2 + kind
                assert np.array_equal(got[j * image:(j + 1) * image], case.expected_extent(l, kind)), (lb, le, l, kind)
        assert _guards_intact(buf, 2 * n * image) and (n > 0 or (buf.cpu().numpy() == CANARY).all())
        k_new, v_new = case.blank_like_source()
        kv.kv_reload_unpack_layers(case.plan, lb, le, dst, case.make_view(k_new, v_new))
        torch.cuda.synchronize()
        _check_restored(case, k_new, v_new, range(lb, le))
        for l in set(range(L)) - set(range(lb, le)):       # layers outside the run keep their fill
            assert (bits(k_new[l]) == 0x7E7E).all() and (bits(v_new[l]) == 0x7E7E).all()
    small = torch.empty(2 * L * image - 16, dtype=torch.uint8, device="cuda")
    for f, args in ((kv.kv_offload_pack_layers, (case.plan, 0, L, case.view, small)),
                    (kv.kv_reload_unpack_layers, (case.plan, 0, L, small, case.view))):
        with pytest.raises(kv.KVError) as e:
            f(*args)
        assert e.value.code == kv.KV_ENOSPC
    with pytest.raises(kv.KVError) as e:
        kv.kv_offload_pack_layers(case.plan, 0, L + 1, case.view, small)
    assert e.value.code == kv.KV_ERANGE


def _check_restored(case, k_new, v_new, layers, fill=0x7E7E):
    cfg = case.cfg
    for layer in layers:
        for kind, new in ((0, k_new), (1, v_new)):
            got, src = bits(new[layer]), bits(case.tensor_cpu(layer, kind))
            if case.paged:
                bt = cfg.block_tokens
                table = case.table_cpu.numpy()
                touched = np.zeros(got.shape[:1] + got.shape[2:3], dtype=bool)   # [n_pool, bt]
                for b, n in enumerate(case.lens):
                    for s in range(n):
                        touched[table[b, s // bt], s % bt] = True
                m = touched[:, None, :, None]
                assert np.array_equal(np.where(m, got, 0), np.where(m, src, 0))
                assert (np.where(m, fill, got) == fill).all()                     # other slots untouched
            else:
                for b, n in enumerate(case.lens):
                    assert np.array_equal(got[b, :, :n], src[b, :, :n])
                    assert (got[b, :, n:] == fill).all()


def test_unpack_whole_tensor(case):
    k_new, v_new = case.blank_like_source()
    view = case.make_view(k_new, v_new)
    layers = sorted({0, case.cfg.n_layers - 1})
    for layer in layers:
        for kind in (0, 1):
            ext = torch.from_numpy(case.expected_extent(layer, kind)).cuda()
            kv.kv_reload_unpack(case.plan, layer, kind, ext, view, kv.KV_SEQ_ALL, 0, 0)
    torch.cuda.synchronize()
    _check_restored(case, k_new, v_new, layers)


def test_unpack_chunk_ranges(case):
    r = case.ref
    k_new, v_new = case.blank_like_source()
    view = case.make_view(k_new, v_new)
    layer = 0
    nseq = len(case.lens) if r.per_seq else 1
    for kind in (0, 1):
        ext = case.expected_extent(layer, kind)
        for b in range(nseq):
            base = int(r.seq_base[b]) * r.lba_size
            for c in kv.kv_plan_chunk_cmds(case.plan, layer, kind, b):
                nbytes = (c.nlb + 1) * r.lba_size
                img = torch.from_numpy(ext[base + c.buf_off: base + c.buf_off + nbytes].copy()).cuda()
                kv.kv_reload_unpack(case.plan, layer, kind, img, view, b, c.tok0, c.ntok)
    torch.cuda.synchronize()
    _check_restored(case, k_new, v_new, [layer])


@pytest.mark.parametrize("cfg", [SMALL[0], SMALL[3], SMALL[5]], ids=lambda c: c.name)
def test_round_trip_raw_bit_patterns(cfg):
    """Pack is a byte move: NaN / Inf / denormal payloads must survive unchanged."""
    case = Case(cfg, "cuda", raw=True, gen_device="cpu", s_extra=3)
    r = case.ref
    k_new, v_new = case.blank_like_source()
    view = case.make_view(k_new, v_new)
    nbytes = r.n_blocks_tensor * r.lba_size
    for layer in range(cfg.n_layers):
        for kind in (0, 1):
            buf, dst = _guarded(nbytes)
            kv.kv_offload_pack(case.plan, layer, kind, case.view, kv.KV_SEQ_ALL, 0, 0, dst)
            torch.cuda.synchronize()
            assert np.array_equal(dst.cpu().numpy(), case.expected_extent(layer, kind))
            kv.kv_reload_unpack(case.plan, layer, kind, dst, view, kv.KV_SEQ_ALL, 0, 0)
    torch.cuda.synchronize()
    _check_restored(case, k_new, v_new, range(cfg.n_layers))


def test_pack_shorter_than_capacity_zero_fills():
    """Valid length below the extent capacity: rows [0,len) then zeros to the end of the extent."""
    cfg = W.shrink(W.CONFIGS[0], seq_len=256)
    case = Case(cfg, "cuda", gen_device="cpu")
    lens = [100]
    view = kv.bhsd_view(case.k, case.v, lens, case.lens_dev)
    r = case.ref
    nbytes = r.n_blocks_tensor * r.lba_size
    buf, dst = _guarded(nbytes)
    kv.kv_offload_pack(case.plan, 1, 0, view, kv.KV_SEQ_ALL, 0, 0, dst)
    torch.cuda.synchronize()
    want = np.zeros(nbytes, dtype=np.uint8)
    t = case.k_cpu[1]
    o.pack(case.source(t), o.u16(t), False, lens, r.seq_base, r.n_blocks_tensor, r.lba_size, want)
    assert np.array_equal(dst.cpu().numpy(), want) and not want[100 * 256:].any()
    assert _guards_intact(buf, nbytes)


def test_kernel_argument_errors(case):
    """Bad arguments are rejected on the host before anything is launched."""
    r = case.ref
    dst = torch.zeros(r.n_blocks_tensor * r.lba_size, dtype=torch.uint8, device="cuda")

    def code(fn):
        with pytest.raises(kv.KVError) as e:
            fn()
        return e.value.code

    cap = case.lens[0]
    assert code(lambda: kv.kv_offload_pack(case.plan, 99, 0, case.view, kv.KV_SEQ_ALL, 0, 0, dst)) == kv.KV_ERANGE
    assert code(lambda: kv.kv_offload_pack(case.plan, 0, 3, case.view, kv.KV_SEQ_ALL, 0, 0, dst)) == kv.KV_EINVAL
    assert code(lambda: kv.kv_offload_pack(case.plan, 0, 0, case.view, 0, 0, cap + 1, dst)) == kv.KV_ERANGE
    assert code(lambda: kv.kv_offload_pack(case.plan, 0, 0, case.view, kv.KV_SEQ_ALL, 0, 0, dst[:4096])) == kv.KV_ENOSPC
    assert code(lambda: kv.kv_offload_pack(case.plan, 0, 0, case.view, kv.KV_SEQ_ALL, 0, 0, dst[8:])) == kv.KV_EINVAL
    if (r.row_bytes % r.lba_size) != 0 and cap > 2:
        assert code(lambda: kv.kv_offload_pack(case.plan, 0, 0, case.view, 0, 1, 1, dst)) == kv.KV_EALIGN
    assert code(lambda: kv.kv_reload_unpack(case.plan, 0, 0, dst[:4096], case.view, kv.KV_SEQ_ALL, 0, 0)) == kv.KV_ENOSPC
    assert code(lambda: kv.kv_reload_unpack(case.plan, -1, 0, dst, case.view, kv.KV_SEQ_ALL, 0, 0)) == kv.KV_ERANGE

    # decode attention
    cfg = case.cfg
    q = W.query(cfg, 0, "cuda")
    out = torch.zeros((len(case.lens), cfg.n_q_heads, cfg.head_dim), dtype=torch.float32, device="cuda")
    ws = torch.empty(kv.kv_decode_attn_workspace(case.plan, 0, max(case.lens)), dtype=torch.uint8, device="cuda")
    attn = lambda **kw: kv.kv_decode_attn(**dict(dict(plan=case.plan, kv=case.view, layer=0, q=q, out=out,
                                                      out_dtype=kv.KV_OUT_F32, n_splits=0, workspace=ws), **kw))
    attn()
    torch.cuda.synchronize()
    assert code(lambda: attn(layer=99)) == kv.KV_ERANGE
    assert code(lambda: attn(out_dtype=5)) == kv.KV_EINVAL
    assert code(lambda: attn(n_splits=1025)) == kv.KV_EINVAL
    assert code(lambda: attn(n_splits=-1)) == kv.KV_EINVAL
    assert code(lambda: attn(workspace=ws[:64])) == kv.KV_ENOSPC
    misaligned = torch.zeros(q.numel() * 2 + 16, dtype=torch.uint8, device="cuda")[2:]
    assert code(lambda: attn(q=misaligned)) == kv.KV_EINVAL


# ------------------------------------------------------------------------------------------ attention
def _attn_check(got: torch.Tensor, want: np.ndarray):
    g = got.double().cpu().numpy()
    err = np.abs(g - want).max()
    scale = np.abs(want).max()
    assert err <= ATTN_ATOL, err
    assert err <= ATTN_REL_OF_MAX * scale, (err, scale)


@pytest.mark.parametrize("n_splits", [0, 1, 3, 70, 200])
def test_decode_attention(case, n_splits):
    cfg = case.cfg
    max_len = max(case.lens)
    ws = torch.empty(kv.kv_decode_attn_workspace(case.plan, n_splits, max_len), dtype=torch.uint8, device="cuda")
    for layer in sorted({0, cfg.n_layers - 1}):
        q = W.query(cfg, layer, "cpu")
        qd = q.cuda()
        out = torch.full((len(case.lens), cfg.n_q_heads, cfg.head_dim), float("nan"), dtype=torch.float32, device="cuda")
        kv.kv_decode_attn(case.plan, case.view, layer, qd, out, kv.KV_OUT_F32, n_splits, ws)
        torch.cuda.synchronize()
        _attn_check(out, case.expected_attention(layer, q))


def test_decode_attention_16bit_output_and_short_lengths(case):
    """Output in the KV dtype is the fp32 result rounded to nearest even; a zero-length sequence gives zeros."""
    cfg = case.cfg
    lens = list(case.lens)
    lens[0] = 1
    if len(lens) > 1:
        lens[1] = 0
    lens_dev = torch.tensor(lens, dtype=torch.int32, device="cuda")
    view = (kv.paged_view(case.k, case.v, case.table_dev, lens, lens_dev) if case.paged
            else kv.bhsd_view(case.k, case.v, lens, lens_dev))
    ws = torch.empty(kv.kv_decode_attn_workspace(case.plan, 0, max(lens)), dtype=torch.uint8, device="cuda")
    q = W.query(cfg, 0, "cpu")
    shape = (len(lens), cfg.n_q_heads, cfg.head_dim)
    out32 = torch.empty(shape, dtype=torch.float32, device="cuda")
    out16 = torch.empty(shape, dtype=cfg.torch_dtype, device="cuda")
    kv.kv_decode_attn(case.plan, view, 0, q.cuda(), out32, kv.KV_OUT_F32, 0, ws)
    kv.kv_decode_attn(case.plan, view, 0, q.cuda(), out16, kv.KV_OUT_SAME, 0, ws)
    torch.cuda.synchronize()
    K, V = case.k_cpu[0], case.v_cpu[0]
    want = o.attention(case.source(K), o.u16(K), o.u16(V), o.u16(q), cfg.dtype == W.BF16, lens, cfg.n_q_heads)
    _attn_check(out32, want)
    assert torch.equal(out16, out32.to(cfg.torch_dtype))
    if len(lens) > 1:
        assert not out32[1].any()


@pytest.mark.parametrize("B", [64, 65, 130])
@pytest.mark.parametrize("n_splits", [0, 5])
def test_decode_attention_many_ragged_sequences(B, n_splits):
    """Ragged batches at and beyond 64 sequences: up to 64 the grid holds only the splits with tokens (the owner
    search uses one lane per sequence), beyond that the full (split, head group, sequence) grid runs and the
    combine pass reads each sequence's own split count.  Some sequences are empty."""
    cfg = W.KVConfig(f"many{B}", 500 + B, 1, 2, 4, 64, B, W.F16, 512, 4, 2, W.PER_SEQ, W.BHSD, 0, len_range=(1, 900))
    lens = W.seq_lens(cfg)
    lens[3] = 0
    lens[B - 1] = 0
    lens[B // 2] = 900
    case = Case(cfg, "cuda", gen_device="cpu", lens=lens)
    view = case.make_view(case.k, case.v, lens)
    q = W.query(cfg, 0, "cpu")
    out = torch.full((B, cfg.n_q_heads, cfg.head_dim), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(kv.kv_decode_attn_workspace(case.plan, n_splits, max(lens)), dtype=torch.uint8, device="cuda")
    kv.kv_decode_attn(case.plan, view, 0, q.cuda(), out, kv.KV_OUT_F32, n_splits, ws)
    torch.cuda.synchronize()
    K, V = case.k_cpu[0], case.v_cpu[0]
    want = o.attention(case.source(K), o.u16(K), o.u16(V), o.u16(q), False, lens, cfg.n_q_heads)
    _attn_check(out, want)
    assert not out[3].any() and not out[B - 1].any()


# ------------------------------------------------------------------------------------------ pipeline
# (span_chunks, depth, copy_streams, d2h_mode, h2d_mode)
@pytest.mark.parametrize("D,G", [(64, 1), (64, 4), (128, 2), (128, 8), (256, 1), (256, 4)])
@pytest.mark.parametrize("paged", [False, True], ids=["bhsd", "paged"])
def test_decode_attention_long_splits_every_head_shape(D, G, paged):
    """Splits long enough that the wavefronts of a workgroup claim steps on demand (more than two rounds of eight),
    for every head width and query-group size the kernel is instantiated for, ragged (per-sequence split table)
    and uniform, automatic and given split counts."""
    H = 2
    for i, lens in enumerate(([5000, 37, 1201], [2100], [777, 777])):
        cfg = W.KVConfig(f"attn_D{D}_G{G}", 900 + 7 * i + D + G, 1, H, H * G, D, len(lens), W.BF16 if (D + G + i) % 2 else W.F16,
                         512, 8, 2, W.PER_SEQ, W.PAGED if paged else W.BHSD, 0, len_range=(1, 2))
        case = Case(cfg, "cuda", lens=list(lens))
        q = W.query(cfg, 0, "cpu")
        want = case.expected_attention(0, q)
        for n_splits in (0, 2):
            out = torch.full((len(lens), H * G, D), float("nan"), dtype=torch.float32, device="cuda")
            ws = torch.empty(kv.kv_decode_attn_workspace(case.plan, n_splits, max(lens)), dtype=torch.uint8, device="cuda")
            kv.kv_decode_attn(case.plan, case.view, 0, q.cuda(), out, kv.KV_OUT_F32, n_splits, ws)
            torch.cuda.synchronize()
            _attn_check(out, want)


@pytest.mark.parametrize("bt", [1, 8, 12, 32, 48])
def test_paged_source_other_block_sizes(bt):
    """Paged pools whose blocks hold other than 16 token rows (a power of two below and above the 16-row tile, sizes
    that are not powers of two, one row per block): pack, unpack, decode attention and a pipeline round trip against
    the checker."""
    torch.cuda.set_device(0)
    H, G, D = 2, 4, 128
    lens = [700, 33, 257]
    cfg = W.KVConfig(f"paged_bt{bt}", 4200 + bt, 2, H, H * G, D, len(lens), W.F16 if bt % 2 else W.BF16, 512, 8, 2, W.PER_SEQ,
                     W.PAGED, 0, len_range=(1, 2), block_tokens=bt)
    case = Case(cfg, "cuda", lens=list(lens), raw=True)
    r = case.ref
    nbytes = r.n_blocks_tensor * r.lba_size
    for layer, kind in ((0, 0), (1, 1)):
        buf, dst = _guarded(nbytes)
        kv.kv_offload_pack(case.plan, layer, kind, case.view, kv.KV_SEQ_ALL, 0, 0, dst)
        torch.cuda.synchronize()
        assert np.array_equal(dst.cpu().numpy(), case.expected_extent(layer, kind)) and _guards_intact(buf, nbytes)
    region = pinned_bytes(r.region_bytes, 0x5A)
    arena = np.full(max(r.pageable_bytes, 1), 0x5A, dtype=np.uint8)
    kv.kv_pipeline_run(case.plan, kv.KV_DIR_OFFLOAD, 0, cfg.n_layers, case.view, region, arena, depth=2)
    want_region, _ = case.expected_host(fill=0x5A)
    assert np.array_equal(region.numpy()[:r.region_bytes], want_region[:r.region_bytes])
    k_new, v_new = case.blank_like_source()
    kv.kv_pipeline_run(case.plan, kv.KV_DIR_RELOAD, 0, cfg.n_layers, case.make_view(k_new, v_new), region, arena, depth=2)
    _check_restored(case, k_new, v_new, range(cfg.n_layers))
    # attention on values that are numbers (the raw bit patterns above include NaNs)
    case = Case(cfg, "cuda", lens=list(lens))
    q = W.query(cfg, 0, "cpu")
    want = case.expected_attention(0, q)
    for n_splits in (0, 3):
        out = torch.full((len(lens), H * G, D), float("nan"), dtype=torch.float32, device="cuda")
        ws = torch.empty(kv.kv_decode_attn_workspace(case.plan, n_splits, max(lens)), dtype=torch.uint8, device="cuda")
        kv.kv_decode_attn(case.plan, case.view, 0, q.cuda(), out, kv.KV_OUT_F32, n_splits, ws)
        torch.cuda.synchronize()
        _attn_check(out, want)


PIPE_VARIANTS = [(0, 3, 0, kv.KV_COPY_AUTO, kv.KV_COPY_AUTO),
                 (1, 2, 1, kv.KV_COPY_MEMCPY, kv.KV_COPY_MEMCPY),
                 (2, 4, 3, kv.KV_COPY_KERNEL, kv.KV_COPY_KERNEL),
                 (0, 1, 0, kv.KV_COPY_AUTO, kv.KV_COPY_AUTO),
                 (0, 8, 4, kv.KV_COPY_MEMCPY, kv.KV_COPY_KERNEL)]


@pytest.mark.parametrize("span_chunks,depth,copy_streams,d2h,h2d", PIPE_VARIANTS)
def test_pipeline_offload_reload(case, span_chunks, depth, copy_streams, d2h, h2d):
    cfg, r = case.cfg, case.ref
    FILL = 0xC3
    region = pinned_bytes(r.region_bytes, FILL)
    arena = np.full(max(r.pageable_bytes, 1), FILL, dtype=np.uint8)
    st = kv.kv_pipeline_run(case.plan, kv.KV_DIR_OFFLOAD, 0, cfg.n_layers, case.view, region, arena,
                            depth=depth, span_chunks=span_chunks, copy_streams=copy_streams, d2h_mode=d2h, h2d_mode=h2d)
    want_region, want_arena = case.expected_host(fill=FILL)
    assert np.array_equal(region.numpy()[:r.region_bytes], want_region[:r.region_bytes])
    assert np.array_equal(arena[:r.pageable_bytes], want_arena[:r.pageable_bytes])
    assert st.max_in_flight <= depth and st.n_chunks > 0
    assert st.bytes_direct == r.direct_blocks * r.lba_size and st.bytes_pagecache == r.pageable_bytes
    assert st.lba_seq_breaks == 0        # K then V, layers ascending: one ascending LBA run (Sec. IV-B placement)

    k_new, v_new = case.blank_like_source()
    view = case.make_view(k_new, v_new)
    st = kv.kv_pipeline_run(case.plan, kv.KV_DIR_RELOAD, 0, cfg.n_layers, view, region, arena,
                            depth=depth, span_chunks=span_chunks, copy_streams=copy_streams, d2h_mode=d2h, h2d_mode=h2d)
    assert st.max_in_flight <= depth
    _check_restored(case, k_new, v_new, range(cfg.n_layers))


@pytest.mark.parametrize("depth", [1, 3])
def test_pipeline_chunk_trace_shows_commands_and_depth_rule(case, depth):
    """The per-command record of a run: the commands are exactly those of Eq. 7-11 for every tensor (and sequence)
    in tensor-id order, as the checker computes them, and the queue-depth rule of Sec. IV-B "Data Flow" holds on the
    issuing thread's clock: command c is issued only after command c - depth was harvested."""
    from oracle import kv_oracle as o
    cfg, r = case.cfg, case.ref
    region = pinned_bytes(r.region_bytes, 0)
    arena = np.zeros(max(r.pageable_bytes, 1), dtype=np.uint8)
    nseq = len(case.lens) if r.per_seq else 1
    want = []
    for n in range(2 * cfg.n_layers):
        for b in range(nseq):
            rc, slba, req = o.token_range(r, n, b, 0, r.cap[b])
            assert rc == o.OK
            req = -(-req // r.lba_size) * r.lba_size           # the range reaches the extent tail: padded to a sector
            for c_slba, nlb, _ in o.chunk_cmds(slba, req, cfg.chunk_tokens * r.row_bytes, r.lba_size):
                want.append((n // 2, n % 2, int(r.path[n]), c_slba * r.lba_size, (nlb + 1) * r.lba_size))
    k_new, v_new = case.blank_like_source()
    for direction, view in ((kv.KV_DIR_OFFLOAD, case.view), (kv.KV_DIR_RELOAD, case.make_view(k_new, v_new))):
        st = kv.kv_pipeline_run(case.plan, direction, 0, cfg.n_layers, view, region, arena, depth=depth,
                                trace_cap=len(want) + 8)
        tr = st.trace
        assert st.n_traced == st.n_chunks == len(want)
        # the checker's path codes are 0 direct / 1 page-cache; the library's constants are compared by meaning
        got = [(t.layer, t.kind, 0 if t.path == kv.KV_PATH_DIRECT else 1, t.host_off, t.bytes) for t in tr]
        assert got == want
        for c, t in enumerate(tr):
            assert 0.0 <= t.t_issue_s <= t.t_done_s <= st.wall_s
            if c > 0:
                assert tr[c - 1].t_issue_s <= t.t_issue_s and tr[c - 1].t_done_s <= t.t_done_s   # harvested in issue order
            if c >= depth:
                assert tr[c - depth].t_done_s <= t.t_issue_s
    _check_restored(case, k_new, v_new, range(cfg.n_layers))
    # a record shorter than the run keeps the first entries only
    st = kv.kv_pipeline_run(case.plan, kv.KV_DIR_OFFLOAD, 0, cfg.n_layers, case.view, region, arena, depth=2, trace_cap=3)
    assert st.n_traced == min(3, st.n_chunks) and [(t.host_off, t.bytes) for t in st.trace] == [w[3:] for w in want[:st.n_traced]]


def test_pipeline_without_issue_pacing(case):
    """KV_PIPE_NO_PACING: every command is queued as soon as the depth rule allows; same bytes either way."""
    cfg, r = case.cfg, case.ref
    FILL = 0x3C
    region = pinned_bytes(r.region_bytes, FILL)
    arena = np.full(max(r.pageable_bytes, 1), FILL, dtype=np.uint8)
    want_region, want_arena = case.expected_host(fill=FILL)
    for pacing in (False, True):
        region.fill_(FILL)
        arena[:] = FILL
        st = kv.kv_pipeline_run(case.plan, kv.KV_DIR_OFFLOAD, 0, cfg.n_layers, case.view, region, arena, depth=3, pacing=pacing)
        assert np.array_equal(region.numpy()[:r.region_bytes], want_region[:r.region_bytes])
        assert np.array_equal(arena[:r.pageable_bytes], want_arena[:r.pageable_bytes])
        assert st.max_in_flight <= 3 and st.pace_GBps >= 0.0
        k_new, v_new = case.blank_like_source()
        kv.kv_pipeline_run(case.plan, kv.KV_DIR_RELOAD, 0, cfg.n_layers, case.make_view(k_new, v_new), region, arena,
                           depth=3, pacing=pacing)
        _check_restored(case, k_new, v_new, range(cfg.n_layers))


def test_pipeline_serialized_reference_run(case):
    """The no-overlap reference of the overlap fraction (every stage to completion before the next): same bytes,
    same reload, same attention, one command in flight."""
    cfg, r = case.cfg, case.ref
    FILL = 0x11
    region = pinned_bytes(r.region_bytes, FILL)
    arena = np.full(max(r.pageable_bytes, 1), FILL, dtype=np.uint8)
    st = kv.kv_pipeline_run(case.plan, kv.KV_DIR_OFFLOAD, 0, cfg.n_layers, case.view, region, arena, depth=1, serialize=True)
    assert st.max_in_flight == 1
    want_region, want_arena = case.expected_host(fill=FILL)
    assert np.array_equal(region.numpy()[:r.region_bytes], want_region[:r.region_bytes])
    assert np.array_equal(arena[:r.pageable_bytes], want_arena[:r.pageable_bytes])
    k_new, v_new = case.blank_like_source()
    qd = [W.query(cfg, l, "cpu").cuda() for l in range(cfg.n_layers)]
    outs = [torch.zeros((len(case.lens), cfg.n_q_heads, cfg.head_dim), dtype=torch.float32, device="cuda")
            for _ in range(cfg.n_layers)]
    st = kv.kv_pipeline_run(case.plan, kv.KV_DIR_RELOAD_ATTN, 0, cfg.n_layers, case.make_view(k_new, v_new), region, arena,
                            depth=1, serialize=True, q_layers=qd, out_layers=outs)
    assert st.max_in_flight == 1
    _check_restored(case, k_new, v_new, range(cfg.n_layers))
    _attn_check(outs[-1], case.expected_attention(cfg.n_layers - 1, qd[-1].cpu()))


@pytest.mark.parametrize("span_chunks", [0, 1])
def test_pipeline_reload_attention(case, span_chunks):
    cfg, r = case.cfg, case.ref
    region = pinned_bytes(r.region_bytes, 0)
    arena = np.zeros(max(r.pageable_bytes, 1), dtype=np.uint8)
    kv.kv_pipeline_run(case.plan, kv.KV_DIR_OFFLOAD, 0, cfg.n_layers, case.view, region, arena, depth=cfg.depth)
    k_new, v_new = case.blank_like_source()
    view = case.make_view(k_new, v_new)
    qs = [W.query(cfg, l, "cpu") for l in range(cfg.n_layers)]
    qd = [q.cuda() for q in qs]
    outs = [torch.full((len(case.lens), cfg.n_q_heads, cfg.head_dim), float("nan"), dtype=torch.float32, device="cuda")
            for _ in range(cfg.n_layers)]
    st = kv.kv_pipeline_run(case.plan, kv.KV_DIR_RELOAD_ATTN, 0, cfg.n_layers, view, region, arena,
                            depth=cfg.depth, q_layers=qd, out_layers=outs, span_chunks=span_chunks, time_kernels=True)
    assert st.kernel_launches[kv.KV_KERNEL_ATTN_PARTIAL] == cfg.n_layers
    for l in range(cfg.n_layers):
        _attn_check(outs[l], case.expected_attention(l, qs[l]))
    _check_restored(case, k_new, v_new, range(cfg.n_layers))


def test_pipeline_reload_attention_from_extent(case):
    """Decode attention fed straight from the staged extent images (no unpack): same outputs, and the
    destination view is neither read nor written."""
    cfg, r = case.cfg, case.ref
    region = pinned_bytes(r.region_bytes, 0)
    arena = np.zeros(max(r.pageable_bytes, 1), dtype=np.uint8)
    kv.kv_pipeline_run(case.plan, kv.KV_DIR_OFFLOAD, 0, cfg.n_layers, case.view, region, arena, depth=cfg.depth)
    k_new, v_new = case.blank_like_source()
    view = case.make_view(k_new, v_new)
    qs = [W.query(cfg, l, "cpu") for l in range(cfg.n_layers)]
    qd = [q.cuda() for q in qs]
    outs = [torch.full((len(case.lens), cfg.n_q_heads, cfg.head_dim), float("nan"), dtype=torch.float32, device="cuda")
            for _ in range(cfg.n_layers)]
    st = kv.kv_pipeline_run(case.plan, kv.KV_DIR_RELOAD_ATTN, 0, cfg.n_layers, view, region, arena,
                            depth=cfg.depth, q_layers=qd, out_layers=outs, attn_from_extent=True)
    assert st.kernel_launches[kv.KV_KERNEL_UNPACK] == 0
    assert st.kernel_launches[kv.KV_KERNEL_ATTN_PARTIAL] == cfg.n_layers
    for l in range(cfg.n_layers):
        _attn_check(outs[l], case.expected_attention(l, qs[l]))
        assert (bits(k_new[l]) == 0x7E7E).all() and (bits(v_new[l]) == 0x7E7E).all()
    with pytest.raises(kv.KVError):
        kv.kv_pipeline_run(case.plan, kv.KV_DIR_RELOAD_ATTN, 0, cfg.n_layers, view, region, arena, depth=cfg.depth,
                           q_layers=qd, out_layers=outs, attn_from_extent=True, span_chunks=1)


@pytest.mark.parametrize("span_chunks,order_pc,order_direct", [(0, kv.KV_ORDER_INTRA, kv.KV_ORDER_INTRA),
                                                              (2, kv.KV_ORDER_INTRA, kv.KV_ORDER_CROSS),
                                                              (0, kv.KV_ORDER_CROSS, kv.KV_ORDER_INTRA)])
def test_pipeline_overlap_orders(case, span_chunks, order_pc, order_direct):
    """Both overlap strategies (K then V, or K and V alternating) move the same bytes; the per-group
    clock runs for every path group that has layers."""
    cfg, r = case.cfg, case.ref
    FILL = 0x3C
    region = pinned_bytes(r.region_bytes, FILL)
    arena = np.full(max(r.pageable_bytes, 1), FILL, dtype=np.uint8)
    kw = dict(depth=cfg.depth, span_chunks=span_chunks, order_pagecache=order_pc, order_direct=order_direct)
    st = kv.kv_pipeline_run(case.plan, kv.KV_DIR_OFFLOAD, 0, cfg.n_layers, case.view, region, arena, **kw)
    want_region, want_arena = case.expected_host(fill=FILL)
    assert np.array_equal(region.numpy()[:r.region_bytes], want_region[:r.region_bytes])
    assert np.array_equal(arena[:r.pageable_bytes], want_arena[:r.pageable_bytes])
    k_new, v_new = case.blank_like_source()
    view = case.make_view(k_new, v_new)
    qd = [W.query(cfg, l, "cuda") for l in range(cfg.n_layers)]
    outs = [torch.zeros((len(case.lens), cfg.n_q_heads, cfg.head_dim), dtype=torch.float32, device="cuda")
            for _ in range(cfg.n_layers)]
    st = kv.kv_pipeline_run(case.plan, kv.KV_DIR_RELOAD_ATTN, 0, cfg.n_layers, view, region, arena,
                            q_layers=qd, out_layers=outs, **kw)
    _check_restored(case, k_new, v_new, range(cfg.n_layers))
    _attn_check(outs[0], case.expected_attention(0, qd[0].cpu()))
    assert (st.group_seconds[0] > 0) == (r.n1 > 0) and (st.group_seconds[1] > 0) == (r.n1 < r.L)
    assert st.max_in_flight <= cfg.depth
    # alternating K and V commands are two interleaved ascending streams: the single run is broken
    if order_direct == kv.KV_ORDER_INTRA and r.n1 < r.L:
        assert st.lba_seq_breaks > 0
    else:
        assert st.lba_seq_breaks == 0


def test_adaptive_strategy_over_decode_iterations(case):
    """Five decode iterations driven by the selector: orders follow warm-up / intra / cross / chosen, and
    every iteration reloads the same bytes."""
    cfg, r = case.cfg, case.ref
    region = pinned_bytes(r.region_bytes, 0)
    arena = np.zeros(max(r.pageable_bytes, 1), dtype=np.uint8)
    kv.kv_pipeline_run(case.plan, kv.KV_DIR_OFFLOAD, 0, cfg.n_layers, case.view, region, arena, depth=cfg.depth)
    a = kv.kv_adapt_init()
    seen = []
    for it in range(5):
        orders = (kv.kv_adapt_order(a, 0), kv.kv_adapt_order(a, 1))
        seen.append(orders)
        k_new, v_new = case.blank_like_source()
        st = kv.kv_pipeline_run(case.plan, kv.KV_DIR_RELOAD, 0, cfg.n_layers, case.make_view(k_new, v_new), region, arena,
                                depth=cfg.depth, order_pagecache=orders[0], order_direct=orders[1])
        _check_restored(case, k_new, v_new, [0, cfg.n_layers - 1])
        kv.kv_adapt_update(a, st)
    I, C_ = kv.KV_ORDER_INTRA, kv.KV_ORDER_CROSS
    assert seen[:3] == [(I, I), (I, I), (C_, C_)]
    assert seen[3] == seen[4] == (a.chosen[0], a.chosen[1])
    for g in (0, 1):
        want = C_ if a.gbps[g][C_] > a.gbps[g][I] else I
        assert a.chosen[g] == want


def test_pipeline_layer_subrange_and_other_chunk_size(case):
    """Only the requested layers move; a different (aligned) chunk size gives the same bytes."""
    cfg, r = case.cfg, case.ref
    if cfg.n_layers < 3:
        pytest.skip("needs 3 layers")
    FILL = 0x5A
    region = pinned_bytes(r.region_bytes, FILL)
    arena = np.full(max(r.pageable_bytes, 1), FILL, dtype=np.uint8)
    sec_rows = max(1, r.lba_size // r.row_bytes)
    C = 3 * sec_rows * 8
    kv.kv_pipeline_run(case.plan, kv.KV_DIR_OFFLOAD, 1, 3, case.view, region, arena, chunk_tokens=C, depth=2)
    want_region, want_arena = case.expected_host(layers=[1, 2], fill=FILL)
    assert np.array_equal(region.numpy()[:r.region_bytes], want_region[:r.region_bytes])
    assert np.array_equal(arena[:r.pageable_bytes], want_arena[:r.pageable_bytes])
    # a chunk larger than any (sub-)extent: one command per tensor (and sequence)
    region2 = pinned_bytes(r.region_bytes, FILL)
    arena2 = np.full(max(r.pageable_bytes, 1), FILL, dtype=np.uint8)
    st = kv.kv_pipeline_run(case.plan, kv.KV_DIR_OFFLOAD, 1, 3, case.view, region2, arena2, chunk_tokens=sec_rows * 100000,
                            depth=8)
    nseq = len(case.lens) if r.per_seq else 1
    assert st.n_chunks == 4 * nseq
    assert np.array_equal(region2.numpy()[:r.region_bytes], want_region[:r.region_bytes])
    assert np.array_equal(arena2[:r.pageable_bytes], want_arena[:r.pageable_bytes])


@pytest.mark.parametrize("span_chunks,limit_sectors", [(0, 1), (0, 3), (2, 5)])
def test_pipeline_transfer_size_limit(case, span_chunks, limit_sectors):
    """A command-size limit (Eq. 7 on a device's maximum transfer size) splits every chunk into commands of at
    most that many whole sectors: same bytes on the host and back, and the command count of Eq. 8 per chunk."""
    cfg, r = case.cfg, case.ref
    FILL = 0xA7
    region = pinned_bytes(r.region_bytes, FILL)
    arena = np.full(max(r.pageable_bytes, 1), FILL, dtype=np.uint8)
    sec = r.lba_size
    limit = limit_sectors * sec + sec // 2          # not a sector multiple: aligned down
    kw = dict(depth=3, span_chunks=span_chunks, max_cmd_bytes=limit)
    st = kv.kv_pipeline_run(case.plan, kv.KV_DIR_OFFLOAD, 0, cfg.n_layers, case.view, region, arena, **kw)
    want_region, want_arena = case.expected_host(fill=FILL)
    assert np.array_equal(region.numpy()[:r.region_bytes], want_region[:r.region_bytes])
    assert np.array_equal(arena[:r.pageable_bytes], want_arena[:r.pageable_bytes])
    nseq = len(case.lens) if r.per_seq else 1
    n_cmds = 0
    for layer in range(cfg.n_layers):
        for kind in (0, 1):
            for b in range(nseq):
                for c in kv.kv_plan_chunk_cmds(case.plan, layer, kind, b):
                    n_cmds += -(-(c.nlb + 1) // limit_sectors)
    assert st.n_chunks == n_cmds and st.max_in_flight <= 3
    k_new, v_new = case.blank_like_source()
    st = kv.kv_pipeline_run(case.plan, kv.KV_DIR_RELOAD, 0, cfg.n_layers, case.make_view(k_new, v_new), region, arena, **kw)
    assert st.n_chunks == n_cmds
    _check_restored(case, k_new, v_new, range(cfg.n_layers))
    with pytest.raises(kv.KVError) as e:
        kv.kv_pipeline_run(case.plan, kv.KV_DIR_OFFLOAD, 0, cfg.n_layers, case.view, region, arena, depth=3,
                           max_cmd_bytes=sec - 1)
    assert e.value.code == kv.KV_EINVAL


def test_pipeline_argument_errors(case):
    cfg, r = case.cfg, case.ref
    region = pinned_bytes(r.region_bytes, 0)
    arena = np.zeros(max(r.pageable_bytes, 1), dtype=np.uint8)

    def code(**kw):
        a = dict(plan=case.plan, direction=kv.KV_DIR_OFFLOAD, layer_begin=0, layer_end=cfg.n_layers, view=case.view,
                 lba_region=region, pageable=arena, depth=2)
        a.update(kw)
        with pytest.raises(kv.KVError) as e:
            kv.kv_pipeline_run(**a)
        return e.value.code

    assert code(depth=0) == kv.KV_EINVAL
    assert code(depth=1025) == kv.KV_EINVAL
    assert code(chunk_tokens=-1) == kv.KV_EINVAL
    assert code(copy_streams=5) == kv.KV_EINVAL
    assert code(d2h_mode=7) == kv.KV_EINVAL and code(h2d_mode=-1) == kv.KV_EINVAL
    assert code(order_pagecache=3) == kv.KV_EINVAL and code(order_direct=-1) == kv.KV_EINVAL
    assert code(host_workers=65) == kv.KV_EINVAL
    assert code(span_chunks=-1) == kv.KV_EINVAL
    assert code(attn_from_extent=True) == kv.KV_EINVAL                      # only with KV_DIR_RELOAD_ATTN
    assert code(direction=9) == kv.KV_EINVAL
    assert code(layer_end=cfg.n_layers + 1) == kv.KV_ERANGE
    assert code(direction=kv.KV_DIR_RELOAD_ATTN) == kv.KV_EINVAL            # no attention arguments
    if r.n1 < r.L:
        assert code(lba_region=region[:r.region_bytes - 1]) == kv.KV_ENOSPC
        unpinned = torch.zeros(r.region_bytes, dtype=torch.uint8)
        assert code(lba_region=unpinned) == kv.KV_EINVAL                     # the LBA region must be pinned
    if r.n1 > 0:
        assert code(pageable=arena[:r.pageable_bytes - 1]) == kv.KV_ENOSPC
    if r.row_bytes % r.lba_size:
        assert code(chunk_tokens=1) == kv.KV_EALIGN


# ------------------------------------------------------------------------------------------ decode append
APPEND_CONFIGS = [
    SMALL[0],                                                    # 256 B rows in 512 B sectors: two rows per sector
    SMALL[5],                                                    # 1920 B rows in 512 B sectors: unaligned, 4-5 sectors
    W.shrink(SMALL[4], seq_len=100, pc_budget_bytes=2 * 103 * 32768),   # 32 KiB rows, 4 KiB sectors: aligned, no merge
    W.shrink(SMALL[3], len_range=(33, 200)),                     # ragged, paged, per-sequence extents, 2 KiB rows
    W.shrink(SMALL[2], seq_len=301, pc_budget_bytes=4 * 304 * 2048),    # both paths, odd length: first append merges
]


@pytest.mark.parametrize("cfg", APPEND_CONFIGS, ids=lambda c: c.name)
def test_decode_append(cfg):
    """Offload len tokens, then append three tokens one by one; after each the host bytes must equal the
    checker's pack of the longer cache.  Only the first append after the offload may read a sector back."""
    EXTRA = 3
    case = Case(cfg, "cuda", gen_device="cpu", cap_extra=EXTRA)
    r = case.ref
    FILL = 0x99
    region = pinned_bytes(r.region_bytes, FILL)
    arena = np.full(max(r.pageable_bytes, 1), FILL, dtype=np.uint8)
    kv.kv_pipeline_run(case.plan, kv.KV_DIR_OFFLOAD, 0, cfg.n_layers, case.view, region, arena, depth=2)
    lens = list(case.lens)
    row, sec = r.row_bytes, r.lba_size
    for step in range(EXTRA):
        lens = [n + 1 for n in lens]
        view = case.make_view(case.k, case.v, lens)
        st = kv.kv_append_tokens(case.plan, 0, cfg.n_layers, view, region, arena)
        want_region, want_arena = case.expected_host(fill=FILL, lens=lens)
        assert np.array_equal(region.numpy()[:r.region_bytes], want_region[:r.region_bytes]), step
        assert np.array_equal(arena[:r.pageable_bytes], want_arena[:r.pageable_bytes]), step
        nseq = len(lens) if r.per_seq else 1
        assert st.n_cmds == 2 * cfg.n_layers * nseq
        starts_inside = sum(((n - 1) * row) % sec != 0 for n in lens[:nseq])
        assert st.n_rmw_reads == (2 * cfg.n_layers * starts_inside if step == 0 else 0)
    # attention over the longer cache includes the appended tokens
    q = W.query(cfg, 0, "cpu")
    out = torch.empty((len(lens), cfg.n_q_heads, cfg.head_dim), dtype=torch.float32, device="cuda")
    ws = torch.empty(kv.kv_decode_attn_workspace(case.plan, 0, max(lens)), dtype=torch.uint8, device="cuda")
    kv.kv_decode_attn(case.plan, view, 0, q.cuda(), out, kv.KV_OUT_F32, 0, ws)
    torch.cuda.synchronize()
    K, V = case.k_cpu[0], case.v_cpu[0]
    want = o.attention(case.source(K), o.u16(K), o.u16(V), o.u16(q), cfg.dtype == W.BF16, lens, cfg.n_q_heads)
    _attn_check(out, want)
    # the next decode step's reload (storage -> staged extent images -> attention) sees the appended rows too
    k_new, v_new = case.blank_like_source()
    qd = [W.query(cfg, l, "cpu").cuda() for l in range(cfg.n_layers)]
    outs = [torch.zeros_like(out) for _ in range(cfg.n_layers)]
    kv.kv_pipeline_run(case.plan, kv.KV_DIR_RELOAD_ATTN, 0, cfg.n_layers, case.make_view(k_new, v_new, lens), region, arena,
                       depth=2, q_layers=qd, out_layers=outs, attn_from_extent=True)
    _attn_check(outs[0], want)
    # capacity is a hard bound
    with pytest.raises(kv.KVError) as e:
        kv.kv_append_tokens(case.plan, 0, cfg.n_layers, case.make_view(case.k, case.v, [n + 1 for n in lens]), region, arena)
    assert e.value.code == kv.KV_ERANGE


def test_append_after_trim_and_after_a_change_of_region():
    """The kept tail-sector image must not outlive the bytes it mirrors: after kv_plan_trim the sector reads zeros,
    and another region buffer holds whatever it holds.  offload, append, trim, append / append into a copy."""
    cfg = APPEND_CONFIGS[0]
    case = Case(cfg, "cuda", gen_device="cpu", cap_extra=2)
    r, L = case.ref, cfg.n_layers
    FILL = 0x99
    region = pinned_bytes(r.region_bytes, FILL)
    arena = np.full(max(r.pageable_bytes, 1), FILL, dtype=np.uint8)
    kv.kv_pipeline_run(case.plan, kv.KV_DIR_OFFLOAD, 0, L, case.view, region, arena, depth=2)
    lens1 = [n + 1 for n in case.lens]
    st = kv.kv_append_tokens(case.plan, 0, L, case.make_view(case.k, case.v, lens1), region, arena)
    assert (((lens1[0] - 1) * r.row_bytes) % r.lba_size != 0) == (st.n_rmw_reads > 0)
    # a second region with the same bytes: the images were taken from `region`, so the library reads this one back
    region2 = pinned_bytes(r.region_bytes, FILL)
    region2.copy_(region)
    arena2 = arena.copy()
    lens2 = [n + 1 for n in lens1]
    kv.kv_append_tokens(case.plan, 0, L, case.make_view(case.k, case.v, lens2), region2, arena2)
    want_region, want_arena = case.expected_host(fill=FILL, lens=lens2)
    assert np.array_equal(region2.numpy()[:r.region_bytes], want_region[:r.region_bytes])
    assert np.array_equal(arena2[:r.pageable_bytes], want_arena[:r.pageable_bytes])
    # trim: every extent reads zeros; the next append merges with zeros, not with the rows written before
    kv.kv_plan_trim(case.plan, 0, L, region2, arena2)
    kv.kv_append_tokens(case.plan, 0, L, case.make_view(case.k, case.v, lens2), region2, arena2)
    got_region, got_arena = region2.numpy(), arena2
    row, sec = r.row_bytes, r.lba_size
    nseq = len(lens2) if r.per_seq else 1
    for n in range(2 * L):
        buf = got_region if r.path[n] == 0 else got_arena
        ext = buf[r.ext_byte_off(n):r.ext_byte_off(n) + r.n_blocks_tensor * sec]
        want = np.zeros_like(ext)
        full = case.expected_extent(n // 2, n % 2, lens=lens2)
        for b in range(nseq):                      # only the appended row of each (sub-)extent is non-zero
            base = int(r.seq_base[b]) * sec if r.per_seq else 0
            a = base + (lens2[b] - 1) * row
            want[a:a + row] = full[a:a + row]
        assert np.array_equal(ext, want), n


def test_pipeline_waits_for_the_callers_stream():
    """KV written by kernels on a side stream, offloaded without any device-wide synchronisation: the library's
    streams must be ordered after the caller's stream (kv_pipe_opts_t.caller_stream), so the host bytes are the
    checker's pack of the final values, not of what the buffers held before."""
    cfg = W.shrink(W.CONFIGS[1], n_layers=2, seq_len=2048)
    case = Case(cfg, "cuda", gen_device="cpu")
    r, L = case.ref, cfg.n_layers
    FILL = 0x42
    region = pinned_bytes(r.region_bytes, FILL)
    arena = np.full(max(r.pageable_bytes, 1), FILL, dtype=np.uint8)
    final_k = [t.clone() for t in case.k]
    final_v = [t.clone() for t in case.v]
    for t in case.k + case.v:
        t.zero_()                                   # what a racing pack would pick up
    big = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        for _ in range(200):                        # tens of milliseconds of queued work ahead of the writes
            big.add_(1)
        for dst, src in zip(case.k + case.v, final_k + final_v):
            dst.copy_(src)
        kv.kv_pipeline_run(case.plan, kv.KV_DIR_OFFLOAD, 0, L, case.view, region, arena, depth=3)
    want_region, want_arena = case.expected_host(fill=FILL)
    assert np.array_equal(region.numpy()[:r.region_bytes], want_region[:r.region_bytes])
    assert np.array_equal(arena[:r.pageable_bytes], want_arena[:r.pageable_bytes])
    # reload into buffers that a kernel on the side stream is still filling: the unpack must come after it
    k_new, v_new = case.blank_like_source()
    with torch.cuda.stream(side):
        for _ in range(200):
            big.add_(1)
        for t in k_new + v_new:
            t.fill_(1.0)
        kv.kv_pipeline_run(case.plan, kv.KV_DIR_RELOAD, 0, L, case.make_view(k_new, v_new), region, arena, depth=3)
    for l in range(L):
        assert np.array_equal(bits(k_new[l]), bits(case.k_cpu[l])) and np.array_equal(bits(v_new[l]), bits(case.v_cpu[l]))


def test_many_sequences_span_several_launches():
    """70 ragged per-sequence sub-extents per tensor: the pack / unpack segment table holds 32 runs, so one tensor
    takes several launches; the append packs 140 rows.  Host bytes, round trip and append against the checker."""
    B, EXTRA = 70, 1
    cfg = W.KVConfig("many_segments", 777, 1, 2, 4, 64, B, W.BF16, 512, 4, 3, W.PER_SEQ, W.BHSD, 0, len_range=(1, 300))
    lens = W.seq_lens(cfg)
    lens[5] = 0
    case = Case(cfg, "cuda", gen_device="cpu", lens=lens, cap_extra=EXTRA)
    r = case.ref
    FILL = 0x6D
    region = pinned_bytes(r.region_bytes, FILL)
    arena = np.full(max(r.pageable_bytes, 1), FILL, dtype=np.uint8)
    kv.kv_pipeline_run(case.plan, kv.KV_DIR_OFFLOAD, 0, 1, case.view, region, arena, depth=3)
    want_region, _ = case.expected_host(fill=FILL)
    assert np.array_equal(region.numpy()[:r.region_bytes], want_region[:r.region_bytes])
    k_new, v_new = case.blank_like_source()
    kv.kv_pipeline_run(case.plan, kv.KV_DIR_RELOAD, 0, 1, case.make_view(k_new, v_new), region, arena, depth=3)
    _check_restored(case, k_new, v_new, [0])
    # attention straight from the staged image: 70 per-sequence base offsets, ragged lengths (full grid: B > 64)
    q = W.query(cfg, 0, "cpu")
    out = [torch.full((B, cfg.n_q_heads, cfg.head_dim), float("nan"), dtype=torch.float32, device="cuda")]
    kv.kv_pipeline_run(case.plan, kv.KV_DIR_RELOAD_ATTN, 0, 1, case.make_view(k_new, v_new), region, arena, depth=3,
                       q_layers=[q.cuda()], out_layers=out, attn_from_extent=True)
    _attn_check(out[0], case.expected_attention(0, q))
    longer = [n + 1 for n in lens]
    st = kv.kv_append_tokens(case.plan, 0, 1, case.make_view(case.k, case.v, longer), region, arena)
    assert st.n_cmds == 2 * B
    want_region, _ = case.expected_host(fill=FILL, lens=longer)
    assert np.array_equal(region.numpy()[:r.region_bytes], want_region[:r.region_bytes])


# ------------------------------------------------------------------------------------------ random shapes
def _random_configs(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        D = int(rng.choice([64, 128, 256]))
        H = int(rng.integers(1, 7))
        G = int(rng.choice([1, 2, 3, 4, 8]))
        B = int(rng.integers(1, 5))
        sector = int(rng.choice([512, 4096]))
        per_seq = bool(rng.integers(0, 2))
        paged = bool(rng.integers(0, 2))
        row = (H if per_seq else B * H) * D * 2
        unit = sector // np.gcd(sector, row)                   # fewest rows that end on a sector boundary
        chunk = int(unit * rng.integers(1, 6))
        dtype = W.F16 if rng.integers(0, 2) else W.BF16
        if per_seq:
            lo = int(rng.integers(1, 40))
            cfg = W.KVConfig(f"rand{i}", 100 + i, 2, H, H * G, D, B, dtype, sector, chunk, int(rng.integers(1, 5)),
                             W.PER_SEQ, W.PAGED if paged else W.BHSD, 0, len_range=(lo, lo + int(rng.integers(0, 300))))
        else:
            cfg = W.KVConfig(f"rand{i}", 100 + i, 2, H, H * G, D, B, dtype, sector, chunk, int(rng.integers(1, 5)),
                             W.TOKEN_MAJOR, W.PAGED if paged else W.BHSD, int(rng.integers(1, 400)))
        # one of the two layers on the page-cache path in half of the cases
        if rng.integers(0, 2):
            lens = W.seq_lens(cfg)
            nb = o.tensor_blocks(per_seq, lens, H, D, 2, sector)[0]
            cfg = W.shrink(cfg, pc_budget_bytes=2 * nb * sector)
        out.append(cfg)
    return out


@pytest.mark.parametrize("cfg", _random_configs(24, 2024), ids=lambda c: c.name)
def test_random_shapes_end_to_end(cfg):
    """Seeded random shapes (head counts, group sizes, head dims, batch, sector, chunk, both extent modes,
    both layouts, mixed paths): offload bytes, round trip and attention against the checker."""
    case = Case(cfg, "cuda", gen_device="cpu", raw=False)
    r = case.ref
    FILL = 0x42
    region = pinned_bytes(r.region_bytes, FILL)
    arena = np.full(max(r.pageable_bytes, 1), FILL, dtype=np.uint8)
    kv.kv_pipeline_run(case.plan, kv.KV_DIR_OFFLOAD, 0, cfg.n_layers, case.view, region, arena, depth=cfg.depth,
                       span_chunks=cfg.index % 3)
    want_region, want_arena = case.expected_host(fill=FILL)
    assert np.array_equal(region.numpy()[:r.region_bytes], want_region[:r.region_bytes])
    assert np.array_equal(arena[:r.pageable_bytes], want_arena[:r.pageable_bytes])
    k_new, v_new = case.blank_like_source()
    view = case.make_view(k_new, v_new)
    qs = [W.query(cfg, l, "cpu") for l in range(cfg.n_layers)]
    qd = [q.cuda() for q in qs]
    outs = [torch.full((len(case.lens), cfg.n_q_heads, cfg.head_dim), float("nan"), dtype=torch.float32, device="cuda")
            for _ in range(cfg.n_layers)]
    kv.kv_pipeline_run(case.plan, kv.KV_DIR_RELOAD_ATTN, 0, cfg.n_layers, view, region, arena, depth=cfg.depth,
                       q_layers=qd, out_layers=outs, span_chunks=(cfg.index + 1) % 3,
                       order_pagecache=cfg.index % 2, order_direct=(cfg.index // 2) % 2)
    _check_restored(case, k_new, v_new, range(cfg.n_layers))
    for l in range(cfg.n_layers):
        _attn_check(outs[l], case.expected_attention(l, qs[l]))
