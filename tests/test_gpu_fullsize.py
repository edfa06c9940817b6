"""GPU parity at the full sizes of the evaluation configs, in the launch configuration bench.py times
(whole-tensor kernel spans, the config's chunk size and depth, default copy engines).

Every tensor of every configuration is compared with the checker byte for byte: one extent image at a time is
packed by the checker from a CPU copy of the same bits and compared with its slice of the region / arena (payload and
zero pad), so the final host bytes equal the checker's pack of the whole cache.  Also:
  * every layer comes back bit for bit after the reload (reload(offload(x)) == x),
  * bytes outside all extents (the hole below lba_start) keep their fill pattern,
  * decode attention is compared with the fp64 checker on every layer of the 4K configuration and on the first and
    last layer of the others (the checker needs seconds per layer there).
Inputs are generated on the GPU from the seeded generator; the checker sees copies of the same bits.
"""
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
FILL = 0xC3


@pytest.mark.parametrize("idx", [1, 2, 3, 4], ids=lambda i: W.CONFIGS[i].name)
def test_full_size_offload_reload_attention(idx):
    torch.cuda.set_device(0)
    cfg = W.CONFIGS[idx]
    print(f"full-size case {cfg.name} seed {cfg.seed}", flush=True)
    case = Case(cfg, "cuda", keep_cpu=False)
    r, L = case.ref, cfg.n_layers
    region = pinned_bytes(r.region_bytes, FILL)
    arena = np.full(max(r.pageable_bytes, 1), FILL, dtype=np.uint8)

    st = kv.kv_pipeline_run(case.plan, kv.KV_DIR_OFFLOAD, 0, L, case.view, region, arena, depth=cfg.depth)
    assert st.max_in_flight <= cfg.depth
    assert st.bytes_direct == r.direct_blocks * r.lba_size and st.bytes_pagecache == r.pageable_bytes

    # every tensor against the checker, byte for byte (payload and zero pad), one extent image at a time
    region_np = region.numpy()
    ext_bytes = r.n_blocks_tensor * r.lba_size
    for layer in range(L):
        for kind in (0, 1):
            t_cpu = (case.k if kind == 0 else case.v)[layer].cpu()
            want = case.expected_extent(layer, kind, t_cpu)
            n = 2 * layer + kind
            buf = region_np if r.path[n] == 0 else arena
            off = r.ext_byte_off(n)
            assert np.array_equal(buf[off:off + ext_bytes], want), (layer, kind)
        if layer % 8 == 7 or layer == L - 1:
            print(f"  offloaded bytes of layers 0..{layer} equal the checker's", flush=True)
    # the extents tile the host buffers exactly: nothing after the last one
    assert r.region_bytes == region_np.size or r.region_bytes == 0
    # the hole below the first LBA is never written
    assert (region_np[:cfg.lba_start * cfg.sector_bytes] == FILL).all()

    # reload + attention; every layer must come back bit for bit
    k_new, v_new = case.blank_like_source()
    view = case.make_view(k_new, v_new)
    qd = [W.query(cfg, l, "cuda") for l in range(L)]
    outs = [torch.full((cfg.batch, cfg.n_q_heads, cfg.head_dim), float("nan"), dtype=torch.float32, device="cuda")
            for _ in range(L)]
    st = kv.kv_pipeline_run(case.plan, kv.KV_DIR_RELOAD_ATTN, 0, L, view, region, arena, depth=cfg.depth,
                            q_layers=qd, out_layers=outs)
    assert st.max_in_flight <= cfg.depth
    if case.paged:
        # slots past a sequence's length are not part of the cache: compare valid tokens only
        bt = cfg.block_tokens
        valid = torch.zeros((case.n_pool, bt), dtype=torch.bool)
        table = case.table_cpu
        for b, n in enumerate(case.lens):
            nb = -(-n // bt)
            valid[table[b, :nb].long()] = True
            if n % bt:
                valid[table[b, nb - 1].long(), n % bt:] = False
        m = valid.cuda()[:, None, :, None]
        for l in range(L):
            for a, b_ in ((case.k[l], k_new[l]), (case.v[l], v_new[l])):
                assert torch.equal(torch.where(m, a.view(torch.int16), 0), torch.where(m, b_.view(torch.int16), 0)), l
    else:
        for l in range(L):
            assert torch.equal(case.k[l].view(torch.int16), k_new[l].view(torch.int16)), l
            assert torch.equal(case.v[l].view(torch.int16), v_new[l].view(torch.int16)), l

    for layer in (range(L) if idx == 1 else sorted({0, L - 1})):
        K, V, q = case.k[layer].cpu(), case.v[layer].cpu(), qd[layer].cpu()
        want = o.attention(case.source(K), o.u16(K), o.u16(V), o.u16(q), cfg.dtype == W.BF16, case.lens, cfg.n_q_heads)
        got = outs[layer].double().cpu().numpy()
        err, scale = np.abs(got - want).max(), np.abs(want).max()
        print(f"  layer {layer}: attention max abs err {err:.3e}, reference max {scale:.3e}", flush=True)
        assert err <= ATTN_ATOL and err <= ATTN_REL_OF_MAX * scale, (layer, err, scale)
    for l in range(L):
        assert torch.isfinite(outs[l]).all()


def test_tensor_larger_than_4_gib():
    """Maximum sizes: one K tensor of 4.58 GiB (byte offsets beyond 2^32, element offsets of the last sequence
    beyond 2^31).  Whole-tensor pack against the checker byte for byte, unpack back bit for bit, and decode
    attention of a long last sequence against the fp64 checker."""
    torch.cuda.set_device(0)
    H, Hq, D, B, S = 8, 32, 128, 8, 300000
    print(f"large-tensor case H={H} D={D} B={B} S={S}", flush=True)
    cfg = W.KVConfig("large_tensor", 4242, 1, H, Hq, D, B, W.F16, 4096, 1024, 3, W.TOKEN_MAJOR, W.BHSD, S)
    lens = [S] * B
    plan = kv.kv_layout_plan(1, H, Hq, D, lens, kv.KV_F16, 4096, 1024, kv.KV_TOKEN_MAJOR, 0, kv.KV_UNBOUNDED, 0,
                             kv.KV_UNBOUNDED)
    ref = o.layout_plan(1, H, Hq, D, lens, 2, 4096, False, 0, 0)
    g = torch.Generator(device="cuda").manual_seed(cfg.seed)
    K = torch.randn((B, H, S, D), dtype=torch.float16, device="cuda", generator=g)
    V = torch.randn((B, H, S, D), dtype=torch.float16, device="cuda", generator=g)
    nbytes = int(plan.info.tensor_blocks) * 4096
    assert nbytes == B * H * S * D * 2 > (1 << 32)
    lens_dev = torch.tensor(lens, dtype=torch.int32, device="cuda")
    view = kv.bhsd_view([K], [V], lens, lens_dev)

    img = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    kv.kv_offload_pack(plan, 0, kv.KV_K, view, kv.KV_SEQ_ALL, 0, 0, img)
    torch.cuda.synchronize()
    K_cpu = K.cpu()
    want = np.full(nbytes, 0xEE, dtype=np.uint8)
    o.pack(o.bhsd_source(K_cpu.shape), o.u16(K_cpu), False, lens, ref.seq_base, ref.n_blocks_tensor, 4096, want)
    got = img.cpu().numpy()
    assert np.array_equal(got, want)
    del got, want

    k_new = torch.full(K.shape, 0x7E7E, dtype=torch.int16, device="cuda").view(torch.float16)
    kv.kv_reload_unpack(plan, 0, kv.KV_K, img, kv.bhsd_view([k_new], [V], lens, lens_dev), kv.KV_SEQ_ALL, 0, 0)
    torch.cuda.synchronize()
    assert torch.equal(k_new.view(torch.int16), K.view(torch.int16))
    del k_new, img

    # the last sequence starts 7/8 of the way into the buffers: element offsets beyond 2^31
    lens2 = [1] * (B - 1) + [50000]
    view2 = kv.bhsd_view([K], [V], lens2, torch.tensor(lens2, dtype=torch.int32, device="cuda"))
    q = torch.randn((B, Hq, D), dtype=torch.float16, device="cuda", generator=g)
    out = torch.full((B, Hq, D), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(kv.kv_decode_attn_workspace(plan, 0, max(lens2)), dtype=torch.uint8, device="cuda")
    kv.kv_decode_attn(plan, view2, 0, q, out, kv.KV_OUT_F32, 0, ws)
    torch.cuda.synchronize()
    V_cpu = V.cpu()
    ref_out = o.attention(o.bhsd_source(K_cpu.shape), o.u16(K_cpu), o.u16(V_cpu), o.u16(q.cpu()), False, lens2, Hq)
    err = np.abs(out.double().cpu().numpy() - ref_out).max()
    scale = np.abs(ref_out[-1]).max()
    print(f"  attention max abs err {err:.3e}, reference max of the long sequence {scale:.3e}", flush=True)
    assert err <= ATTN_ATOL and np.abs(out[-1].double().cpu().numpy() - ref_out[-1]).max() <= ATTN_REL_OF_MAX * scale
    # a single-token sequence attends to its only token: the output is that V row
    assert torch.equal(out[0, 0], V[0, 0, 0].float())
