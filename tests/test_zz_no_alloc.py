"""The decode-attention entry point that allocates nothing (for callers that cannot call hipMalloc):
its output must equal kv_decode_attn's on the same inputs, on two calls in a row, the second smaller,
since both calls share one static device array that keeps the first call's partials."""
import numpy as np
import pytest
import torch

from paper_2604_26557_amd import binding as kv
from paper_2604_26557_amd import workloads as W
from kvcase import Case

pytestmark = pytest.mark.gpu

ATTN_ATOL = 2e-3
ATTN_REL_OF_MAX = 1e-2


def _both(case, layer, lens, q):
    cfg = case.cfg
    view = case.make_view(case.k, case.v, lens)
    shape = (cfg.batch, cfg.n_q_heads, cfg.head_dim)
    want = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
    got = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(kv.kv_decode_attn_workspace(case.plan, 0, max(lens)), dtype=torch.uint8, device="cuda")
    kv.kv_decode_attn(case.plan, view, layer, q, want, kv.KV_OUT_F32, 0, ws)
    kv.kv_decode_attn_static(case.plan, view, layer, q, got, kv.KV_OUT_F32, 0)
    torch.cuda.synchronize()
    return want.double().cpu().numpy(), got.double().cpu().numpy()


@pytest.mark.parametrize("idx,small", [(2, dict(n_layers=2, seq_len=4224)),
                                        (3, dict(n_layers=2, batch=3, len_range=(100, 700)))],
                         ids=["bhsd_bf16", "ragged_paged_f16"])
def test_static_scratch_entry_matches_workspace_entry(idx, small):
    torch.cuda.set_device(0)
    cfg = W.shrink(W.CONFIGS[idx], **small)
    print(f"no-alloc case {cfg.name} seed {cfg.seed}", flush=True)
    case = Case(cfg, "cuda")
    q = [W.query(cfg, l, "cuda") for l in range(cfg.n_layers)]
    # first call: full lengths; second call: about a third of them (fewer splits, so most of the array
    # still holds the first call's partials)
    for layer, lens in ((0, case.lens), (1, [max(1, n // 3) for n in case.lens])):
        want, got = _both(case, layer, lens, q[layer])
        assert np.isfinite(got).all()
        err, scale = np.abs(got - want).max(), np.abs(want).max()
        assert err <= ATTN_ATOL and err <= ATTN_REL_OF_MAX * scale, (layer, err, scale)
        # and against the fp64 checker (the CPU copies hold all rows; only the first `lens` are attended)
        from oracle import kv_oracle as o
        K, V = case.k_cpu[layer], case.v_cpu[layer]
        ref = o.attention(case.source(K), o.u16(K), o.u16(V), o.u16(q[layer].cpu()), cfg.dtype == W.BF16, lens,
                          cfg.n_q_heads)
        err = np.abs(got - ref).max()
        assert err <= ATTN_ATOL and err <= ATTN_REL_OF_MAX * np.abs(ref).max(), (layer, err)


def test_static_scratch_entry_rejects_oversized_request():
    torch.cuda.set_device(0)
    cfg = W.shrink(W.CONFIGS[2], n_layers=1, seq_len=2048)
    case = Case(cfg, "cuda")
    q = W.query(cfg, 0, "cuda")
    out = torch.zeros((cfg.batch, cfg.n_q_heads, cfg.head_dim), dtype=torch.float32, device="cuda")
    per_split = cfg.batch * cfg.n_q_heads * (cfg.head_dim + 2) * 4
    too_many = kv.KV_ATTN_SCRATCH_BYTES // per_split + 1
    assert too_many <= 1024
    with pytest.raises(kv.KVError) as e:
        kv.kv_decode_attn_static(case.plan, case.view, 0, q, out, kv.KV_OUT_F32, too_many)
    assert e.value.code == kv.KV_ENOSPC
    kv.kv_decode_attn_static(case.plan, case.view, 0, q, out, kv.KV_OUT_F32, too_many - 1)   # the largest that fits
    torch.cuda.synchronize()


def test_static_scratch_entry_under_graph_capture():
    """What the entry point is for: the attention launches of several layers recorded in one HIP graph.  The graph is
    replayed several times, with eager launches and synchronisations of the same calls in between, and every replay
    is checked against the eager result (the split partials of all layers pass through the one static array; results
    may differ from run to run by rounding, since the wavefronts claim their steps on demand)."""
    torch.cuda.set_device(0)
    cfg = W.shrink(W.CONFIGS[3], n_layers=3, batch=3, len_range=(300, 1500))
    print(f"graph-capture case {cfg.name} seed {cfg.seed}", flush=True)
    case = Case(cfg, "cuda")
    L = cfg.n_layers
    q = [W.query(cfg, l, "cuda") for l in range(L)]
    outs = [torch.zeros((cfg.batch, cfg.n_q_heads, cfg.head_dim), dtype=torch.float32, device="cuda") for _ in range(L)]

    def run():
        for l in range(L):
            kv.kv_decode_attn_static(case.plan, case.view, l, q[l], outs[l], kv.KV_OUT_F32, 0)

    run()                                   # eager: resolves the static array before anything is captured
    torch.cuda.synchronize()
    want = [o.double().cpu().numpy() for o in outs]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run()
    torch.cuda.synchronize()
    for replay in range(4):
        for o in outs:
            o.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for l in range(L):
            got = outs[l].double().cpu().numpy()
            assert np.isfinite(got).all(), (replay, l)
            err, scale = np.abs(got - want[l]).max(), np.abs(want[l]).max()
            assert err <= 1e-5 * scale, (replay, l, err, scale)
        run()                               # the program's own eager work between replays
        torch.cuda.synchronize()
