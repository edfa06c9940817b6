"""Pins for the CPU checker's decode attention (unblocked softmax(q K^T / sqrt(D)) V in double).

Closed forms (constant keys, one token, a two-key logistic), the head-group map, a library
softmax, a blocked running-max formulation, and exact 16-bit decoding over every bit pattern.
"""
import numpy as np
import pytest
import torch

from oracle import kv_oracle as o


def _bits(t: torch.Tensor) -> np.ndarray:
    return o.u16(t)


def _case(B, H, Hq, S, D, dtype, seed):
    g = torch.Generator().manual_seed(seed)
    K = torch.randn(B, H, S, D, generator=g).to(dtype)
    V = torch.randn(B, H, S, D, generator=g).to(dtype)
    q = torch.randn(B, Hq, D, generator=g).to(dtype)
    return K, V, q


def _run(K, V, q, lens=None):
    B, H, S, D = K.shape
    lens = [S] * B if lens is None else lens
    return o.attention(o.bhsd_source(K.shape), _bits(K), _bits(V), _bits(q),
                       K.dtype == torch.bfloat16, lens, q.shape[1])


def test_decode_f16_all_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    got = o.decode16(bits, False)
    want = bits.view(np.float16).astype(np.float64)
    assert np.array_equal(np.isnan(got), np.isnan(want))
    m = ~np.isnan(want)
    assert np.array_equal(got[m], want[m])
    assert np.array_equal(np.signbit(got[m]), np.signbit(want[m]))


def test_decode_bf16_all_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    got = o.decode16(bits, True)
    want = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(np.isnan(got), np.isnan(want))
    m = ~np.isnan(want)
    assert np.array_equal(got[m], want[m])


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
def test_constant_keys_give_mean_of_values(dtype):
    K, V, q = _case(2, 2, 4, 37, 64, dtype, 1)
    K[:] = K[:, :, :1, :]                                      # every key identical -> uniform weights
    out = _run(K, V, q)
    want = V.double().mean(dim=2)                              # [B,H,D]
    for hq in range(4):
        assert np.allclose(out[:, hq], want[:, hq // 2].numpy(), rtol=0, atol=1e-13)


def test_single_token_returns_its_value():
    K, V, q = _case(3, 2, 2, 9, 32, torch.float16, 2)
    out = _run(K, V, q, lens=[1, 1, 1])
    assert np.array_equal(out, V[:, :, 0, :].double().numpy())


def test_zero_length_gives_zeros_and_ragged_lengths():
    K, V, q = _case(2, 1, 1, 20, 32, torch.float16, 3)
    out = _run(K, V, q, lens=[0, 7])
    assert not out[0].any()
    ref = _run(K[1:, :, :7].contiguous(), V[1:, :, :7].contiguous(), q[1:])
    assert np.array_equal(out[1:], ref)                        # tokens past len_b are not attended


def test_dominant_key_selects_its_value():
    K, V, q = _case(1, 1, 1, 50, 64, torch.float16, 4)
    q[:] = 0
    q[0, 0, 0] = 16.0
    K[0, 0, :, 0] = 0
    K[0, 0, 23, 0] = 64.0                                      # score 16*64/8 = 128 above all others
    out = _run(K, V, q)
    assert np.allclose(out[0, 0], V[0, 0, 23].double().numpy(), atol=1e-12)


def test_two_key_logistic_fixes_scale():
    """q = a e_0, K_0 = c e_0, K_1 = 0: p_0 = 1 / (1 + exp(-a c / sqrt(D))).  Pins the 1/sqrt(D) scale
    (a missing or squared scale changes p_0) and the sign of the exponent."""
    for D, a, c in ((64, 2.0, 3.0), (128, 4.0, 1.5), (256, 8.0, 2.0)):
        K = torch.zeros(1, 1, 2, D, dtype=torch.float16)
        V = torch.zeros(1, 1, 2, D, dtype=torch.float16)
        q = torch.zeros(1, 1, D, dtype=torch.float16)
        q[0, 0, 0], K[0, 0, 0, 0] = a, c
        V[0, 0, 0, 0], V[0, 0, 1, 1] = 1.0, 1.0                # out[0] = p_0, out[1] = p_1
        out = _run(K, V, q)
        p0 = 1.0 / (1.0 + np.exp(-a * c / np.sqrt(D)))
        assert abs(out[0, 0, 0] - p0) < 1e-15 and abs(out[0, 0, 1] - (1 - p0)) < 1e-15


def test_group_map_is_integer_division():
    """V of kv head h is the constant h+1, so every output element of query head hq is hq // G + 1."""
    B, H, Hq, S, D = 1, 4, 12, 10, 32
    K, V, q = _case(B, H, Hq, S, D, torch.float16, 5)
    for h in range(H):
        V[:, h] = float(h + 1)
    out = _run(K, V, q)
    for hq in range(Hq):
        assert np.allclose(out[0, hq], hq // 3 + 1, atol=1e-13)


def test_identical_queries_in_a_group_agree():
    K, V, q = _case(2, 2, 8, 33, 64, torch.bfloat16, 6)
    q[:, 1] = q[:, 0]
    q[:, 3] = q[:, 0]
    out = _run(K, V, q)
    assert np.array_equal(out[:, 0], out[:, 1]) and np.array_equal(out[:, 0], out[:, 3])
    assert not np.array_equal(out[:, 0], out[:, 4])            # other kv head


@pytest.mark.parametrize("dtype,B,H,Hq,S,D", [(torch.float16, 2, 2, 4, 100, 64), (torch.bfloat16, 1, 2, 8, 300, 128)])
def test_against_library_softmax(dtype, B, H, Hq, S, D):
    K, V, q = _case(B, H, Hq, S, D, dtype, 7)
    out = _run(K, V, q)
    G = Hq // H
    Kd = K.double().repeat_interleave(G, dim=1)                # [B,Hq,S,D]
    Vd = V.double().repeat_interleave(G, dim=1)
    s = torch.einsum("bhd,bhsd->bhs", q.double(), Kd) / np.sqrt(D)
    want = torch.einsum("bhs,bhsd->bhd", torch.softmax(s, dim=-1), Vd).numpy()
    assert np.allclose(out, want, rtol=0, atol=1e-13)


def test_blocked_running_max_formulation_agrees():
    """Splitting the tokens into ranges with (m, l, acc) partials and merging them is the same function."""
    K, V, q = _case(1, 2, 4, 257, 64, torch.float16, 8)
    out = _run(K, V, q)
    Kd, Vd, qd = K.double().numpy(), V.double().numpy(), q.double().numpy()
    for hq in range(4):
        h = hq // 2
        parts = []
        for t0 in range(0, 257, 64):
            s = Kd[0, h, t0:t0 + 64] @ qd[0, hq] / 8.0
            m = s.max()
            p = np.exp(s - m)
            parts.append((m, p.sum(), p @ Vd[0, h, t0:t0 + 64]))
        M = max(m for m, _, _ in parts)
        num = sum(np.exp(m - M) * acc for m, _, acc in parts)
        den = sum(np.exp(m - M) * l for m, l, _ in parts)
        assert np.allclose(out[0, hq], num / den, rtol=0, atol=1e-12)


def test_paged_source_attention_equals_gathered():
    H, D, bt, lens = 2, 32, 16, [40, 9]
    rng = np.random.default_rng(0)
    per = [-(-n // bt) for n in lens]
    perm = rng.permutation(sum(per))
    table = np.full((2, max(per)), -1, dtype=np.int32)
    table[0, :per[0]] = perm[:per[0]]
    table[1, :per[1]] = perm[per[0]:]
    g = torch.Generator().manual_seed(9)
    Kp = torch.randn(sum(per), H, bt, D, generator=g).half()
    Vp = torch.randn(sum(per), H, bt, D, generator=g).half()
    q = torch.randn(2, 4, D, generator=g).half()
    src = o.Source(H=H, D=D, paged=True, block_table=table, block_tokens=bt)
    out = o.attention(src, _bits(Kp), _bits(Vp), _bits(q), False, lens, 4)
    for b, n in enumerate(lens):
        Kb = torch.stack([Kp[table[b, s // bt], :, s % bt] for s in range(n)], dim=1)[None]   # [1,H,n,D]
        Vb = torch.stack([Vp[table[b, s // bt], :, s % bt] for s in range(n)], dim=1)[None]
        ref = _run(Kb.contiguous(), Vb.contiguous(), q[b:b + 1])
        assert np.array_equal(out[b], ref[0])
