"""Pins for the attention oracle (CPU only): quantiser fixture, softmax closed forms, PyTorch's fp64 attention."""
import os

import numpy as np
import pytest

from oracle import oracle_attn as oa
from workloads import attn as wa

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def test_kv_quantise_hand_worked_row():
    rows = []
    for line in open(os.path.join(GOLD, "quant_group_8bit.txt")):
        line = line.split("#")[0].split()
        if line:
            rows.append((float(line[0]), int(line[1]), float(line[2])))
    x = np.array([r[0] for r in rows], np.float32)[None, :]                 # one token-head of 12 values
    q, s, z = oa.kv_quantise(x)
    assert float(s[0]) == 0.015625 and float(z[0]) == 64.0
    assert q[0].tolist() == [r[1] for r in rows]
    assert oa.kv_dequant(q, s, z)[0].tolist() == [r[2] for r in rows]
    # constant row: scale falls back to 1, zero-point clamps
    q, s, z = oa.kv_quantise(np.full((1, 8), 3.0, np.float32))
    assert float(s[0]) == 1.0 and np.all(oa.kv_dequant(q, s, z) == 3.0)


def _random_cache(rng, B, Hkv, T, D=128):
    K = rng.standard_normal((B, Hkv, T, D)).astype(np.float16)
    V = rng.standard_normal((B, Hkv, T, D)).astype(np.float16)
    return oa.kv_quantise(K) + oa.kv_quantise(V)


def test_attn_decode_closed_forms():
    rng = np.random.default_rng(1)
    B, Hq, Hkv, T, D = 2, 4, 2, 9, 128
    Kq, Ks, Kz, Vq, Vs, Vz = _random_cache(rng, B, Hkv, T)
    lens = np.array([9, 5])
    V = oa.kv_dequant(Vq, Vs, Vz)
    # zero query: uniform weights -> mean of the cached values
    O = oa.attn_decode(np.zeros((B, Hq, D), np.float16), Kq, Ks, Kz, Vq, Vs, Vz, lens, 0.1)
    for b in range(B):
        for h in range(Hq):
            assert np.allclose(O[b, h].astype(np.float64), V[b, h // 2, :lens[b]].mean(axis=0), rtol=2e-3, atol=2e-3)
    # one cached token: the output is that token's value, whatever the query
    Q = rng.standard_normal((B, Hq, D)).astype(np.float16)
    O = oa.attn_decode(Q, Kq, Ks, Kz, Vq, Vs, Vz, np.array([1, 1]), 0.1)
    assert np.array_equal(O[1, 3], V[1, 1, 0].astype(np.float16))
    # a query aligned with one key and a huge scale: the output is that token's value
    K = oa.kv_dequant(Kq, Ks, Kz)
    Q2 = np.zeros((B, Hq, D), np.float16)
    Q2[0, 0] = K[0, 0, 4].astype(np.float16)
    O = oa.attn_decode(Q2, Kq, Ks, Kz, Vq, Vs, Vz, lens, 50.0)
    assert np.allclose(O[0, 0].astype(np.float64), V[0, 0, 4], rtol=2e-3, atol=2e-3)
    # tokens past lens are ignored
    Kq2 = Kq.copy(); Kq2[:, :, 5:] = 255
    assert np.array_equal(oa.attn_decode(Q, Kq2, Ks, Kz, Vq, Vs, Vz, lens, 0.1)[1], oa.attn_decode(Q, Kq, Ks, Kz, Vq, Vs, Vz, lens, 0.1)[1])


def test_attn_decode_against_torch_sdpa():
    import torch
    rng = np.random.default_rng(2)
    B, Hq, Hkv, T, D = 2, 8, 2, 37, 128
    Kq, Ks, Kz, Vq, Vs, Vz = _random_cache(rng, B, Hkv, T)
    Q = rng.standard_normal((B, Hq, D)).astype(np.float16)
    lens = np.array([37, 20])
    scale = 1.0 / np.sqrt(D)
    O = oa.attn_decode(Q, Kq, Ks, Kz, Vq, Vs, Vz, lens, scale).astype(np.float64)
    K = torch.from_numpy(oa.kv_dequant(Kq, Ks, Kz)).repeat_interleave(Hq // Hkv, dim=1)     # [B, Hq, T, D]
    V = torch.from_numpy(oa.kv_dequant(Vq, Vs, Vz)).repeat_interleave(Hq // Hkv, dim=1)
    for b in range(B):
        L = int(lens[b])
        ref = torch.nn.functional.scaled_dot_product_attention(
            torch.from_numpy(Q[b].astype(np.float64))[:, None, :], K[b, :, :L], V[b, :, :L], scale=scale)[:, 0].numpy()
        assert np.allclose(O[b], ref, rtol=1e-3, atol=1e-3)


def test_cache_layout_inverse_against_generator_encoder():
    """The oracle's inverse of the library's cache layout undoes the input generator's independent encoder, and single
    position codes land where the layout rule says."""
    rng = np.random.default_rng(3)
    B, Hkv, cap = 2, 3, 64
    Kq = rng.integers(0, 256, (B, Hkv, cap, 128), dtype=np.uint8)
    Vq = rng.integers(0, 256, (B, Hkv, cap, 128), dtype=np.uint8)
    s = [rng.uniform(0.001, 0.1, (B, Hkv, cap)).astype(np.float16) for _ in range(2)]
    z = [rng.integers(0, 256, (B, Hkv, cap)).astype(np.float16) for _ in range(2)]
    kbuf, vbuf, szbuf = wa.encode_cache(Kq, s[0], z[0], Vq, s[1], z[1])
    out = oa.kv_cache_unpack(kbuf, vbuf, szbuf, B, Hkv, cap)
    for a, b in zip(out, (Kq, s[0], z[0], Vq, s[1], z[1])):
        assert np.array_equal(a.view(np.uint16) if a.dtype == np.float16 else a, b.view(np.uint16) if b.dtype == np.float16 else b)
    # hand-placed bytes in block 0: value of token 21 (u = 21: hh = 1, e = 1 + 4 = 5), dimension 35 (c = 3, i = 2):
    # ((2/2)*64 + 16*1 + 3)*16 + 0*8 + 5; key of token 21 (j = 1, c = 5), dimension 83 (hh = 2, half = 1, x = 3):
    # ((1*2 + 1)*64 + 16*2 + 5)*16 + 3
    n = B * Hkv * cap * 128
    vb = np.zeros(n, np.uint8)
    vb[(64 + 16 + 3) * 16 + 5] = 77
    kb = np.zeros(n, np.uint8)
    kb[(3 * 64 + 32 + 5) * 16 + 3] = 99
    Ku, _, _, Vu, _, _ = oa.kv_cache_unpack(kb, vb, np.zeros(B * Hkv * cap * 2, np.uint32), B, Hkv, cap)
    assert Vu[0, 0, 21, 35] == 77 and Vu.sum() == 77
    assert Ku[0, 0, 21, 83] == 99 and Ku.sum() == 99


def test_kv_quantise_hand_worked_row_4bit():
    rows = []
    for line in open(os.path.join(GOLD, "kv_quant_row_4bit.txt")):
        line = line.split("#")[0].split()
        if line:
            rows.append((float(line[0]), int(line[1]), float(line[2])))
    x = np.array([r[0] for r in rows], np.float32)[None, :]
    q, s, z = oa.kv_quantise(x, bits=4)
    assert float(s[0]) == 0.125 and float(z[0]) == 8.0
    assert q[0].tolist() == [r[1] for r in rows]
    assert oa.kv_dequant(q, s, z)[0].tolist() == [r[2] for r in rows]
    # codes never leave [0, 15], also where the rounded scale makes the largest value overshoot
    q, s, z = oa.kv_quantise(np.random.default_rng(0).standard_normal((50, 128)).astype(np.float16), bits=4)
    assert q.max() == 15 and q.min() == 0 and z.max() <= 15


def test_cache_layout_inverse_4bit():
    """4-bit codes: the oracle's inverse undoes the generator's reshape-based encoder, and single hand-placed codes land
    where the layout rule says."""
    rng = np.random.default_rng(4)
    B, Hkv, cap = 2, 2, 96
    Kq = rng.integers(0, 16, (B, Hkv, cap, 128), dtype=np.uint8)
    Vq = rng.integers(0, 16, (B, Hkv, cap, 128), dtype=np.uint8)
    s = [rng.uniform(0.01, 0.5, (B, Hkv, cap)).astype(np.float16) for _ in range(2)]
    z = [rng.integers(0, 16, (B, Hkv, cap)).astype(np.float16) for _ in range(2)]
    kbuf, vbuf, szbuf = wa.encode_cache(Kq, s[0], z[0], Vq, s[1], z[1], bits=4)
    assert kbuf.size == vbuf.size == B * Hkv * cap * 64
    out = oa.kv_cache_unpack(kbuf, vbuf, szbuf, B, Hkv, cap, bits=4)
    for a, b in zip(out, (Kq, s[0], z[0], Vq, s[1], z[1])):
        assert np.array_equal(a.view(np.uint16) if a.dtype == np.float16 else a, b.view(np.uint16) if b.dtype == np.float16 else b)
    # key of token 21 (tile 1, row 5), dimension 83 = 32*2 + 8*2 + 3: word ((1*64 + 16*2 + 5)*4 + 2), element 3 ->
    # nibble 3/2 + 4*1 = 5, i.e. the high half of byte 2 of that word
    n = B * Hkv * cap * 64
    kb = np.zeros(n, np.uint8)
    kb[((64 + 32 + 5) * 4 + 2) * 4 + 2] = 0xB0
    # value of token 21 (hh = 1, element 1 + 4 = 5 -> nibble 5/2 + 4 = 6), dimension 99 = 16*6 + 3: word
    # ((6/4)*64 + 16*1 + 3)*4 + 6%4, low half of byte 3
    vb = np.zeros(n, np.uint8)
    vb[((64 + 16 + 3) * 4 + 2) * 4 + 3] = 0x0D
    Ku, _, _, Vu, _, _ = oa.kv_cache_unpack(kb, vb, np.zeros(B * Hkv * cap * 2, np.uint32), B, Hkv, cap, bits=4)
    assert Ku[0, 0, 21, 83] == 11 and Ku.sum() == 11
    assert Vu[0, 0, 21, 99] == 13 and Vu.sum() == 13


def test_attn_decode_4bit_codes_against_torch_sdpa():
    """The decode oracle on a 4-bit cache equals PyTorch's CPU attention on the dequantised keys and values."""
    import torch
    rng = np.random.default_rng(5)
    B, Hq, Hkv, T = 2, 8, 2, 40
    K = rng.standard_normal((B, Hkv, T, 128)).astype(np.float16)
    V = rng.standard_normal((B, Hkv, T, 128)).astype(np.float16)
    Q = rng.standard_normal((B, Hq, 128)).astype(np.float16)
    kq, vq = oa.kv_quantise(K, bits=4), oa.kv_quantise(V, bits=4)
    O = oa.attn_decode(Q, *kq, *vq, np.array([T, T]), 0.1)
    Kd = torch.from_numpy(oa.kv_dequant(*kq)).double().repeat_interleave(Hq // Hkv, dim=1)
    Vd = torch.from_numpy(oa.kv_dequant(*vq)).double().repeat_interleave(Hq // Hkv, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(torch.from_numpy(Q).double()[:, :, None, :], Kd, Vd, scale=0.1)
    assert np.allclose(O.astype(np.float64), ref[:, :, 0].numpy(), rtol=2e-3, atol=1e-3)


def test_attn_prefill_against_torch_sdpa_causal():
    """Whole prompt from position 0: PyTorch's fp64 attention with its causal mask on the dequantised cache."""
    import torch
    rng = np.random.default_rng(11)
    for bits in (8, 4):
        B, Hq, Hkv, T, D = 2, 4, 2, 37, 128
        K = rng.standard_normal((B, Hkv, T, D)).astype(np.float16)
        V = rng.standard_normal((B, Hkv, T, D)).astype(np.float16)
        kq, vq = oa.kv_quantise(K, bits), oa.kv_quantise(V, bits)
        Q = rng.standard_normal((B, T, Hq, D)).astype(np.float16)
        O = oa.attn_prefill(Q, *kq, *vq, np.zeros(B, np.int32), np.full(B, T), 0.09)
        Kd = torch.from_numpy(oa.kv_dequant(*kq)).repeat_interleave(Hq // Hkv, dim=1)      # [B, Hq, T, D]
        Vd = torch.from_numpy(oa.kv_dequant(*vq)).repeat_interleave(Hq // Hkv, dim=1)
        Qt = torch.from_numpy(Q.astype(np.float64)).permute(0, 2, 1, 3)                    # [B, Hq, T, D]
        ref = torch.nn.functional.scaled_dot_product_attention(Qt, Kd, Vd, is_causal=True, scale=0.09).permute(0, 2, 1, 3).numpy()
        assert np.abs(O.astype(np.float64) - ref).max() <= 1e-3 * np.abs(ref).max() + 1e-3       # one fp16 rounding apart


def test_attn_prefill_chunks_positions_and_closed_forms():
    rng = np.random.default_rng(12)
    B, Hq, Hkv, T, D = 2, 4, 2, 29, 128
    kq = oa.kv_quantise(rng.standard_normal((B, Hkv, T, D)).astype(np.float16))
    vq = oa.kv_quantise(rng.standard_normal((B, Hkv, T, D)).astype(np.float16))
    Q = rng.standard_normal((B, T, Hq, D)).astype(np.float16)
    full = oa.attn_prefill(Q, *kq, *vq, np.zeros(B, np.int32), np.full(B, T), 0.1)
    # a later chunk of the same prompt: query tokens 10 .. 17 of sequence 0, 20 .. 24 of sequence 1 (ragged counts)
    pos, cnt = np.array([10, 20]), np.array([8, 5])
    Qc = np.zeros((B, 8, Hq, D), np.float16)
    for b in range(B):
        Qc[b, :cnt[b]] = Q[b, pos[b]:pos[b] + cnt[b]]
    part = oa.attn_prefill(Qc, *kq, *vq, pos, cnt, 0.1)
    for b in range(B):
        assert np.array_equal(part[b, :cnt[b]], full[b, pos[b]:pos[b] + cnt[b]])
        assert not part[b, cnt[b]:].any()                                            # rows past the count stay zero
    # the last token of a chunk is a decoding step over the same context
    dec = oa.attn_decode(Q[:, T - 1], *kq, *vq, np.full(B, T), 0.1)
    assert np.array_equal(dec, full[:, T - 1])
    # the first prompt token sees only itself: its output is its own value row
    V = oa.kv_dequant(*vq)
    assert np.array_equal(full[1, 0, 3], V[1, 1, 0].astype(np.float16))
    # zero queries: uniform weights over the causal prefix -> running mean of the values
    O0 = oa.attn_prefill(np.zeros_like(Q), *kq, *vq, np.zeros(B, np.int32), np.full(B, T), 0.1)
    for i in (0, 4, T - 1):
        assert np.allclose(O0[0, i, 2].astype(np.float64), V[0, 1, :i + 1].mean(axis=0), rtol=2e-3, atol=2e-3)
    # causality: changing later cache entries leaves earlier outputs alone
    kq2 = (kq[0].copy(), kq[1], kq[2]); kq2[0][:, :, 15:] = 0
    early = oa.attn_prefill(Q, *kq2, *vq, np.zeros(B, np.int32), np.full(B, T), 0.1)
    assert np.array_equal(early[:, :15], full[:, :15]) and not np.array_equal(early[:, 15:], full[:, 15:])
