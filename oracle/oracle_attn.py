"""Reference (oracle) for attention over a quantised KV cache: one decoding step, and a chunk of prompt tokens.  TEST INFRASTRUCTURE ONLY: imported by tests/,
__graft_entry__.smoke() and bench.py's cpu_baseline leg, never by the GPU library or its binding.

Plain numpy, fp64 throughout, one loop per (sequence, head); no blocking, no online softmax, no fused dequantisation.

What it follows (paper Sec. 3.3 "attention pipeline design", Sec. 4.2, Sec. 4.4): at a decoding step every query head
attends over the keys and values cached for its sequence; the cache holds low-bit integer codes that are dequantised to
floating point before S = Q K^T and O = P V.  The paper does not state the granularity of the cache quantisation; the
reading taken here is the usual one for such caches: one asymmetric scale / zero-point pair per token and KV head over the
head dimension, x^ = (q - z) * s, with the same rounding rules as the weight recipe (s rounded to fp16 first, round half
to even, clamp to the code range).

Parity status: every function is pinned in tests/test_oracle_attn_pins.py (hand-worked quantiser group, softmax closed
forms, PyTorch's CPU scaled_dot_product_attention in fp64, brute-force layout inverse).  Nothing is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

HEAD_DIM = 128


def kv_quantise(x: np.ndarray, bits: int = 8):
    """x [..., D] (fp16 or fp32 values) -> (q uint8 [..., D], s float16 [...], z float16 [...]).
    Per last axis: s = fp16((max - min) / (2^bits - 1)) (1 if that is 0 or not finite), z = clip(rint(-min / s), 0, qmax),
    q = clip(rint(x / s) + z, 0, qmax); fp32 arithmetic with the rounded s."""
    qmax = np.float32((1 << bits) - 1)
    x = np.asarray(x, dtype=np.float32)
    mn = x.min(axis=-1)
    mx = x.max(axis=-1)
    s16 = ((mx - mn) / qmax).astype(np.float32).astype(np.float16)
    sf = s16.astype(np.float32)
    bad = ~(sf > 0) | np.isinf(sf)
    sf = np.where(bad, np.float32(1.0), sf).astype(np.float32)
    s16 = np.where(bad, np.float16(1.0), s16).astype(np.float16)
    z = np.clip(np.rint(-mn / sf), 0, qmax).astype(np.float32)
    q = np.clip(np.rint(x / sf[..., None]) + z[..., None], 0, qmax)
    return q.astype(np.uint8), s16, z.astype(np.float16)


def kv_dequant(q: np.ndarray, s: np.ndarray, z: np.ndarray) -> np.ndarray:
    """(q - z) * s in fp64, exact."""
    return (q.astype(np.float64) - z.astype(np.float64)[..., None]) * s.astype(np.float64)[..., None]


def attn_decode(Q, Kq, Ks, Kz, Vq, Vs, Vz, lens, scale: float) -> np.ndarray:
    """One decoding step.  Q float16 [B, Hq, D]; K/V codes uint8 [B, Hkv, T, D] with scale / zero float16 [B, Hkv, T];
    lens int [B] (tokens cached per sequence, 1..T); query head h uses KV head h // (Hq / Hkv).
    O[b, h] = softmax(scale * K^ q) V^ over the first lens[b] tokens, computed in fp64, rounded once to float16."""
    Q = np.asarray(Q)
    B, Hq, D = Q.shape
    Hkv = Kq.shape[1]
    G = Hq // Hkv
    O = np.zeros((B, Hq, D), np.float16)
    for b in range(B):
        L = int(lens[b])
        for h in range(Hq):
            kv = h // G
            K = kv_dequant(Kq[b, kv, :L], Ks[b, kv, :L], Kz[b, kv, :L])          # [L, D]
            V = kv_dequant(Vq[b, kv, :L], Vs[b, kv, :L], Vz[b, kv, :L])
            sc = (K @ Q[b, h].astype(np.float64)) * float(scale)                # [L]
            e = np.exp(sc - sc.max())
            p = e / e.sum()
            O[b, h] = (p @ V).astype(np.float16)
    return O


def attn_prefill(Q, Kq, Ks, Kz, Vq, Vs, Vz, positions, counts, scale: float) -> np.ndarray:
    """Attention of a chunk of prompt tokens over the quantised cache (paper Sec. 3.3: the attention pipeline serves the
    prefill phase as it serves decoding; the evaluation of Sec. 5.3 times both).  Q float16 [B, n, Hq, D]: query token i of
    sequence b sits at cache position positions[b] + i, its own key and value already cached, and attends causally over
    cache tokens 0 .. positions[b] + i.  counts int [B]: query tokens each sequence really has (rows past that stay 0).
    O[b, i, h] = softmax(scale * K^[:L] q) V^[:L],  L = positions[b] + i + 1, in fp64, rounded once to float16.
    The definition written out, one query row at a time: no mask matrix, no blocking, no online softmax."""
    Q = np.asarray(Q)
    B, n, Hq, D = Q.shape
    Hkv = Kq.shape[1]
    G = Hq // Hkv
    O = np.zeros((B, n, Hq, D), np.float16)
    for b in range(B):
        for i in range(min(n, int(counts[b]))):
            L = int(positions[b]) + i + 1
            for h in range(Hq):
                kv = h // G
                K = kv_dequant(Kq[b, kv, :L], Ks[b, kv, :L], Kz[b, kv, :L])          # [L, D]
                V = kv_dequant(Vq[b, kv, :L], Vs[b, kv, :L], Vz[b, kv, :L])
                sc = (K @ Q[b, i, h].astype(np.float64)) * float(scale)
                e = np.exp(sc - sc.max())
                p = e / e.sum()
                O[b, i, h] = (p @ V).astype(np.float16)
    return O


def kv_cache_unpack(kbuf, vbuf, szbuf, B: int, Hkv: int, cap: int, bits: int = 8):
    """Inverse of the library's cache layout, written from its specification.  Codes live in blocks of 32 tokens x 128
    dimensions, block index (b*Hkv + h)*(cap/32) + t/32, token u = t % 32 inside it.
    8-bit codes (4096-byte blocks):
      K block:  byte ((j*2 + half)*64 + 16*hh + c)*16 + x   for dimension d,  j = u / 16, c = u % 16, hh = d / 32,
                half = (d % 32) / 16, x = d % 16
      V block:  byte ((i/2)*64 + 16*hh + c)*16 + (i % 2)*8 + e   for dimension d,  c = d % 16, i = d / 16,
                hh = (u % 16) / 4, e = u % 4 + 4*(u / 16)
    4-bit codes (2048-byte blocks of little-endian 32-bit words; the code of operand element e sits in bits 4p .. 4p+3
    with p = e/2 + 4*(e % 2)):
      K block:  word ((u/16)*64 + 16*(d/32) + u%16)*4 + (d%32)/8,  element e = d % 8
      V block:  word ((i/4)*64 + 16*hh + c)*4 + i%4,  i = d / 16, c = d % 16, hh = (u % 16) / 4,
                element e = u % 4 + 4*(u / 16)
    scale/zero: u32 words, word ((b*Hkv + h)*cap + t)*2 + {0: K, 1: V} = scale bits | zero bits << 16
    -> (Kq, Ks, Kz, Vq, Vs, Vz) in the plain [B, Hkv, cap, (D)] arrangement."""
    if bits == 4:
        return _kv_cache_unpack4(kbuf, vbuf, szbuf, B, Hkv, cap)
    assert bits == 8 and cap % 32 == 0
    D = HEAD_DIM
    kbuf = np.asarray(kbuf, np.uint8).reshape(-1)
    vbuf = np.asarray(vbuf, np.uint8).reshape(-1)
    szbuf = np.asarray(szbuf, np.uint32).reshape(-1)
    Kq = np.empty((B, Hkv, cap, D), np.uint8)
    Vq = np.empty((B, Hkv, cap, D), np.uint8)
    bh = np.arange(B)[:, None] * Hkv + np.arange(Hkv)[None, :]
    for t in range(cap):
        u = t % 32
        blk = bh * (cap // 32) + t // 32
        for d in range(D):
            koff = (((u // 16) * 2 + (d % 32) // 16) * 64 + 16 * (d // 32) + u % 16) * 16 + d % 16
            Kq[:, :, t, d] = kbuf[blk * 4096 + koff]
            i, c = d // 16, d % 16
            hh, e = (u % 16) // 4, u % 4 + 4 * (u // 16)
            voff = ((i // 2) * 64 + 16 * hh + c) * 16 + (i % 2) * 8 + e
            Vq[:, :, t, d] = vbuf[blk * 4096 + voff]
    sz = szbuf.reshape(B, Hkv, cap, 2)
    s = (sz & 0xFFFF).astype(np.uint16).view(np.float16)
    z = (sz >> 16).astype(np.uint16).view(np.float16)
    return Kq, s[..., 0], z[..., 0], Vq, s[..., 1], z[..., 1]


def _kv_cache_unpack4(kbuf, vbuf, szbuf, B: int, Hkv: int, cap: int):
    assert cap % 32 == 0
    D = HEAD_DIM
    kw = np.asarray(kbuf, np.uint8).reshape(-1).view("<u4")
    vw = np.asarray(vbuf, np.uint8).reshape(-1).view("<u4")
    szbuf = np.asarray(szbuf, np.uint32).reshape(-1)
    Kq = np.empty((B, Hkv, cap, D), np.uint8)
    Vq = np.empty((B, Hkv, cap, D), np.uint8)
    bh = np.arange(B)[:, None] * Hkv + np.arange(Hkv)[None, :]
    for t in range(cap):
        u = t % 32
        blk = bh * (cap // 32) + t // 32                       # 512 words per block
        for d in range(D):
            e = d % 8
            word = ((u // 16) * 64 + 16 * (d // 32) + u % 16) * 4 + (d % 32) // 8
            Kq[:, :, t, d] = (kw[blk * 512 + word] >> (4 * (e // 2 + 4 * (e % 2)))) & 15
            i, c = d // 16, d % 16
            hh, e = (u % 16) // 4, u % 4 + 4 * (u // 16)
            word = ((i // 4) * 64 + 16 * hh + c) * 4 + i % 4
            Vq[:, :, t, d] = (vw[blk * 512 + word] >> (4 * (e // 2 + 4 * (e % 2)))) & 15
    sz = szbuf.reshape(B, Hkv, cap, 2)
    s = (sz & 0xFFFF).astype(np.uint16).view(np.float16)
    z = (sz >> 16).astype(np.uint16).view(np.float16)
    return Kq, s[..., 0], z[..., 0], Vq, s[..., 1], z[..., 1]
