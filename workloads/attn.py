"""Seeded synthetic inputs for decode attention over a quantised KV cache: Gaussian queries, keys and values in the
shapes of the grouped-query-attention models the paper evaluates (head dimension 128), per-sequence context lengths, and
the byte-level encoder of the cache layout the library reads (an input *format*, no arithmetic of the method).

The cache layout (8-bit codes), per sequence b and KV head h, capacity cap tokens (a multiple of 32): codes in blocks of
32 tokens x 128 dimensions (4096 bytes each, block (b*Hkv + h)*(cap/32) + t/32), token u = t % 32:
  K block   byte ((j*2 + half)*64 + 16*hh + c)*16 + x,  j = u / 16, c = u % 16, hh = d / 32, half = (d % 32) / 16, x = d % 16
  V block   byte ((i/2)*64 + 16*hh + c)*16 + (i % 2)*8 + e,  c = d % 16, i = d / 16, hh = (u % 16) / 4, e = u % 4 + 4*(u / 16)
  scale/zero words  u32 [(b*Hkv + h)*cap + t][2]: K pair, V pair; scale bits | zero bits << 16
"""
from __future__ import annotations

import numpy as np


def draw(B: int, Hq: int, Hkv: int, T: int, seed: int, D: int = 128, min_len: int = 1):
    """-> Q float16 [B,Hq,D], K, V float16 [B,Hkv,T,D], lens int32 [B] (uniform in [min_len, T], the first one = T)."""
    rng = np.random.default_rng(seed)
    Q = rng.standard_normal((B, Hq, D)).astype(np.float16)
    K = rng.standard_normal((B, Hkv, T, D)).astype(np.float16)
    V = rng.standard_normal((B, Hkv, T, D)).astype(np.float16)
    lens = rng.integers(min_len, T + 1, B).astype(np.int32)
    lens[0] = T
    return Q, K, V, lens


_NIBBLE_ELEMENT = [0, 2, 4, 6, 1, 3, 5, 7]      # operand element held by nibble p = 0..7 of a 32-bit word (4-bit codes)


def _nibbles_to_bytes(x):
    """[..., 8] codes in nibble order p -> [..., 4] bytes of the little-endian word."""
    x = x.astype(np.uint8)
    return x[..., 0::2] | (x[..., 1::2] << 4)


def encode_cache(Kq, Ks, Kz, Vq, Vs, Vz, bits: int = 8):
    """Plain arrays ([B,Hkv,cap,128] codes, [B,Hkv,cap] float16 scale / zero) -> (kbuf, vbuf uint8, szbuf uint32) in
    the library's cache layout, written with reshapes."""
    B, Hkv, cap, D = Kq.shape
    assert D == 128 and cap % 32 == 0
    if bits == 4:
        # K: token u = 16*j + c ; d = 32*hh + 8*tt + e  ->  [blk][j][hh][c][tt][nibble p]
        k = Kq.reshape(B, Hkv, cap // 32, 2, 16, 4, 4, 8)        # [b,h,blk,j,c,hh,tt,e]
        k = k.transpose(0, 1, 2, 3, 5, 4, 6, 7)[..., _NIBBLE_ELEMENT]
        kbuf = np.ascontiguousarray(_nibbles_to_bytes(k)).reshape(-1)
        # V: token u = 16*e_hi + 4*hh + e_lo ; e = e_lo + 4*e_hi ; d = 16*(4*i_hi + i_lo) + c
        #    ->  [blk][i_hi][hh][c][i_lo][nibble p]
        v = Vq.reshape(B, Hkv, cap // 32, 2, 4, 4, 2, 4, 16)     # [b,h,blk,e_hi,hh,e_lo,i_hi,i_lo,c]
        v = v.transpose(0, 1, 2, 6, 4, 8, 7, 3, 5).reshape(B, Hkv, cap // 32, 2, 4, 16, 4, 8)[..., _NIBBLE_ELEMENT]
        vbuf = np.ascontiguousarray(_nibbles_to_bytes(v)).reshape(-1)
        szbuf = np.ascontiguousarray(np.stack([_words(Ks, Kz), _words(Vs, Vz)], axis=-1)).reshape(-1)
        return kbuf, vbuf, szbuf
    # K: token u = 16*j + c ; d = 32*hh + 16*half + x  ->  [blk][j][half][hh][c][x]
    k = Kq.reshape(B, Hkv, cap // 32, 2, 16, 4, 2, 16)           # [b,h,blk,j,c,hh,half,x]
    kbuf = np.ascontiguousarray(k.transpose(0, 1, 2, 3, 6, 5, 4, 7)).reshape(-1)
    # V: token u = 16*e_hi + 4*hh + e_lo ; e = e_lo + 4*e_hi ; d = 16*(2*i2 + i_lo) + c  ->  [blk][i2][hh][c][i_lo][e_hi][e_lo]
    v = Vq.reshape(B, Hkv, cap // 32, 2, 4, 4, 4, 2, 16)         # [b,h,blk,e_hi,hh,e_lo,i2,i_lo,c]
    vbuf = np.ascontiguousarray(v.transpose(0, 1, 2, 6, 4, 8, 7, 3, 5)).reshape(-1)
    szbuf = np.ascontiguousarray(np.stack([_words(Ks, Kz), _words(Vs, Vz)], axis=-1)).reshape(-1)
    return kbuf, vbuf, szbuf


def _words(s, z):
    return s.view(np.uint16).astype(np.uint32) | (z.view(np.uint16).astype(np.uint32) << 16)
