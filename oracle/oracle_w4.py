"""ctypes wrapper around the scalar C oracle (``oracle_w4.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()`` and by the
``cpu_baseline`` leg of ``bench.py``.  The GPU library never imports or links anything from here.

Every function takes and returns numpy arrays; fp16 data travels as ``numpy.float16`` (or uint16 bit
patterns) and is reinterpreted, never converted, on the way in and out.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# ORACLE_W4_SRC names another copy of the C source to build and load instead (beside which its library is put): the
# mutation and sanitizer tests run the pins against a deliberately damaged or an instrumented oracle that way.
_SRC = os.environ.get("ORACLE_W4_SRC") or os.path.join(_HERE, "oracle_w4.c")
_LIB = os.path.join(os.path.dirname(os.path.abspath(_SRC)), "liboracle_w4.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (scalar code, no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c11", "-O2", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-fvisibility=hidden", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        c = ctypes
        vp = c.c_void_p
        lib.orc_fp16_to_double.restype = c.c_double
        lib.orc_fp16_to_double.argtypes = [c.c_uint16]
        lib.orc_double_to_fp16.restype = c.c_uint16
        lib.orc_double_to_fp16.argtypes = [c.c_double]
        lib.orc_quantise.argtypes = [vp, c.c_int, c.c_int, c.c_int, vp, vp, vp]
        lib.orc_pack_canonical.argtypes = [vp, c.c_int, c.c_int, vp]
        lib.orc_unpack_canonical.argtypes = [vp, c.c_int, c.c_int, vp]
        for f in (lib.orc_pack_n8i, lib.orc_unpack_n8i, lib.orc_pack_k8, lib.orc_unpack_k8):
            f.argtypes = [vp, c.c_int, c.c_int, vp]
        lib.orc_quantise_bits.argtypes = [vp, c.c_int, c.c_int, c.c_int, c.c_int, vp, vp, vp]
        lib.orc_pack_canonical8.argtypes = [vp, c.c_int, c.c_int, vp]
        lib.orc_unpack_canonical8.argtypes = [vp, c.c_int, c.c_int, vp]
        lib.orc_unpack_packed8.argtypes = [vp, vp, c.c_int, c.c_int, c.c_int, vp, vp, vp]
        lib.orc_fp8e4m3_decode_table.argtypes = [vp]
        lib.orc_fp8e4m3_decode_table.restype = None
        lib.orc_quantise_fp8.argtypes = [vp, c.c_int, c.c_int, c.c_int, vp, vp]
        lib.orc_dequant_fp8.argtypes = [vp, vp, c.c_int, c.c_int, c.c_int, vp]
        lib.orc_gemm_fp8.argtypes = [vp, c.c_int, vp, vp, c.c_int, c.c_int, c.c_int, vp, vp]
        lib.orc_dequant_gidx.argtypes = [vp, vp, vp, vp, c.c_int, c.c_int, c.c_int, vp]
        lib.orc_gemm_gidx.argtypes = [vp, c.c_int, vp, vp, vp, vp, c.c_int, c.c_int, c.c_int, vp]
        lib.orc_unpack_packed.argtypes = [vp, vp, c.c_int, c.c_int, c.c_int, vp, vp, vp]
        lib.orc_dequant.argtypes = [vp, vp, vp, c.c_int, c.c_int, c.c_int, vp]
        lib.orc_gemm.argtypes = [vp, c.c_int, vp, vp, vp, c.c_int, c.c_int, c.c_int, vp, vp]
        lib.orc_gemm_sampled.argtypes = [vp, c.c_int, vp, vp, vp, c.c_int, c.c_int, c.c_int,
                                         vp, vp, c.c_long, vp, vp]
        lib.orc_num_threads.restype = c.c_int
        _lib = lib
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _as(a, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16 and dtype == np.uint16:
        a = a.view(np.uint16)
    if a.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {a.dtype}")
    return a


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"oracle {what} rejected its arguments (code {rc})")


def num_threads() -> int:
    return int(_load().orc_num_threads())


def fp16_to_double(bits: int) -> float:
    return float(_load().orc_fp16_to_double(int(bits) & 0xFFFF))


def double_to_fp16(x: float) -> int:
    return int(_load().orc_double_to_fp16(float(x)))


def quantise(W: np.ndarray, group: int, bits: int = 4):
    """W fp32 [K,N] -> (q uint8 [K,N] codes 0..2^bits-1, s float16 [K/g,N], z float16 [K/g,N])."""
    W = _as(W, np.float32)
    K, N = W.shape
    q = np.empty((K, N), np.uint8)
    s = np.empty((K // group, N), np.uint16)
    z = np.empty((K // group, N), np.uint16)
    _check(_load().orc_quantise_bits(_ptr(W), K, N, group, bits, _ptr(q), _ptr(s), _ptr(z)), "quantise")
    return q, s.view(np.float16), z.view(np.float16)


def pack_canonical8(q: np.ndarray) -> np.ndarray:
    """8-bit codes q u8 [K,N] -> u32 [K,N/4], byte t of word (k,j) = q[k][4j+t]."""
    q = _as(q, np.uint8)
    K, N = q.shape
    out = np.empty((K, N // 4), np.uint32)
    _check(_load().orc_pack_canonical8(_ptr(q), K, N, _ptr(out)), "pack_canonical8")
    return out


def unpack_canonical8(words: np.ndarray, N: int) -> np.ndarray:
    words = _as(words, np.uint32)
    K = words.shape[0]
    q = np.empty((K, N), np.uint8)
    _check(_load().orc_unpack_canonical8(_ptr(words), K, N, _ptr(q)), "unpack_canonical8")
    return q


def pack_canonical(q: np.ndarray) -> np.ndarray:
    q = _as(q, np.uint8)
    K, N = q.shape
    out = np.empty((K, N // 8), np.uint32)
    _check(_load().orc_pack_canonical(_ptr(q), K, N, _ptr(out)), "pack_canonical")
    return out


def unpack_canonical(words: np.ndarray, N: int) -> np.ndarray:
    words = _as(words, np.uint32)
    K = words.shape[0]
    q = np.empty((K, N), np.uint8)
    _check(_load().orc_unpack_canonical(_ptr(words), K, N, _ptr(q)), "unpack_canonical")
    return q


def pack_n8i(q: np.ndarray) -> np.ndarray:
    """q u8 [K,N] -> u32 [K,N/8], nibble p of word (k,j) = q[k][8j + (0,2,4,6,1,3,5,7)[p]]."""
    q = _as(q, np.uint8)
    K, N = q.shape
    out = np.empty((K, N // 8), np.uint32)
    _check(_load().orc_pack_n8i(_ptr(q), K, N, _ptr(out)), "pack_n8i")
    return out


def unpack_n8i(words: np.ndarray, N: int) -> np.ndarray:
    words = _as(words, np.uint32)
    K = words.shape[0]
    q = np.empty((K, N), np.uint8)
    _check(_load().orc_unpack_n8i(_ptr(words), K, N, _ptr(q)), "unpack_n8i")
    return q


def pack_k8(q: np.ndarray) -> np.ndarray:
    """q u8 [K,N] -> u32 [K/8,N], nibble t of word (i,n) = q[8i+t][n]."""
    q = _as(q, np.uint8)
    K, N = q.shape
    out = np.empty((K // 8, N), np.uint32)
    _check(_load().orc_pack_k8(_ptr(q), K, N, _ptr(out)), "pack_k8")
    return out


def unpack_k8(words: np.ndarray, K: int) -> np.ndarray:
    words = _as(words, np.uint32)
    N = words.shape[1]
    q = np.empty((K, N), np.uint8)
    _check(_load().orc_unpack_k8(_ptr(words), K, N, _ptr(q)), "unpack_k8")
    return q


def unpack_packed(wbuf: np.ndarray, szbuf: np.ndarray, K: int, N: int, group: int, bits: int = 4):
    """Invert the library's fragment-ordered buffers -> (q, s, z) in the plain [K,N] / [K/g,N] layouts."""
    wbuf = _as(wbuf, np.uint32).reshape(-1)
    szbuf = _as(szbuf, np.uint32).reshape(-1)
    if bits not in (4, 8):
        raise ValueError("bits must be 4 or 8")
    if wbuf.size != K * N * bits // 32 or szbuf.size != (K // group) * N:
        raise ValueError("packed buffer sizes do not match K, N, group, bits")
    q = np.empty((K, N), np.uint8)
    s = np.empty((K // group, N), np.uint16)
    z = np.empty((K // group, N), np.uint16)
    fn = _load().orc_unpack_packed if bits == 4 else _load().orc_unpack_packed8
    _check(fn(_ptr(wbuf), _ptr(szbuf), K, N, group, _ptr(q), _ptr(s), _ptr(z)), "unpack_packed")
    return q, s.view(np.float16), z.view(np.float16)


def dequant(q: np.ndarray, s: np.ndarray, z: np.ndarray, group: int) -> np.ndarray:
    q = _as(q, np.uint8)
    s = _as(s, np.uint16)
    z = _as(z, np.uint16)
    K, N = q.shape
    out = np.empty((K, N), np.float64)
    _check(_load().orc_dequant(_ptr(q), _ptr(s), _ptr(z), K, N, group, _ptr(out)), "dequant")
    return out


def gemm(X: np.ndarray, q: np.ndarray, s: np.ndarray, z: np.ndarray, group: int, want_fp64: bool = False):
    """Y = fp16(X @ dequant(q,s,z)) with fp64 accumulation; optionally also the unrounded fp64 sums."""
    X = _as(X, np.uint16)
    q = _as(q, np.uint8)
    s = _as(s, np.uint16)
    z = _as(z, np.uint16)
    M, K = X.shape
    K2, N = q.shape
    if K2 != K:
        raise ValueError("X and q disagree on K")
    Y = np.empty((M, N), np.uint16)
    Yd = np.empty((M, N), np.float64) if want_fp64 else None
    _check(_load().orc_gemm(_ptr(X), M, _ptr(q), _ptr(s), _ptr(z), K, N, group, _ptr(Y),
                            _ptr(Yd) if want_fp64 else None), "gemm")
    return (Y.view(np.float16), Yd) if want_fp64 else Y.view(np.float16)


def dequant_gidx(q: np.ndarray, s: np.ndarray, z: np.ndarray, g_idx: np.ndarray) -> np.ndarray:
    """(q - z[g_idx[k]]) * s[g_idx[k]]: the K-group of row k is g_idx[k] (activation-order checkpoints)."""
    q = _as(q, np.uint8); s = _as(s, np.uint16); z = _as(z, np.uint16); g_idx = _as(g_idx, np.int32)
    K, N = q.shape
    out = np.empty((K, N), np.float64)
    _check(_load().orc_dequant_gidx(_ptr(q), _ptr(s), _ptr(z), _ptr(g_idx), K, N, s.shape[0], _ptr(out)), "dequant_gidx")
    return out


def gemm_gidx(X: np.ndarray, q: np.ndarray, s: np.ndarray, z: np.ndarray, g_idx: np.ndarray) -> np.ndarray:
    """Y = fp16(X @ dequant_gidx(q, s, z, g_idx)), fp64 accumulation with k ascending in the checkpoint's row order."""
    X = _as(X, np.uint16); q = _as(q, np.uint8); s = _as(s, np.uint16); z = _as(z, np.uint16)
    g_idx = _as(g_idx, np.int32)
    M, K = X.shape
    N = q.shape[1]
    Y = np.empty((M, N), np.uint16)
    _check(_load().orc_gemm_gidx(_ptr(X), M, _ptr(q), _ptr(s), _ptr(z), _ptr(g_idx), K, N, s.shape[0], _ptr(Y)),
           "gemm_gidx")
    return Y.view(np.float16)


def fp8e4m3_table() -> np.ndarray:
    """The 256 values of the OCP FP8 E4M3 (finite-only) codes as float64 (NaN at 0x7F and 0xFF)."""
    out = np.empty(256, np.float64)
    _load().orc_fp8e4m3_decode_table(_ptr(out))
    return out


def quantise_fp8(W: np.ndarray, group: int):
    """W fp32 [K,N] -> (q uint8 [K,N] FP8 E4M3 codes, s float16 [K/g,N]), s = fp16(max|w|/448) per group."""
    W = _as(W, np.float32)
    K, N = W.shape
    q = np.empty((K, N), np.uint8)
    s = np.empty((K // group, N), np.uint16)
    _check(_load().orc_quantise_fp8(_ptr(W), K, N, group, _ptr(q), _ptr(s)), "quantise_fp8")
    return q, s.view(np.float16)


def dequant_fp8(q: np.ndarray, s: np.ndarray, group: int) -> np.ndarray:
    q = _as(q, np.uint8)
    s = _as(s, np.uint16)
    K, N = q.shape
    out = np.empty((K, N), np.float64)
    _check(_load().orc_dequant_fp8(_ptr(q), _ptr(s), K, N, group, _ptr(out)), "dequant_fp8")
    return out


def gemm_fp8(X: np.ndarray, q: np.ndarray, s: np.ndarray, group: int) -> np.ndarray:
    """Y = fp16(X @ (fp8(q) * s)) with fp64 accumulation, k ascending."""
    X = _as(X, np.uint16)
    q = _as(q, np.uint8)
    s = _as(s, np.uint16)
    M, K = X.shape
    N = q.shape[1]
    Y = np.empty((M, N), np.uint16)
    _check(_load().orc_gemm_fp8(_ptr(X), M, _ptr(q), _ptr(s), K, N, group, _ptr(Y), None), "gemm_fp8")
    return Y.view(np.float16)


def gemm_grouped(X: np.ndarray, experts, offsets, group: int) -> np.ndarray:
    """Mixture-of-experts layer with rows sorted by expert (the MoE models of paper Sec. 5.1 run the GEMM of Sec. 3.1
    once per expert): rows offsets[e] <= r < offsets[e+1] of X go through expert e = (q, s, z).  Rows no expert
    claims come back as NaN so that a test can see they were left alone.  One gemm() call per expert, nothing else."""
    X = np.asarray(X)
    N = experts[0][0].shape[1]
    Y = np.full((X.shape[0], N), np.nan, np.float16)
    for e, (q, s, z) in enumerate(experts):
        r0, r1 = int(offsets[e]), int(offsets[e + 1])
        if r1 > r0:
            Y[r0:r1] = gemm(X[r0:r1], q, s, z, group)
    return Y


def gemm_sampled(X, q, s, z, group: int, ms, ns, want_fp64: bool = False):
    """The plain triple loop evaluated only at the listed (m, n) pairs."""
    X = _as(X, np.uint16)
    q = _as(q, np.uint8)
    s = _as(s, np.uint16)
    z = _as(z, np.uint16)
    ms = np.ascontiguousarray(ms, dtype=np.int32)
    ns = np.ascontiguousarray(ns, dtype=np.int32)
    M, K = X.shape
    _, N = q.shape
    Y = np.empty(ms.shape, np.uint16)
    Yd = np.empty(ms.shape, np.float64) if want_fp64 else None
    _check(_load().orc_gemm_sampled(_ptr(X), M, _ptr(q), _ptr(s), _ptr(z), K, N, group, _ptr(ms), _ptr(ns),
                                    ms.size, _ptr(Y), _ptr(Yd) if want_fp64 else None), "gemm_sampled")
    return (Y.view(np.float16), Yd) if want_fp64 else Y.view(np.float16)


def epilogue(Yd: np.ndarray, bias=None, residual=None, act: str = "none") -> np.ndarray:
    """What surrounds the matrix product in a transformer block, written out in fp64 (not in the paper: the widened
    "fused epilogue" row): Yd [M, N] unrounded sums -> fp16.
      bias      [N]: added to every row
      act       "none", or "silu_mul": the columns are [gate | up] halves and the result is silu(gate) * up, [M, N/2],
                silu(x) = x / (1 + exp(-x))
      residual  [M, N_out]: added last."""
    Y = np.asarray(Yd, np.float64)
    if bias is not None:
        Y = Y + np.asarray(bias).astype(np.float64)[None, :]
    if act == "silu_mul":
        half = Y.shape[1] // 2
        g, u = Y[:, :half], Y[:, half:]
        Y = g / (1.0 + np.exp(-g)) * u
    elif act != "none":
        raise ValueError(act)
    if residual is not None:
        Y = Y + np.asarray(residual).astype(np.float64)
    return Y.astype(np.float16)
