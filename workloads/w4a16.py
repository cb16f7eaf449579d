"""Seeded synthetic workloads for the W4A16 GEMM  Y = X * dequant(Wq).

This module only *draws inputs*: Gaussian weight matrices of LLM-layer shape, the group-wise asymmetric
int4 recipe that turns them into (q, s, z), and Gaussian fp16 activations.  It holds none of the method's
arithmetic (no packing into the kernel layout, no dequantisation, no matrix multiply) and is imported by the
tests and the bench, never by the oracle or by the GPU library.

Recipe (one ``numpy.random.default_rng(seed)`` per case; W is drawn in 1024-row chunks, per chunk W -> outlier
mask, and X is drawn last):
  W   = sigma * standard_normal((K, N)) as fp32; optionally a Bernoulli(outlier_frac) mask multiplies entries by 20
  per column n and K-group of ``group`` rows:
        s = fp16((max - min) / 15)          (fp32 arithmetic, then one rounding to fp16; 1.0 if that is 0)
        z = clip(rint(-min / s), 0, 15)     (rint = round-half-to-even, fp32, with the rounded s)
        q = clip(rint(w / s) + z, 0, 15)
  X   = fp16(standard_normal((M, K)))
The synthetic shapes stand in for the Llama/Qwen-class AWQ/GPTQ checkpoints the paper evaluates
(Sec. 5.1, Sec. 5.3): only layer shapes and value distributions matter to a GEMM.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Case:
    name: str
    M: int
    K: int
    N: int
    group: int
    sigma: float = 0.02
    outlier_frac: float = 0.0
    seed: int = 0


def quantise_recipe(W: np.ndarray, group: int, bits: int = 4):
    """Vectorised statement of the quantiser recipe: W fp32 [K,N] -> q uint8 [K,N], s,z float16 [K/g,N].
    bits = 8 is the same recipe with 255 levels (codes 0..255) for the 8-bit weight format."""
    qmax = np.float32((1 << bits) - 1)
    W = np.ascontiguousarray(W, dtype=np.float32)
    K, N = W.shape
    Wg = W.reshape(K // group, group, N)
    mn = Wg.min(axis=1)
    mx = Wg.max(axis=1)
    s32 = (mx - mn) / qmax
    s16 = s32.astype(np.float16)
    sf = s16.astype(np.float32)
    bad = ~(sf > 0) | np.isinf(sf)
    sf = np.where(bad, np.float32(1.0), sf).astype(np.float32)
    s16 = np.where(bad, np.float16(1.0), s16).astype(np.float16)
    z = np.clip(np.rint(-mn / sf), 0, qmax).astype(np.float32)
    q = np.clip(np.rint(Wg / sf[:, None, :]) + z[:, None, :], 0, qmax)
    return q.reshape(K, N).astype(np.uint8), s16, z.astype(np.float16)


def pack_interchange(q: np.ndarray) -> np.ndarray:
    """q uint8 [K,N] -> uint32 [K,N/8], nibble t of word (k,j) = q[k][8j+t] (the layout tm_pack_w4 accepts)."""
    K, N = q.shape
    q32 = q.astype(np.uint32).reshape(K, N // 8, 8)
    shifts = (4 * np.arange(8, dtype=np.uint32))[None, None, :]
    return np.bitwise_or.reduce(q32 << shifts, axis=2).astype(np.uint32)


# Interchange layouts tm_pack_w4_layout accepts (values of its ``layout`` argument).
LAYOUT_N8, LAYOUT_N8_INTERLEAVED, LAYOUT_K8 = 0, 1, 2
_N8I_ORDER = (0, 2, 4, 6, 1, 3, 5, 7)


def encode_layout(q: np.ndarray, z: np.ndarray, layout: int):
    """(q uint8 [K,N], z float16 [K/g,N] integer-valued) -> (qweight, zeros) as a checkpoint of that layout stores them.

    LAYOUT_N8              qweight u32 [K,N/8] nibble t = column 8j+t;                    zeros fp16 [K/g,N]
    LAYOUT_N8_INTERLEAVED  qweight u32 [K,N/8] nibble p = column 8j+(0,2,4,6,1,3,5,7)[p]; zeros u32 [K/g,N/8], same order
    LAYOUT_K8              qweight u32 [K/8,N] nibble t = row 8i+t;                       zeros u32 [K/g,N/8] nibble t = column 8j+t
    Only a storage format: no arithmetic of the method."""
    shifts = 4 * np.arange(8, dtype=np.uint32)
    zi = z.astype(np.float32).astype(np.uint8)
    if layout == LAYOUT_N8:
        return pack_interchange(q), z
    if layout == LAYOUT_N8_INTERLEAVED:
        def rows(a):
            R, N = a.shape
            a = a.astype(np.uint32).reshape(R, N // 8, 8)[:, :, list(_N8I_ORDER)]
            return np.bitwise_or.reduce(a << shifts[None, None, :], axis=2).astype(np.uint32)
        return rows(q), rows(zi)
    if layout == LAYOUT_K8:
        K, N = q.shape
        a = q.astype(np.uint32).reshape(K // 8, 8, N)
        qw = np.bitwise_or.reduce(a << shifts[None, :, None], axis=1).astype(np.uint32)
        return qw, pack_interchange(zi)
    raise ValueError(f"unknown layout {layout}")


def quantise_fp8_recipe(W: np.ndarray, group: int):
    """FP8 (E4M3, finite-only) weight recipe: per column and K-group s = fp16(max|w| / 448) (1.0 if that is 0),
    q = nearest FP8 code of w / s (fp32 division, round-to-nearest-even), written with PyTorch's CPU float8 type.
    -> (q uint8 [K,N] codes, s float16 [K/g,N])."""
    import torch
    W = np.ascontiguousarray(W, dtype=np.float32)
    K, N = W.shape
    Wg = W.reshape(K // group, group, N)
    s32 = np.abs(Wg).max(axis=1) / np.float32(448.0)
    s16 = s32.astype(np.float16)
    sf = s16.astype(np.float32)
    bad = ~(sf > 0) | np.isinf(sf)
    sf = np.where(bad, np.float32(1.0), sf).astype(np.float32)
    s16 = np.where(bad, np.float16(1.0), s16).astype(np.float16)
    r = np.clip(Wg / sf[:, None, :], -448.0, 448.0).astype(np.float32)
    q = torch.from_numpy(r).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    return q.reshape(K, N), s16


def pack_interchange8(q: np.ndarray) -> np.ndarray:
    """8-bit codes q uint8 [K,N] -> uint32 [K,N/4], byte t of word (k,j) = q[k][4j+t] (the layout tm_pack_w8 accepts)."""
    K, N = q.shape
    q32 = q.astype(np.uint32).reshape(K, N // 4, 4)
    shifts = (8 * np.arange(4, dtype=np.uint32))[None, None, :]
    return np.bitwise_or.reduce(q32 << shifts, axis=2).astype(np.uint32)


def draw_act_order(K: int, group: int, rng: np.random.Generator) -> np.ndarray:
    """Group index per row as an activation-order (act-order) checkpoint stores it: a random permutation of the rows is
    cut into consecutive groups, so every group has exactly ``group`` rows scattered over K.  int32 [K]."""
    g_idx = np.empty(K, np.int32)
    g_idx[rng.permutation(K)] = np.arange(K, dtype=np.int32) // group
    return g_idx


def draw_weights(case: Case, rng: np.random.Generator) -> np.ndarray:
    W = (case.sigma * rng.standard_normal((case.K, case.N), dtype=np.float32)).astype(np.float32)
    if case.outlier_frac > 0:
        mask = rng.random((case.K, case.N), dtype=np.float32) < case.outlier_frac
        W = np.where(mask, W * np.float32(20.0), W).astype(np.float32)
    return W


def draw_activations(case: Case, rng: np.random.Generator, M: int | None = None) -> np.ndarray:
    M = case.M if M is None else M
    return rng.standard_normal((M, case.K), dtype=np.float32).astype(np.float16)


def make(case: Case, keep_W: bool = False, chunk_rows: int = 1024):
    """-> dict(q u8, s f16, z f16, qweight u32 interchange words, X f16[, W fp32]).

    W is drawn and quantised in chunks of ``chunk_rows`` rows (a multiple of the group) so the largest shapes
    never hold several fp32 copies of the matrix.  Draw order: per chunk W -> outlier mask; X last."""
    rng = np.random.default_rng(case.seed)
    chunk_rows = max(case.group, (chunk_rows // case.group) * case.group)
    Ws, qs, ss, zs = [], [], [], []
    for k0 in range(0, case.K, chunk_rows):
        rows = min(chunk_rows, case.K - k0)
        sub = Case(case.name, case.M, rows, case.N, case.group, case.sigma, case.outlier_frac, case.seed)
        W = draw_weights(sub, rng)
        q, s, z = quantise_recipe(W, case.group)
        qs.append(q); ss.append(s); zs.append(z)
        if keep_W:
            Ws.append(W)
    q = np.concatenate(qs); s = np.concatenate(ss); z = np.concatenate(zs)
    X = draw_activations(case, rng)
    out = {"q": q, "s": s, "z": z, "qweight": pack_interchange(q), "X": X, "case": case}
    if keep_W:
        out["W"] = np.concatenate(Ws)
    return out


# ---------------------------------------------------------------------------------------------
# The five benchmark configurations (layer shapes, group sizes and value distributions of the headline metric).

def config_cases():
    cases = [Case("cfg1_tiny_M1", 1, 512, 512, 128)]
    for M in (1, 4, 8, 16):
        cases.append(Case(f"cfg2_attn_out_M{M}", M, 4096, 4096, 128))
        cases.append(Case(f"cfg2_qkv_M{M}", M, 4096, 12288, 128))
    for M in (1, 16, 32, 64):
        cases.append(Case(f"cfg3_gate_up_M{M}", M, 4096, 22016, 128))
        cases.append(Case(f"cfg3_down_M{M}", M, 11008, 4096, 128))
    cases.append(Case("cfg4_prefill_70b_mlp", 4096, 8192, 28672, 128, sigma=0.01))
    for M in (1, 2, 4, 8, 32, 128, 256, 1024):
        cases.append(Case(f"cfg5_sweep_M{M}", M, 8192, 8192, 64, outlier_frac=0.01))
    return cases


def case_by_name(name: str) -> Case:
    for c in config_cases():
        if c.name == name:
            return c
    raise KeyError(name)


def algorithmic_bytes(M: int, K: int, N: int, group: int, bits: int = 4) -> int:
    """Bytes the method itself must move: int4 (or int8) weights + fp16 scale and zero per group + X + Y."""
    return K * N * bits // 8 + 4 * K * N // group + 2 * M * K + 2 * M * N


def flops(M: int, K: int, N: int) -> int:
    return 2 * M * K * N
