"""Pins for the CPU oracle: every check compares it with something it did not produce itself
(numpy's float16, hand-worked fixtures, closed forms, brute force, numpy matmul, an independently written
numpy statement of the same recipe/layout)."""
import os
from fractions import Fraction

import numpy as np
import pytest

from workloads import w4a16 as wl
from helpers import acceptance

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ fp16 conversion

def test_fp16_to_double_exhaustive(oracle):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.fp16_to_double(int(b)) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_double_to_fp16_roundtrip_exhaustive(oracle):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    vals = bits.view(np.float16).astype(np.float64)
    for b, v in zip(bits, vals):
        if np.isnan(v):
            assert (oracle.double_to_fp16(v) & 0x7C00) == 0x7C00 and (oracle.double_to_fp16(v) & 0x3FF)
        else:
            assert oracle.double_to_fp16(float(v)) == int(b)


def test_double_to_fp16_matches_numpy_on_random_and_edges(oracle):
    rng = np.random.default_rng(1)
    xs = np.concatenate([
        rng.standard_normal(60000),
        rng.standard_normal(30000) * 1e-4,                 # around the subnormal boundary 6.1e-5
        rng.standard_normal(30000) * 1e-7,                 # deep subnormals / underflow to zero
        rng.standard_normal(30000) * 3e4,                  # around overflow 65504 / 65520
        np.ldexp(rng.uniform(1, 2, 30000), rng.integers(-30, 18, 30000)),
    ])
    # exact ties between neighbouring fp16 values, at every exponent, both parities
    h = np.arange(0, 0x7BFF, 7, dtype=np.uint16)
    lo = h.view(np.float16).astype(np.float64)
    hi = (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    ties = (lo + hi) / 2
    edges = np.array([0.0, -0.0, 2.0 ** -25, np.nextafter(2.0 ** -25, 1), 2.0 ** -24, 65504.0, 65519.999,
                      65520.0, 65536.0, 1e300, -1e300, np.inf, -np.inf, 2.0 ** -14, np.nextafter(2.0 ** -14, 0)])
    xs = np.concatenate([xs, ties, -ties, np.nextafter(ties, np.inf), np.nextafter(ties, -np.inf), edges])
    with np.errstate(over="ignore"):
        want = xs.astype(np.float16).view(np.uint16)
    got = np.array([oracle.double_to_fp16(float(x)) for x in xs], dtype=np.uint16)
    assert np.array_equal(got, want)


# ------------------------------------------------------------------ quantiser

def _read_quant_fixture(name="quant_group_pow2.txt"):
    rows = []
    for line in open(os.path.join(GOLD, name)):
        line = line.split("#")[0].strip()
        if line:
            w, q, d = line.split()
            rows.append((float(w), int(q), float(d)))
    return rows


def test_quantise_hand_worked_group(oracle):
    rows = _read_quant_fixture()
    W = np.array([[r[0]] for r in rows], np.float32)           # K = 10, N = 1, one group
    q, s, z = oracle.quantise(W, len(rows))
    assert float(s[0, 0]) == 0.125 and float(z[0, 0]) == 8.0
    assert q[:, 0].tolist() == [r[1] for r in rows]
    deq = oracle.dequant(q, s, z, len(rows))
    assert deq[:, 0].tolist() == [r[2] for r in rows]


def test_quantise_8bit_hand_worked_group(oracle):
    rows = _read_quant_fixture("quant_group_8bit.txt")
    W = np.array([[r[0]] for r in rows], np.float32)
    q, s, z = oracle.quantise(W, len(rows), bits=8)
    assert float(s[0, 0]) == 0.015625 and float(z[0, 0]) == 64.0
    assert q[:, 0].tolist() == [r[1] for r in rows]
    assert oracle.dequant(q, s, z, len(rows))[:, 0].tolist() == [r[2] for r in rows]
    # and the independent vectorised recipe agrees bit for bit on random data
    rng = np.random.default_rng(8)
    Wr = (0.02 * rng.standard_normal((256, 24))).astype(np.float32)
    for g in (32, 128):
        q1, s1, z1 = oracle.quantise(Wr, g, bits=8)
        q2, s2, z2 = wl.quantise_recipe(Wr, g, bits=8)
        assert np.array_equal(q1, q2) and np.array_equal(s1.view(np.uint16), s2.view(np.uint16))
        assert np.array_equal(z1.view(np.uint16), z2.view(np.uint16)) and q1.max() > 200


def test_quantise_zero_point_tie_fixture(oracle):
    rows = _read_quant_fixture("quant_group_ztie.txt")
    W = np.array([[r[0]] for r in rows], np.float32)
    q, s, z = oracle.quantise(W, len(rows))
    assert float(s[0, 0]) == 0.125 and float(z[0, 0]) == 6.0
    assert q[:, 0].tolist() == [r[1] for r in rows]
    assert oracle.dequant(q, s, z, len(rows))[:, 0].tolist() == [r[2] for r in rows]


def test_quantise_matches_recipe_statement_and_invariants(oracle):
    rng = np.random.default_rng(3)
    for (K, N, g, sigma, outl) in [(256, 48, 128, 0.02, 0.0), (256, 32, 64, 0.02, 0.01), (96, 8, 32, 1.0, 0.0)]:
        case = wl.Case("t", 1, K, N, g, sigma, outl, seed=int(rng.integers(1 << 30)))
        W = wl.draw_weights(case, np.random.default_rng(case.seed))
        q, s, z = oracle.quantise(W, g)
        q2, s2, z2 = wl.quantise_recipe(W, g)               # independent vectorised statement of the recipe
        assert np.array_equal(q, q2) and np.array_equal(s.view(np.uint16), s2.view(np.uint16))
        assert np.array_equal(z.view(np.uint16), z2.view(np.uint16))
        assert q.max() <= 15 and z.astype(np.float32).max() <= 15 and z.astype(np.float32).min() >= 0
        sf = np.repeat(s.astype(np.float64), g, axis=0)
        zf = np.repeat(z.astype(np.float64), g, axis=0)
        deq = oracle.dequant(q, s, z, g)
        assert np.array_equal(deq, (q.astype(np.float64) - zf) * sf)     # closed form, exact in fp64
        err = np.abs(W.astype(np.float64) - deq)
        pre = np.rint(W / sf.astype(np.float32)) + zf                    # value before the clamp
        unclamped = (pre >= 0) & (pre <= 15)
        assert (err[unclamped] <= 0.5 * sf[unclamped] * (1 + 1e-6)).all()
        assert (err <= 1.5 * sf * (1 + 1e-6)).all()
        # group minimum maps to code 0 whenever the zero-point was not clamped
        Wg = W.reshape(K // g, g, N)
        zraw = np.rint(-Wg.min(axis=1) / s.astype(np.float32))
        ok = (zraw >= 0) & (zraw <= 15)
        qmin = np.take_along_axis(q.reshape(K // g, g, N), Wg.argmin(axis=1)[:, None, :], axis=1)[:, 0, :]
        assert (qmin[ok] == 0).all()


def test_quantise_degenerate_groups(oracle):
    W = np.zeros((64, 4), np.float32)
    W[:, 1] = 3.0                      # constant, positive
    W[:, 2] = -2.0                     # constant, negative
    W[:32, 3] = 1e-9                   # range far below fp16 resolution
    q, s, z = oracle.quantise(W, 64)
    assert (s.astype(np.float32) == 1.0).all()
    assert z[0].astype(np.float32).tolist() == [0.0, 0.0, 2.0, 0.0]
    assert (q[:, 0] == 0).all() and (q[:, 1] == 3).all() and (q[:, 2] == 0).all() and (q[:, 3] == 0).all()


# ------------------------------------------------------------------ canonical interchange layout

def test_pack_canonical_hand_example(oracle):
    q = np.array([[1, 2, 3, 4, 5, 6, 7, 8], [15, 0, 0, 0, 0, 0, 0, 0], [0, 0, 0, 0, 0, 0, 0, 15]], np.uint8)
    assert oracle.pack_canonical(q)[:, 0].tolist() == [0x87654321, 0x0000000F, 0xF0000000]


def test_pack_canonical_roundtrip_and_agrees_with_generator(oracle):
    rng = np.random.default_rng(5)
    for K, N in [(1, 8), (7, 24), (128, 64)]:
        q = rng.integers(0, 16, (K, N), dtype=np.uint8)
        w = oracle.pack_canonical(q)
        assert np.array_equal(oracle.unpack_canonical(w, N), q)
        assert np.array_equal(w, wl.pack_interchange(q))


def test_alternative_layout_word_fixture(oracle):
    n = 0
    for line in open(os.path.join(GOLD, "interchange_word_orders.txt")):
        line = line.split("#")[0].split()
        if not line:
            continue
        vals, want = np.array([int(v) for v in line[1:9]], np.uint8), int(line[9], 16)
        if line[0] == "n8i":
            got = oracle.pack_n8i(vals.reshape(1, 8))
        elif line[0] == "q8":
            got = oracle.pack_canonical8(vals[:4].reshape(1, 4))
        else:
            got = oracle.pack_k8(vals.reshape(8, 1))
        assert got.shape == (1, 1) and int(got[0, 0]) == want, line
        n += 1
    assert n >= 10


def test_alternative_layouts_roundtrip_bruteforce_and_generator(oracle):
    rng = np.random.default_rng(6)
    order = [0, 2, 4, 6, 1, 3, 5, 7]
    for K, N in [(8, 8), (16, 24), (128, 64)]:
        q = rng.integers(0, 16, (K, N), dtype=np.uint8)
        z = rng.integers(0, 16, (K // 8, N)).astype(np.float16)
        wi, wk = oracle.pack_n8i(q), oracle.pack_k8(q)
        assert np.array_equal(oracle.unpack_n8i(wi, N), q) and np.array_equal(oracle.unpack_k8(wk, K), q)
        if K * N <= 512:                                   # every nibble, one by one
            for k in range(K):
                for n in range(N):
                    assert (int(wi[k, n // 8]) >> (4 * order.index(n % 8))) & 15 == q[k, n]
                    assert (int(wk[k // 8, n]) >> (4 * (k % 8))) & 15 == q[k, n]
        # the same integers in a different order: interleaving permutes nibbles inside each canonical word
        wc = oracle.pack_canonical(q)
        assert np.array_equal(np.sort(np.stack([(wc >> (4 * t)) & 15 for t in range(8)]), axis=0),
                              np.sort(np.stack([(wi >> (4 * t)) & 15 for t in range(8)]), axis=0))
        # the input generator's encoders write the same words
        for layout, wq in ((wl.LAYOUT_N8, wc), (wl.LAYOUT_N8_INTERLEAVED, wi), (wl.LAYOUT_K8, wk)):
            gq, gz = wl.encode_layout(q, z, layout)
            assert np.array_equal(gq, wq)
            zi = z.astype(np.uint8)
            if layout == wl.LAYOUT_N8:
                assert gz is z
            elif layout == wl.LAYOUT_N8_INTERLEAVED:
                assert np.array_equal(gz, oracle.pack_n8i(zi))
            else:
                assert np.array_equal(gz, oracle.pack_canonical(zi))


# ------------------------------------------------------------------ fragment-ordered layout (inverse map)

def _pack_fragment_order_numpy(q, s, z, g):
    """Forward statement of the layout rule, written with reshapes (independent of the oracle's index loop):
    unit (nt, ku) -> lane 16h+c -> word t -> nibble 4*(e&1)+(e>>1), rows k = 128ku + 32t + 8h + e."""
    K, N = q.shape
    a = q.reshape(K // 128, 4, 4, 8, N // 16, 16)            # [ku, t, h, e, nt, c]
    a = a.transpose(4, 0, 2, 5, 1, 3).astype(np.uint32)      # [nt, ku, h, c, t, e]
    nib = np.array([4 * (e & 1) + (e >> 1) for e in range(8)], np.uint32)
    words = np.bitwise_or.reduce(a << (4 * nib), axis=-1)    # [nt, ku, h, c, t]
    G = K // g
    sz = (s.view(np.uint16).astype(np.uint32) | (z.view(np.uint16).astype(np.uint32) << 16))   # [G, N]
    sz = sz.reshape(G, N // 16, 16).transpose(1, 0, 2)       # [nt, G, c]
    return np.ascontiguousarray(words).reshape(-1), np.ascontiguousarray(sz).reshape(-1)


def test_unpack_packed_word_order_fixture(oracle):
    K, N, g = 128, 16, 128
    s = np.ones((1, N), np.float16)
    z = np.zeros((1, N), np.float16)
    sz = (s.view(np.uint16).astype(np.uint32) | (z.view(np.uint16).astype(np.uint32) << 16)).reshape(-1)
    for line in open(os.path.join(GOLD, "fragment_word_orders.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        *es, word = line.split()
        es = [int(e) for e in es]
        wbuf = np.full(K * N // 8, int(word, 16), np.uint32)
        q, _, _ = oracle.unpack_packed(wbuf, sz, K, N, g)
        want = np.tile(np.array(es, np.uint8)[None, :], (K // 8, 1)).reshape(K)   # q[k][n] = es[k % 8]
        assert np.array_equal(q, np.repeat(want[:, None], N, axis=1))


def test_unpack_packed_position_codes(oracle):
    """Buffers filled with a code of one layout coordinate must unpack to that coordinate's closed form."""
    K, N, g = 256, 32, 64
    KU, NT = K // 128, N // 16
    nt, ku, h, c, t = np.meshgrid(np.arange(NT), np.arange(KU), np.arange(4), np.arange(16), np.arange(4),
                                  indexing="ij")                      # buffer order [nt, ku, lane=16h+c, t]
    k = np.arange(K)[:, None] * np.ones((1, N), int)
    n = np.ones((K, 1), int) * np.arange(N)[None, :]
    sz = np.zeros((K // g) * N, np.uint32)
    for code, want in [(h, (k % 32) // 8), (t, (k % 128) // 32), (c, n % 16), (nt * KU + ku, (n // 16) * KU + k // 128)]:
        wbuf = (code.astype(np.uint32) * np.uint32(0x11111111)).reshape(-1)
        q, _, _ = oracle.unpack_packed(wbuf, sz, K, N, g)
        assert np.array_equal(q, want.astype(np.uint8))
    # scale/zero words: low half scale, high half zero, [nt][G][c]
    G = K // g
    szw = np.arange(NT * G * 16, dtype=np.uint32)
    szw = (szw * 3 + 1) | ((szw * 5 + 2) << 16)
    _, s, z = oracle.unpack_packed(np.zeros(K * N // 8, np.uint32), szw, K, N, g)
    gi, nn = np.meshgrid(np.arange(G), np.arange(N), indexing="ij")
    idx = ((nn // 16) * G + gi) * 16 + nn % 16
    assert np.array_equal(s.view(np.uint16), (idx * 3 + 1).astype(np.uint16))
    assert np.array_equal(z.view(np.uint16), (idx * 5 + 2).astype(np.uint16))


def test_8bit_canonical_and_packed_layout(oracle):
    """8-bit words: round trip and generator agreement for the interchange layout; the fragment-ordered layout
    against hand-worked words, position codes and an independent forward statement written with reshapes."""
    rng = np.random.default_rng(9)
    for K, N in [(1, 4), (5, 12), (128, 32)]:
        q = rng.integers(0, 256, (K, N), dtype=np.uint8)
        w = oracle.pack_canonical8(q)
        assert np.array_equal(oracle.unpack_canonical8(w, N), q) and np.array_equal(w, wl.pack_interchange8(q))
    # hand-worked fragment words: every lane's word pair (2*tt, 2*tt+1) set to the fixture's pair
    K, N, g = 128, 16, 128
    sz = np.zeros(N, np.uint32)
    for line in open(os.path.join(GOLD, "fragment_word_orders_8bit.txt")):
        line = line.split("#")[0].split()
        if not line:
            continue
        es, w0, w1 = [int(e) for e in line[:8]], int(line[8], 16), int(line[9], 16)
        wbuf = np.tile(np.array([w0, w1], np.uint32), K * N // 8)
        q, _, _ = oracle.unpack_packed(wbuf, sz, K, N, g, bits=8)
        assert np.array_equal(q, np.repeat(np.tile(np.array(es, np.uint8), K // 8)[:, None], N, axis=1))
    # position codes: a buffer filled with one layout coordinate unpacks to that coordinate's closed form
    K, N, g = 256, 32, 64
    KS, NT = K // 64, N // 16
    nt, ks, h, c, tt, hf = np.meshgrid(np.arange(NT), np.arange(KS), np.arange(4), np.arange(16), np.arange(2),
                                       np.arange(2), indexing="ij")        # buffer order [nt, ks, lane=16h+c, 2tt+hf]
    k = np.arange(K)[:, None] * np.ones((1, N), int)
    n = np.ones((K, 1), int) * np.arange(N)[None, :]
    sz = np.zeros((K // g) * N, np.uint32)
    for code, want in [(h, (k % 32) // 8), (tt, (k % 64) // 32), (hf, (k % 8) // 4), (c, n % 16),
                       (nt * KS + ks, (n // 16) * KS + k // 64)]:
        wbuf = (code.astype(np.uint32) * np.uint32(0x01010101)).reshape(-1)
        q, _, _ = oracle.unpack_packed(wbuf, sz, K, N, g, bits=8)
        assert np.array_equal(q, want.astype(np.uint8))
    wbuf = np.tile(np.array([0x03020100], np.uint32), K * N // 4)           # byte index b = k % 4
    q, _, _ = oracle.unpack_packed(wbuf, sz, K, N, g, bits=8)
    assert np.array_equal(q, (k % 4).astype(np.uint8))
    # forward statement with reshapes: [ks, tt, h, hf, b, nt, c] -> [nt, ks, h, c, tt, hf] words of bytes b
    q = rng.integers(0, 256, (K, N), dtype=np.uint8)
    s = rng.uniform(0.001, 0.02, (K // g, N)).astype(np.float16)
    z = rng.integers(0, 256, (K // g, N)).astype(np.float16)
    a = q.reshape(KS, 2, 4, 2, 4, NT, 16).transpose(5, 0, 2, 6, 1, 3, 4).astype(np.uint32)
    words = np.bitwise_or.reduce(a << (8 * np.arange(4, dtype=np.uint32)), axis=-1).reshape(-1)
    szw = (s.view(np.uint16).astype(np.uint32) | (z.view(np.uint16).astype(np.uint32) << 16))
    szw = np.ascontiguousarray(szw.reshape(K // g, NT, 16).transpose(1, 0, 2)).reshape(-1)
    q2, s2, z2 = oracle.unpack_packed(words, szw, K, N, g, bits=8)
    assert np.array_equal(q2, q) and np.array_equal(s2.view(np.uint16), s.view(np.uint16))
    assert np.array_equal(z2.view(np.uint16), z.view(np.uint16))


@pytest.mark.parametrize("K,N,g", [(128, 16, 128), (384, 80, 64), (256, 48, 32)])
def test_unpack_packed_inverts_forward_statement(oracle, K, N, g):
    rng = np.random.default_rng(K + N)
    q = rng.integers(0, 16, (K, N), dtype=np.uint8)
    s = rng.standard_normal((K // g, N)).astype(np.float16)
    z = rng.integers(0, 16, (K // g, N)).astype(np.float16)
    wbuf, szbuf = _pack_fragment_order_numpy(q, s, z, g)
    q2, s2, z2 = oracle.unpack_packed(wbuf, szbuf, K, N, g)
    assert np.array_equal(q2, q)
    assert np.array_equal(s2.view(np.uint16), s.view(np.uint16))
    assert np.array_equal(z2.view(np.uint16), z.view(np.uint16))


# ------------------------------------------------------------------ matmul

def _tiny_problem(seed, M, K, N, g):
    rng = np.random.default_rng(seed)
    q = rng.integers(0, 16, (K, N), dtype=np.uint8)
    s = (rng.uniform(0.003, 0.01, (K // g, N))).astype(np.float16)
    z = rng.integers(0, 16, (K // g, N)).astype(np.float16)
    X = rng.standard_normal((M, K)).astype(np.float16)
    return X, q, s, z


def test_gemm_brute_force_exact_rationals(oracle):
    """Triple loop in exact rational arithmetic on a tiny case; fp64 sums must agree to rounding noise and the
    fp16 result must be the correctly rounded exact value wherever that is not within 1e-9 of a tie."""
    M, K, N, g = 3, 64, 8, 32
    X, q, s, z = _tiny_problem(11, M, K, N, g)
    Y, Yd = oracle.gemm(X, q, s, z, g, want_fp64=True)
    for m in range(M):
        for n in range(N):
            acc = Fraction(0)
            for k in range(K):
                w = (int(q[k, n]) - Fraction(float(z[k // g, n]))) * Fraction(float(s[k // g, n]))
                acc += Fraction(float(X[m, k])) * w
            exact = float(acc)
            assert abs(Yd[m, n] - exact) <= 1e-13 * max(1.0, abs(exact))
            assert np.float16(exact) == Y[m, n]


def test_gemm_matches_numpy_matmul(oracle):
    for seed, (M, K, N, g) in enumerate([(5, 256, 40, 128), (17, 384, 272, 64), (1, 512, 512, 128)]):
        X, q, s, z = _tiny_problem(seed, M, K, N, g)
        What = (q.astype(np.float64) - np.repeat(z.astype(np.float64), g, 0)) * np.repeat(s.astype(np.float64), g, 0)
        ref = X.astype(np.float64) @ What
        Y, Yd = oracle.gemm(X, q, s, z, g, want_fp64=True)
        assert np.abs(Yd - ref).max() <= 1e-12 * np.abs(ref).max()
        near_tie = np.abs(ref.astype(np.float16).astype(np.float64) - ref) > 0.4999 * np.spacing(np.abs(ref).astype(np.float16)).astype(np.float64)
        assert np.array_equal(Y[~near_tie], ref.astype(np.float16)[~near_tie])
        # sampled triple loop agrees with the whole-matrix routine element for element
        ms = np.repeat(np.arange(M), 3)
        ns = (np.arange(ms.size) * 7) % N
        Ys, Yds = oracle.gemm_sampled(X, q, s, z, g, ms, ns, want_fp64=True)
        assert np.array_equal(Ys.view(np.uint16), Y[ms, ns].view(np.uint16)) and np.array_equal(Yds, Yd[ms, ns])


def test_gemm_integer_exact_case(oracle):
    """s = 1, small integer X: every product and partial sum is an exactly representable integer."""
    rng = np.random.default_rng(2)
    M, K, N, g = 4, 64, 16, 32
    q = rng.integers(0, 16, (K, N), dtype=np.uint8)
    z = rng.integers(0, 16, (K // g, N)).astype(np.float16)
    s = np.ones((K // g, N), np.float16)
    X = rng.integers(-2, 3, (M, K)).astype(np.float16)
    want = X.astype(np.int64) @ (q.astype(np.int64) - np.repeat(z.astype(np.int64), g, 0))
    assert np.abs(want).max() < 2048
    Y = oracle.gemm(X, q, s, z, g)
    assert np.array_equal(Y.astype(np.int64), want)


def test_gemm_one_hot_rows_return_dequantised_weights(oracle):
    M, K, N, g = 6, 128, 32, 64
    _, q, s, z = _tiny_problem(4, M, K, N, g)
    rows = [0, 1, 63, 64, 100, 127]
    X = np.zeros((M, K), np.float16)
    for m, k in enumerate(rows):
        X[m, k] = 1.0
    Y = oracle.gemm(X, q, s, z, g)
    want = ((q[rows].astype(np.float64) - z.astype(np.float64)[[k // g for k in rows]]) *
            s.astype(np.float64)[[k // g for k in rows]]).astype(np.float16)
    assert np.array_equal(Y.view(np.uint16), want.view(np.uint16))


def test_gemm_transposed_operand_would_fail(oracle):
    """A non-square case pins the operand orientation: X[M,K] times W[K,N], not its transpose."""
    M, K, N, g = 2, 128, 16, 128
    X, q, s, z = _tiny_problem(9, M, K, N, g)
    Y = oracle.gemm(X, q, s, z, g)
    assert Y.shape == (M, N)
    k0 = 37
    X1 = np.zeros((1, K), np.float16); X1[0, k0] = 2.0
    Y1 = oracle.gemm(X1, q, s, z, g)
    assert np.array_equal(Y1[0].astype(np.float64), ((2.0 * (q[k0].astype(np.float64) - z[0].astype(np.float64)) * s[0].astype(np.float64)).astype(np.float16)).astype(np.float64))


# ------------------------------------------------------------------ the tolerance has teeth

def test_acceptance_rejects_planted_mistakes(oracle):
    case = wl.Case("t", 8, 512, 256, 128, seed=21)
    d = wl.make(case)
    q, s, z, X, g = d["q"], d["s"], d["z"], d["X"], case.group
    Yref = oracle.gemm(X, q, s, z, g)

    def fp16_path(qm, sm, zm):
        # a correct fp16-dequant + fp32-accumulate model of the GPU arithmetic, in numpy
        What = ((qm.astype(np.float32) - np.repeat(zm.astype(np.float32), g, 0)).astype(np.float16).astype(np.float32)
                * np.repeat(sm.astype(np.float32), g, 0)).astype(np.float16)
        return (X.astype(np.float32) @ What.astype(np.float32)).astype(np.float16)

    ok, worst, fro = acceptance(fp16_path(q, s, z), Yref)
    assert ok and fro < 1e-3
    # (a) one swapped pair of neighbouring rows inside every 8-row fragment
    qs = q.copy(); qs[0::8], qs[1::8] = q[1::8].copy(), q[0::8].copy()
    assert not acceptance(fp16_path(qs, s, z), Yref)[0]
    # (b) zero-point off by one
    assert not acceptance(fp16_path(q, s, (z.astype(np.float32) + 1).astype(np.float16)), Yref)[0]
    # (c) scale of the neighbouring group
    assert not acceptance(fp16_path(q, np.roll(s, 1, axis=0), z), Yref)[0]
    # (d) neighbouring column's scale/zero (a lane-to-column slip)
    assert not acceptance(fp16_path(q, np.roll(s, 1, axis=1), np.roll(z, 1, axis=1)), Yref)[0]
    # (e) a dropped k-tile
    X2 = X.copy(); X2[:, 128:160] = 0
    assert not acceptance((X2.astype(np.float32) @ oracle.dequant(q, s, z, g).astype(np.float32)).astype(np.float16), Yref)[0]


def test_acceptance_rule_itself():
    r = np.array([[1.0, -2.0, 0.0]], np.float16)
    assert acceptance(r, r)[0]
    y = r.copy(); y[0, 2] = 0.0101
    assert not acceptance(y, r)[0]                 # absolute part: 1e-2
    y = r.copy(); y[0, 1] = np.float16(-2.0 - 0.03)
    assert not acceptance(y, r)[0]                 # 1e-2 + 5e-3*2 = 0.02 < 0.03


# ------------------------------------------------------------------ grouped (mixture-of-experts) form

def test_gemm_grouped_equals_masked_sum_of_dense_products(oracle):
    """Row r of the grouped result is row r of X times the matrix of the one expert that owns r: written here as a
    sum over experts of (row mask) * (X @ W_e) with numpy, which shares nothing with the slice-and-call loop."""
    rng = np.random.default_rng(21)
    K, N, g, E = 64, 16, 32, 4
    experts, What = [], []
    for e in range(E):
        q = rng.integers(0, 16, (K, N), dtype=np.uint8)
        s = rng.uniform(0.01, 0.05, (K // g, N)).astype(np.float16)
        z = rng.integers(0, 16, (K // g, N)).astype(np.float16)
        experts.append((q, s, z))
        What.append((q.astype(np.float64) - np.repeat(z.astype(np.float64), g, 0)) * np.repeat(s.astype(np.float64), g, 0))
    offsets = np.array([0, 3, 3, 8, 9], np.int32)           # expert 1 has no rows; row 9 belongs to nobody
    X = rng.standard_normal((10, K)).astype(np.float16)
    Y = oracle.gemm_grouped(X, experts, offsets, g)
    owner = np.full(10, -1)
    for e in range(E):
        owner[offsets[e]:offsets[e + 1]] = e
    want = sum((owner == e)[:, None] * (X.astype(np.float64) @ What[e]) for e in range(E))
    assert np.isnan(Y[9]).all() and not np.isnan(Y[:9]).any()
    assert np.allclose(Y[:9].astype(np.float64), want[:9], rtol=2e-3, atol=1e-3)
    # one-hot rows pick single dequantised weights, which fp16 holds after one rounding
    X1 = np.zeros((10, K), np.float16)
    for r in range(10):
        X1[r, (7 * r) % K] = 1.0
    Y1 = oracle.gemm_grouped(X1, experts, offsets, g)
    for r in range(9):
        assert np.array_equal(Y1[r], What[owner[r]][(7 * r) % K].astype(np.float16))


# ------------------------------------------------------------------ FP8 (E4M3) weight codes

def test_fp8_decode_table_against_closed_forms_and_torch(oracle):
    import torch
    t = oracle.fp8e4m3_table()
    # closed forms of the format: zero, smallest subnormal 2^-9, smallest normal 2^-6, 1.0 = code 0x38, largest 448
    assert t[0] == 0.0 and t[1] == 2.0 ** -9 and t[8] == 2.0 ** -6 and t[0x38] == 1.0 and t[0x7E] == 448.0
    assert np.isnan(t[0x7F]) and np.isnan(t[0xFF]) and t[0x80] == 0.0 and np.signbit(t[0x80])
    assert np.array_equal(t[128:255], -t[0:127])
    assert np.all(np.diff(t[:127]) > 0)                                   # codes are ordered like their values
    ref = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(np.isnan(t), np.isnan(ref)) and np.array_equal(t[~np.isnan(t)], ref[~np.isnan(ref)])


def test_fp8_quantiser_against_torch_and_generator(oracle):
    import torch
    rng = np.random.default_rng(12)
    W = (0.02 * rng.standard_normal((256, 24))).astype(np.float32)
    W[0, 0] = 0.0
    W[5, 1] = -0.0
    for g in (32, 128):
        q, s = oracle.quantise_fp8(W, g)
        q2, s2 = wl.quantise_fp8_recipe(W, g)
        assert np.array_equal(s.view(np.uint16), s2.view(np.uint16)) and np.array_equal(q, q2)
        assert (q & 0x7F).max() == 0x7E                                   # every group's maximum lands on 448
    # exact ties between neighbouring codes go to the even mantissa: 17 -> 16 (0x58), 19 -> 20 (0x5A), 18 stays (0x59)
    Wt = np.array([[448.0], [17.0], [18.0], [19.0], [-17.0], [0.0009765625]], np.float32)    # s = 1 exactly
    qt, st = oracle.quantise_fp8(Wt, 6)
    assert float(st[0, 0]) == 1.0 and qt[:, 0].tolist() == [0x7E, 0x58, 0x59, 0x5A, 0xD8, 0x00]
    assert qt[:, 0].tolist() == torch.from_numpy(Wt[:, 0]).to(torch.float8_e4m3fn).view(torch.uint8).tolist()


def test_fp8_gemm_against_numpy(oracle):
    rng = np.random.default_rng(13)
    K, N, g, M = 128, 24, 32, 5
    q = rng.integers(0, 256, (K, N), dtype=np.uint8)
    q[(q & 0x7F) == 0x7F] = 0x3C                                          # no NaN codes
    s = rng.uniform(0.001, 0.01, (K // g, N)).astype(np.float16)
    X = rng.standard_normal((M, K)).astype(np.float16)
    What = oracle.fp8e4m3_table()[q] * np.repeat(s.astype(np.float64), g, axis=0)
    assert np.array_equal(oracle.dequant_fp8(q, s, g), What)
    want = X.astype(np.float64) @ What
    Y = oracle.gemm_fp8(X, q, s, g)
    assert np.allclose(Y.astype(np.float64), want, rtol=1e-3, atol=1e-6)
    # one-hot rows pick single dequantised weights, rounded once
    X1 = np.zeros((M, K), np.float16)
    X1[np.arange(M), [3, 40, 77, 100, 127]] = 1.0
    assert np.array_equal(oracle.gemm_fp8(X1, q, s, g), What[[3, 40, 77, 100, 127]].astype(np.float16))


# ------------------------------------------------------------------ explicit group index (activation order)

def test_gidx_forms_against_plain_forms_and_numpy(oracle):
    rng = np.random.default_rng(14)
    K, N, g, M = 96, 16, 32, 4
    q = rng.integers(0, 16, (K, N), dtype=np.uint8)
    s = rng.uniform(0.01, 0.05, (K // g, N)).astype(np.float16)
    z = rng.integers(0, 16, (K // g, N)).astype(np.float16)
    X = rng.standard_normal((M, K)).astype(np.float16)
    plain = (np.arange(K) // g).astype(np.int32)
    assert np.array_equal(oracle.dequant_gidx(q, s, z, plain), oracle.dequant(q, s, z, g))
    assert np.array_equal(oracle.gemm_gidx(X, q, s, z, plain), oracle.gemm(X, q, s, z, g))
    gi = wl.draw_act_order(K, g, rng)
    assert sorted(np.bincount(gi).tolist()) == [g] * (K // g) and not np.array_equal(gi, plain)
    What = (q.astype(np.float64) - z.astype(np.float64)[gi]) * s.astype(np.float64)[gi]          # numpy gather
    assert np.array_equal(oracle.dequant_gidx(q, s, z, gi), What)
    assert np.allclose(oracle.gemm_gidx(X, q, s, z, gi).astype(np.float64), X.astype(np.float64) @ What, rtol=2e-3, atol=1e-3)
    # sorting the rows by group (and the columns of X the same way) gives the plain grouped problem with the same Y
    perm = np.argsort(gi, kind="stable")
    Y1 = oracle.gemm_gidx(X, q, s, z, gi).astype(np.float64)
    Y2 = oracle.gemm(np.ascontiguousarray(X[:, perm]), np.ascontiguousarray(q[perm]), s, z, g).astype(np.float64)
    assert np.allclose(Y1, Y2, rtol=2e-3, atol=2e-3)
    with pytest.raises(ValueError):
        oracle.gemm_gidx(X, q, s, z, np.full(K, K // g, np.int32))                                # index out of range


def test_epilogue_closed_forms_and_torch_silu(oracle):
    """The epilogue oracle against values fixed by the definition and against PyTorch's CPU silu."""
    import torch
    Y = np.array([[0.0, 1.0, -1.0, 20.0, 2.0, 3.0, 4.0, 0.5]], np.float64)          # gate = first four, up = last four
    out = oracle.epilogue(Y, act="silu_mul").astype(np.float64)
    want = [0.0, 1.0 / (1.0 + np.e ** -1.0) * 3.0, -1.0 / (1.0 + np.e) * 4.0, 20.0 * 0.5]
    assert out.shape == (1, 4) and np.allclose(out[0], want, rtol=1e-3)
    assert out[0, 0] == 0.0 and abs(out[0, 3] - 10.0) < 1e-2                           # silu(0) = 0, silu(x) -> x
    # bias is added before the activation, the residual after it
    b = np.array([1.0, 0, 0, 0, 0, 0, 0, 0])
    r = np.full((1, 4), 0.25)
    out2 = oracle.epilogue(Y, bias=b, residual=r, act="silu_mul").astype(np.float64)
    assert abs(out2[0, 0] - (1.0 / (1.0 + np.e ** -1.0) * 2.0 + 0.25)) < 2e-3
    assert np.allclose(out2[0, 1:], out[0, 1:] + 0.25, atol=4e-3)
    # without activation: plain sums, rounded once
    out3 = oracle.epilogue(Y, bias=b, residual=np.ones((1, 8)))
    assert out3.dtype == np.float16 and out3[0].tolist() == [2.0, 2.0, 0.0, 21.0, 3.0, 4.0, 5.0, 1.5]
    rng = np.random.default_rng(0)
    G, U = rng.standard_normal((5, 64)) * 4, rng.standard_normal((5, 64)) * 4
    ref = (torch.nn.functional.silu(torch.from_numpy(G)) * torch.from_numpy(U)).numpy()
    got = oracle.epilogue(np.concatenate([G, U], axis=1), act="silu_mul").astype(np.float64)
    assert np.allclose(got, ref, rtol=1e-3, atol=1e-3)
