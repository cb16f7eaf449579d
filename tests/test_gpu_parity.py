"""GPU parity tests: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs.

Packing is compared bit for bit; GEMM outputs element by element under the acceptance rule
|Y - Yref| <= 1e-2 + 5e-3*|Yref| and relative Frobenius error <= 2e-3 (helpers.acceptance)."""
import sys

import numpy as np
import pytest

from workloads import w4a16 as wl
from helpers import acceptance
import gpu_util as gu

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def tm():
    import torch
    import paper_2508_15601_amd as tm
    assert torch.cuda.is_available(), "GPU tests need a device"
    tm.load_library()                       # fails loudly if the HIP library was not built
    yield tm
    tm.tm_set_variant(-1, 0)
    tm.tm_set_launch(0, 0)


def _random_problem(seed, M, K, N, g):
    case = wl.Case(f"rand_{M}x{K}x{N}g{g}", M, K, N, g, seed=seed)
    return wl.make(case)


# ------------------------------------------------------------------ packing: bit-exact

# small and ragged shapes, then the weight matrix of every benchmark configuration (11008 rows = 86 packed units,
# the one unit count that is not a power of two)
PACK_SHAPES = [(128, 16, 128), (384, 80, 64), (256, 48, 32), (512, 512, 128), (1152, 272, 128),
               (4096, 4096, 128), (4096, 12288, 128), (4096, 22016, 128), (11008, 4096, 128), (8192, 28672, 128),
               (8192, 8192, 64)]


@pytest.mark.parametrize("K,N,g", PACK_SHAPES)
def test_pack_bit_exact_against_oracle_unpack(tm, oracle, K, N, g):
    _say(f"pack K={K} N={N} g={g}")
    rng = np.random.default_rng(K * 7 + N)
    q = rng.integers(0, 16, (K, N), dtype=np.uint8)
    # position codes in a second pass so that every nibble slot is distinguished
    kk, nn = np.arange(K, dtype=np.int32)[:, None], np.arange(N, dtype=np.int32)[None, :]
    for qq in (q, ((kk * 5 + nn * 3 + (kk >> 3) + (nn >> 4)) & 15).astype(np.uint8)):
        s = rng.uniform(0.001, 0.02, (K // g, N)).astype(np.float16)
        z = rng.integers(0, 16, (K // g, N)).astype(np.float16)
        d = {"q": qq, "s": s, "z": z, "qweight": wl.pack_interchange(qq)}
        packed = gu.pack(d, g)
        wbuf, szbuf = tm.tm_packed_raw(packed)
        q2, s2, z2 = oracle.unpack_packed(wbuf, szbuf, K, N, g)
        assert np.array_equal(q2, qq)
        assert np.array_equal(s2.view(np.uint16), s.view(np.uint16))
        assert np.array_equal(z2.view(np.uint16), z.view(np.uint16))
        # device-side inverse permutation returns the interchange words
        qw, sd, zd = tm.tm_unpack_w4(packed)
        assert np.array_equal(qw.cpu().numpy().view(np.uint32), d["qweight"])
        assert np.array_equal(sd.cpu().numpy().view(np.uint16), s.view(np.uint16))
        assert np.array_equal(zd.cpu().numpy().view(np.uint16), z.view(np.uint16))
        packed.close()


def test_pack_round_trips_on_random_shapes(tm, oracle):
    """Sixteen shapes drawn at random (K a multiple of 128 up to 2048, N a multiple of 16 up to 1264, every group size,
    every interchange layout): the oracle's inverse of the library layout returns the codes, and the library's own
    inverse returns the canonical words."""
    import torch
    rng = np.random.default_rng(2024)
    for it in range(16):
        g = int(rng.choice([32, 64, 128]))
        K = 128 * int(rng.integers(1, 17))
        N = 16 * int(rng.integers(1, 80))
        layout = int(rng.integers(0, 3))
        if layout != 0:
            N = max(N // 16 * 16, 16)
        _say(f"random pack #{it}: K={K} N={N} g={g} layout={layout}")
        q = rng.integers(0, 16, (K, N), dtype=np.uint8)
        s = rng.uniform(0.001, 0.02, (K // g, N)).astype(np.float16)
        z = rng.integers(0, 16, (K // g, N)).astype(np.float16)
        if layout == 0:
            packed = gu.pack({"q": q, "qweight": wl.pack_interchange(q), "s": s, "z": z}, g)
        else:
            if N % 8:
                continue
            qw, zs = wl.encode_layout(q, z, layout)
            packed = tm.tm_pack_w4_layout(torch.from_numpy(qw.view(np.int32)).cuda(), gu.to_dev(s),
                                          torch.from_numpy(zs.view(np.int32)).cuda(), K, N, g, layout)
        wbuf, szbuf = tm.tm_packed_raw(packed)
        q2, s2, z2 = oracle.unpack_packed(wbuf, szbuf, K, N, g)
        assert np.array_equal(q2, q)
        assert np.array_equal(s2.view(np.uint16), s.view(np.uint16)) and np.array_equal(z2.view(np.uint16), z.view(np.uint16))
        qw2, _, _ = tm.tm_unpack_w4(packed)
        assert np.array_equal(qw2.cpu().numpy().view(np.uint32), wl.pack_interchange(q))
        packed.close()


@pytest.mark.parametrize("layout", [0, 1, 2])
@pytest.mark.parametrize("K,N,g", [(128, 16, 128), (256, 48, 32), (384, 2064, 64), (1024, 272, 128)])
def test_pack_layouts_bit_exact(tm, oracle, K, N, g, layout):
    """Every interchange layout packs to the same fragment-ordered buffer: checked through the oracle's inverse
    map (paper Sec. 4.1) and against the canonical-layout pack, bit for bit."""
    import torch
    _say(f"pack layout={layout} K={K} N={N} g={g}")
    rng = np.random.default_rng(K * 11 + N + layout)
    kk, nn = np.meshgrid(np.arange(K), np.arange(N), indexing="ij")
    for qq in (rng.integers(0, 16, (K, N), dtype=np.uint8),
               ((kk * 5 + nn * 3 + (kk >> 3) + (nn >> 4)) & 15).astype(np.uint8)):
        s = rng.uniform(0.001, 0.02, (K // g, N)).astype(np.float16)
        z = rng.integers(0, 16, (K // g, N)).astype(np.float16)
        qw, zs = wl.encode_layout(qq, z, layout)
        zt = gu.to_dev(zs) if layout == 0 else torch.from_numpy(zs.view(np.int32)).cuda()
        packed = tm.tm_pack_w4_layout(torch.from_numpy(qw.view(np.int32)).cuda(), gu.to_dev(s), zt, K, N, g, layout)
        wbuf, szbuf = tm.tm_packed_raw(packed)
        q2, s2, z2 = oracle.unpack_packed(wbuf, szbuf, K, N, g)
        assert np.array_equal(q2, qq)
        assert np.array_equal(s2.view(np.uint16), s.view(np.uint16))
        assert np.array_equal(z2.view(np.uint16), z.view(np.uint16))
        ref = gu.pack({"q": qq, "qweight": wl.pack_interchange(qq), "s": s, "z": z}, g)
        wref, szref = tm.tm_packed_raw(ref)
        assert np.array_equal(wbuf, wref) and np.array_equal(szbuf, szref)
        packed.close(); ref.close()


@pytest.mark.parametrize("K,N,g,M", [(512, 48, 256, 5), (1024, 272, 1024, 3), (768, 528, 384, 40), (2048, 1040, 2048, 300)])
@pytest.mark.parametrize("symmetric", [False, True])
def test_coarse_groups_and_symmetric(tm, oracle, K, N, g, M, symmetric):
    """Groups coarser than 128 rows (up to one scale per channel) and symmetric weights (zero-point 8, passed as
    no zeros at all): the stored buffer holds the repeated rows, and the GEMM matches the oracle run with the
    caller's own group size."""
    import torch
    _say(f"coarse group K={K} N={N} g={g} M={M} symmetric={symmetric}")
    rng = np.random.default_rng(K + N + g)
    q = rng.integers(0, 16, (K, N), dtype=np.uint8)
    s = rng.uniform(0.001, 0.02, (K // g, N)).astype(np.float16)
    z = np.full((K // g, N), 8, np.float16) if symmetric else rng.integers(0, 16, (K // g, N)).astype(np.float16)
    X = rng.standard_normal((M, K)).astype(np.float16)
    packed = tm.tm_pack_w4(gu.to_dev(wl.pack_interchange(q)), gu.to_dev(s), None if symmetric else gu.to_dev(z), K, N, g)
    assert packed.group == 128
    wbuf, szbuf = tm.tm_packed_raw(packed)
    q2, s2, z2 = oracle.unpack_packed(wbuf, szbuf, K, N, 128)
    assert np.array_equal(q2, q)
    assert np.array_equal(s2.view(np.uint16), np.repeat(s, g // 128, axis=0).view(np.uint16))
    assert np.array_equal(z2.view(np.uint16), np.repeat(z, g // 128, axis=0).view(np.uint16))
    Y = gu.gemm(packed, X)
    ok, worst, fro = acceptance(Y, oracle.gemm(X, q, s, z, g))
    assert ok, (worst, fro)
    packed.close()


@pytest.mark.parametrize("layout", [1, 2])
def test_gemm_from_layouts(tm, oracle, layout):
    """End to end from a non-canonical checkpoint layout: pack, multiply, compare with the oracle GEMM."""
    import torch
    case = wl.Case("layout", 24, 1024, 528, 64, seed=77 + layout)
    _say(f"gemm layout={layout} {case}")
    d = wl.make(case)
    qw, zs = wl.encode_layout(d["q"], d["z"], layout)
    packed = tm.tm_pack_w4_layout(torch.from_numpy(qw.view(np.int32)).cuda(), gu.to_dev(d["s"]),
                                  torch.from_numpy(zs.view(np.int32)).cuda(), case.K, case.N, case.group, layout)
    X = gu.to_dev(d["X"])
    Y = torch.empty((case.M, case.N), dtype=torch.float16, device="cuda")
    tm.tm_gemm_w4a16(X, packed, Y)
    torch.cuda.synchronize()
    Yref = oracle.gemm(d["X"], d["q"], d["s"], d["z"], case.group)
    ok, worst, fro = acceptance(Y.cpu().numpy(), Yref)
    assert ok, (layout, worst, fro)
    packed.close()


# ------------------------------------------------------------------ GEMM: exact special cases

@pytest.mark.parametrize("variant", [-1] + list(range(24)))
def test_one_hot_rows_return_dequantised_weights_bit_exactly(tm, oracle, variant):
    """X = one-hot rows: a single non-zero product per output, so the fp16-dequantised weight must come back
    exactly; pins layout, nibble order, group indexing and the conversion constants on the device."""
    K, N, g = 384, 80, 64
    d = _random_problem(5, 1, K, N, g)
    packed = gu.pack(d, g)
    tm.tm_set_variant(variant, 0)
    for k0 in range(0, K, 16):
        rows = list(range(k0, k0 + 16))
        X = np.zeros((len(rows), K), np.float16)
        X[np.arange(len(rows)), rows] = 1.0
        _say(f"one-hot variant={variant} k0={k0}")
        Y = gu.gemm(packed, X)
        Yref = oracle.gemm(X, d["q"], d["s"], d["z"], g)
        assert np.array_equal(Y.view(np.uint16), Yref.view(np.uint16))
    tm.tm_set_variant(-1, 0)


@pytest.mark.parametrize("M,variant,split", [(4, -1, 0), (4, 0, 3), (12, 1, 2), (16, 2, 1), (30, 3, 1), (30, 4, 3),
                                             (40, -1, 0), (31, 5, 1), (60, 6, 2), (100, 7, 0), (200, 7, 2),
                                             (100, 8, 1)])
def test_integer_exact_case(tm, oracle, M, variant, split):
    """s = 1 and small integer activations: every partial sum is an exactly representable integer, so any
    summation order gives the oracle's bits."""
    rng = np.random.default_rng(M)
    K, N, g = 384, 112, 128
    q = rng.integers(0, 16, (K, N), dtype=np.uint8)
    z = rng.integers(0, 16, (K // g, N)).astype(np.float16)
    s = np.ones((K // g, N), np.float16)
    X = (rng.integers(-1, 2, (M, K)) * (rng.random((M, K)) < 0.25)).astype(np.float16)
    d = {"q": q, "s": s, "z": z, "qweight": wl.pack_interchange(q)}
    packed = gu.pack(d, g)
    tm.tm_set_variant(variant, split)
    _say(f"integer-exact M={M} variant={variant} split={split} plan={tm.tm_get_plan(packed, M)}")
    Y = gu.gemm(packed, X)
    tm.tm_set_variant(-1, 0)
    Yref = oracle.gemm(X, q, s, z, g)
    assert np.abs(Yref.astype(np.float64)).max() < 2048
    assert np.array_equal(Y.view(np.uint16), Yref.view(np.uint16))


# The two prefill tiles exist with the 16x16x32 and with the 32x32x16 matrix instruction (the latter on request only):
# both forms of both tiles, exact cases first.
@pytest.mark.parametrize("shape", [16, 32])
@pytest.mark.parametrize("variant", [7, 12])
def test_prefill_tiles_both_mfma_shapes_exact_cases(tm, oracle, variant, shape):
    K, N, g = 384, 80, 64
    d = _random_problem(5, 1, K, N, g)
    packed = gu.pack(d, g)
    tm.tm_set_variant(variant, 1)
    tm.tm_set_launch(4 if variant == 7 else 8, 0)        # one wave set (a launch this small would take two)
    tm.tm_set_mfma_shape(shape)
    try:
        plan = tm.tm_get_plan(packed, 16)
        _say(f"mfma shape={shape} variant={variant} plan={plan}")
        assert plan["variant"] == variant and plan["mfma_shape"] == shape
        for k0 in range(0, K, 16):                       # one-hot rows: the dequantised weights come back exactly
            X = np.zeros((16, K), np.float16)
            X[np.arange(16), np.arange(k0, k0 + 16)] = 1.0
            Y = gu.gemm(packed, X)
            assert np.array_equal(Y.view(np.uint16), oracle.gemm(X, d["q"], d["s"], d["z"], g).view(np.uint16)), k0
        rng = np.random.default_rng(variant + shape)     # unit scales, small integers: any summation order is exact
        M, K2, N2, g2 = 150, 512, 1040, 128
        q = rng.integers(0, 16, (K2, N2), dtype=np.uint8)
        z = rng.integers(0, 16, (K2 // g2, N2)).astype(np.float16)
        s1 = np.ones((K2 // g2, N2), np.float16)
        X = (rng.integers(-1, 2, (M, K2)) * (rng.random((M, K2)) < 0.25)).astype(np.float16)
        packed2 = gu.pack({"q": q, "s": s1, "z": z, "qweight": wl.pack_interchange(q)}, g2)
        Y = gu.gemm(packed2, X)
        Yref = oracle.gemm(X, q, s1, z, g2)
        assert np.abs(Yref.astype(np.float64)).max() < 2048
        assert np.array_equal(Y.view(np.uint16), Yref.view(np.uint16))
    finally:
        tm.tm_set_variant(-1, 0)
        tm.tm_set_launch(0, 0)
        tm.tm_set_mfma_shape(0)


@pytest.mark.parametrize("shape", [16, 32])
@pytest.mark.parametrize("variant", [7, 12])
@pytest.mark.parametrize("M,K,N,g", [(130, 1152, 528, 64), (300, 640, 400, 128), (257, 384, 272, 32), (128, 2816, 1040, 128),
                                     (513, 1024, 1552, 64)])
def test_prefill_tiles_both_mfma_shapes(tm, oracle, variant, shape, M, K, N, g):
    """Ragged rows and columns, every group size, K of 3 ... 22 packed units, several CTA tiles in both directions."""
    d = _random_problem(variant * 7 + shape + M, M, K, N, g)
    packed = gu.pack(d, g)
    tm.tm_set_variant(variant, 1)
    tm.tm_set_launch(4 if variant == 7 else 8, 0)        # one wave set (a launch this small would take two)
    tm.tm_set_mfma_shape(shape)
    try:
        plan = tm.tm_get_plan(packed, M)
        _say(f"mfma shape={shape} variant={variant} M={M} K={K} N={N} g={g} plan={plan}")
        assert plan["variant"] == variant and plan["mfma_shape"] == shape
        Y = gu.gemm(packed, d["X"])
        Y2 = gu.gemm(packed, d["X"])
    finally:
        tm.tm_set_variant(-1, 0)
        tm.tm_set_launch(0, 0)
        tm.tm_set_mfma_shape(0)
    ok, worst, fro = acceptance(Y, oracle.gemm(d["X"], d["q"], d["s"], d["z"], g))
    assert ok, (worst, fro)
    assert np.array_equal(Y.view(np.uint16), Y2.view(np.uint16))


# ------------------------------------------------------------------ GEMM: tolerance parity on ragged small shapes

SMALL = [
    # M, K, N, group           several tiles in every dimension plus ragged tails
    (1, 128, 16, 128), (3, 384, 80, 64), (16, 1152, 272, 128), (17, 384, 528, 32), (33, 1152, 80, 128),
    (64, 640, 272, 64), (65, 384, 272, 128), (130, 1152, 528, 64), (300, 640, 400, 128), (257, 384, 272, 32),
    # more than eight column tiles per compute unit: decode strips in two whole rounds
    (5, 512, 33040, 128), (16, 384, 41008, 64),
]


@pytest.mark.parametrize("M,K,N,g", SMALL)
def test_small_shapes_auto_plan(tm, oracle, M, K, N, g):
    d = _random_problem(M + K + N, M, K, N, g)
    packed = gu.pack(d, g)
    _say(f"small auto M={M} K={K} N={N} g={g} plan={tm.tm_get_plan(packed, M)}")
    Y = gu.gemm(packed, d["X"])
    Yref = oracle.gemm(d["X"], d["q"], d["s"], d["z"], g)
    ok, worst, fro = acceptance(Y, Yref)
    assert ok, (worst, fro)


@pytest.mark.parametrize("seed", range(36))
def test_random_layer_shapes_auto_plan(tm, oracle, seed):
    """Layer-sized shapes drawn at random (K 1536 ... 28672, N 256 ... 12288, every row-count regime): whatever plan the
    dispatcher's cost models pick - strip width and K split of the decode kernels, tile shape and wave sets above 64
    rows - must launch and meet the oracle.  Codes, zero-points and scales are drawn directly (no quantiser run)."""
    rng = np.random.default_rng(4000 + seed)
    if seed < 18:
        K = 128 * int(rng.integers(12, 113))
        N = 16 * int(rng.integers(64, 769))
    else:                                        # deep and narrow: K up to 28672, the K-split plans
        K = 128 * int(rng.integers(64, 225))
        N = 16 * int(rng.integers(16, 129))
    while K * N > 36_000_000:
        N = (N // 32) * 16
    g = int(rng.choice([32, 64, 128, 128]))
    M = int([1, 5, 16, 24, 32, 48, 64, 96, 128, 200, 384, 512, 17, 33, 65, 300, 8, 256][seed % 18])
    q = rng.integers(0, 16, (K, N), dtype=np.uint8)
    z = rng.integers(0, 16, (K // g, N)).astype(np.float16)
    s = (rng.random((K // g, N)) * 0.02 + 0.001).astype(np.float16)
    X = rng.standard_normal((M, K)).astype(np.float16)
    d = {"q": q, "s": s, "z": z, "X": X, "qweight": wl.pack_interchange(q)}
    packed = gu.pack(d, g)
    plan = tm.tm_get_plan(packed, M)
    _say(f"random layer seed={seed} M={M} K={K} N={N} g={g} plan={plan}")
    Y = gu.gemm(packed, X)
    Yref = oracle.gemm(X, q, s, z, g)
    ok, worst, fro = acceptance(Y, Yref)
    assert ok, (worst, fro, plan)
    packed.close()


@pytest.mark.parametrize("variant,split,waves", [(0, 1, 8), (0, 2, 16), (0, 5, 8), (1, 1, 16), (1, 3, 8), (2, 1, 8),
                                                 (2, 2, 16), (3, 1, 8), (3, 3, 16), (4, 1, 16), (4, 2, 8), (5, 1, 0),
                                                 (5, 3, 0), (6, 1, 0), (6, 2, 0), (7, 1, 0), (7, 3, 0), (8, 1, 0),
                                                 (8, 2, 0), (9, 1, 0), (9, 2, 0), (10, 1, 0), (10, 3, 0),
                                                 (11, 1, 0), (11, 2, 0), (12, 1, 0), (12, 2, 0), (12, 3, 0), (13, 1, 0), (13, 2, 0),
                                                 (14, 1, 8), (14, 2, 16), (15, 1, 16), (15, 3, 0), (15, 1, 8), (16, 1, 0), (16, 2, 16), (16, 2, 8),
                                                 (17, 1, 0), (17, 2, 0), (18, 1, 0), (18, 3, 0), (19, 1, 0), (19, 2, 0),
                                                 (20, 1, 0), (20, 2, 0), (21, 1, 0), (21, 3, 0),
                                                 (22, 1, 0), (22, 2, 4), (23, 1, 0), (23, 3, 8)])
@pytest.mark.parametrize("g,stage", [(32, 0), (64, 2), (128, 4), (64, 8)])
def test_every_variant_and_split(tm, oracle, variant, split, waves, g, stage):
    M = {0: 13, 1: 9, 2: 16, 3: 29, 4: 32, 5: 30, 6: 50, 8: 300, 9: 70, 11: 200, 12: 130, 13: 33, 14: 7, 15: 16, 16: 11, 17: 40, 18: 64, 19: 57, 20: 30, 21: 60, 22: 61, 23: 120}.get(variant, 150)
    tm.tm_set_launch(waves, stage)
    K, N = 1152, 336
    d = _random_problem(variant * 10 + split, M, K, N, g)
    packed = gu.pack(d, g)
    tm.tm_set_variant(variant, split)
    plan = tm.tm_get_plan(packed, M)
    _say(f"variant={variant} split={split} g={g} plan={plan}")
    assert plan["variant"] == variant
    Y = gu.gemm(packed, d["X"])
    Y2 = gu.gemm(packed, d["X"])
    tm.tm_set_variant(-1, 0)
    tm.tm_set_launch(0, 0)
    Yref = oracle.gemm(d["X"], d["q"], d["s"], d["z"], g)
    ok, worst, fro = acceptance(Y, Yref)
    assert ok, (worst, fro)
    assert np.array_equal(Y.view(np.uint16), Y2.view(np.uint16)), "split-K reduction must be run-to-run deterministic"


# The decode shapes (M <= 16) have a one-shot and a ring-buffered form of their kernels: both forms of every strip width,
# CTAs of 8 and 16 waves, K ranges that leave some waves a unit short, strips of two widths, K split across CTAs.
@pytest.mark.parametrize("form", ["one_shot", "ring"])
@pytest.mark.parametrize("variant", [0, 1, 14, 2, 15, 16])
@pytest.mark.parametrize("M,K,N,g,waves,split", [(1, 1152, 336, 128, 16, 1), (5, 2048, 528, 64, 8, 1), (16, 1536, 1040, 32, 16, 2),
                                                 (13, 4096, 272, 128, 16, 1), (8, 2560, 2064, 128, 8, 3), (16, 1024, 80, 64, 16, 1)])
def test_decode_kernel_forms(tm, oracle, form, variant, M, K, N, g, waves, split):
    d = _random_problem(variant * 31 + M + K, M, K, N, g)
    packed = gu.pack(d, g)
    tm.tm_set_variant(variant, split)
    tm.tm_set_launch(waves, 1 if form == "ring" else 0)
    try:
        plan = tm.tm_get_plan(packed, M)
        _say(f"decode form={form} variant={variant} M={M} K={K} N={N} g={g} waves={waves} split={split} plan={plan}")
        assert plan["variant"] == variant
        if form == "ring":
            assert plan["one_shot_units_per_wave"] == 0
        Y = gu.gemm(packed, d["X"])
        Y2 = gu.gemm(packed, d["X"])
    finally:
        tm.tm_set_variant(-1, 0)
        tm.tm_set_launch(0, 0)
    ok, worst, fro = acceptance(Y, oracle.gemm(d["X"], d["q"], d["s"], d["z"], g))
    assert ok, (plan, worst, fro)
    assert np.array_equal(Y.view(np.uint16), Y2.view(np.uint16))
    packed.close()


def _x_ring_built(M, ntw, g, kus, NT):
    """The library's rule for which X-ring kernels exist, restated: registers for the weights in flight, the accumulators
    and one step of fragments within 128 per lane (CTAs of 16 waves, two row tiles only) or 250 (CTAs of 8 waves)."""
    tm_rows, gpu = (2 if M <= 32 else 4), 128 // g
    ntw = -(-NT // -(-NT // ntw))                       # widest strip after the tiles are dealt evenly
    for waves in ((16, 8) if tm_rows == 2 else (8,)):
        ni = next((b for b in (1, 2, 3, 4, 6, 8) if b >= -(-kus // waves)), None)
        if ni is None:
            continue
        regs = ni * ntw * (4 + gpu) + tm_rows * ntw * 4 + 4 * tm_rows + 3 * ntw + 24
        if (regs <= 128 if waves == 16 else (regs <= 250 if tm_rows == 4 else 128 < regs <= 250)):
            return True
    return False


# 16 < M <= 64: the one-shot kernels with a ring of X pieces per wave (two row tiles per wave up to M = 32, four beyond).  A forced 16-row variant fixes the strip width;
# every width, CTAs of 8 and 16 waves, K ranges that leave waves a unit short or without any, strips of two widths, K
# split across CTAs, both group sizes the kernels are built for, the smallest and the largest row count.
@pytest.mark.parametrize("variant", [0, 1, 14, 2, 15, 16])
@pytest.mark.parametrize("M,K,N,g,split", [(17, 1152, 336, 128, 1), (32, 2048, 528, 64, 1), (24, 1536, 1040, 128, 2),
                                           (31, 4096, 272, 128, 1), (32, 2560, 2064, 64, 3), (20, 1024, 80, 64, 1),
                                           (32, 8192, 512, 128, 1), (33, 1152, 336, 128, 1), (64, 2048, 528, 64, 2),
                                           (50, 4096, 272, 128, 1), (64, 1536, 1040, 64, 3), (47, 11008, 256, 128, 4)])
def test_decode_kernels_with_x_ring(tm, oracle, variant, M, K, N, g, split):
    d = _random_problem(variant * 37 + M + K, M, K, N, g)
    packed = gu.pack(d, g)
    tm.tm_set_variant(variant, split)
    tm.tm_set_launch(0, 0)                  # 16 waves per CTA where a wave's share fits 128 registers, else 8
    try:
        plan = tm.tm_get_plan(packed, M)
        _say(f"x-ring variant={variant} M={M} K={K} N={N} g={g} split={split} plan={plan}")
        # where a wave's share of the weights exceeds its registers even in CTAs of 8 waves no such kernel is built and
        # the ring-buffered form takes the launch
        assert (plan["one_shot_units_per_wave"] > 0) == _x_ring_built(M, {0: 1, 1: 2, 14: 3, 2: 4, 15: 6, 16: 8}[variant], g,
                                                                      -(-(K // 128) // split), N // 16), plan
        Y = gu.gemm(packed, d["X"])
        Y2 = gu.gemm(packed, d["X"])
    finally:
        tm.tm_set_variant(-1, 0)
        tm.tm_set_launch(0, 0)
    ok, worst, fro = acceptance(Y, oracle.gemm(d["X"], d["q"], d["s"], d["z"], g))
    assert ok, (plan, worst, fro)
    assert np.array_equal(Y.view(np.uint16), Y2.view(np.uint16))
    packed.close()


def test_x_ring_form_is_taken_and_exact(tm, oracle):
    """The benchmark's narrow layers at M = 32 and 64 run the X-ring kernels (one_shot_units_per_wave > 0 in the plan; the
    deepest one at M = 64 takes split CTA tiles instead), and those kernels give the oracle's bits on integer-exact and
    one-hot inputs."""
    import torch
    for K, N, g in ((11008, 4096, 128), (8192, 8192, 64)):
        qw = torch.zeros((K, N // 8), dtype=torch.int32, device="cuda")
        s = torch.ones((K // g, N), dtype=torch.float16, device="cuda")
        packed = tm.tm_pack_w4(qw, s, None, K, N, g)
        for M in (32, 64):
            plan = tm.tm_get_plan(packed, M)
            _say(f"x-ring plan K={K} N={N} M={M}: {plan}")
            if (K, M) == (11008, 64):
                # deep and narrow at 33 ... 64 rows: 64 x 64 CTA tiles with K split in four outrun the X ring there
                assert plan["name"] == "tile64x64" and plan["split_k"] == 4, plan
            else:
                assert plan["one_shot_units_per_wave"] > 0, (K, N, M, plan)
        packed.close()
    rng = np.random.default_rng(5)
    M, K, N, g = 29, 1280, 400, 128
    q = rng.integers(0, 16, (K, N), dtype=np.uint8)
    z = rng.integers(0, 16, (K // g, N)).astype(np.float16)
    s = np.exp2(rng.integers(-3, 2, (K // g, N))).astype(np.float16)         # power-of-two scales: every product exact
    X = rng.integers(-3, 4, (M, K)).astype(np.float16)
    X[5] = 0
    X[5, 777] = 1                                                           # a one-hot row picks out one dequantised row
    d = {"q": q, "s": s, "z": z, "X": X, "qweight": wl.pack_interchange(q)}
    packed = gu.pack(d, g)
    plan = tm.tm_get_plan(packed, M)
    assert plan["one_shot_units_per_wave"] > 0, plan
    Y = gu.gemm(packed, X)
    Yref = oracle.gemm(X, q, s, z, g)
    assert np.array_equal(Y.view(np.uint16), Yref.view(np.uint16))
    packed.close()


def test_decode_configs_take_the_one_shot_form(tm):
    """The benchmark's decode layers (M <= 16) and deep or narrow layers of other models run the one-shot kernels."""
    import torch
    for K, N, g, Ms in ((4096, 4096, 128, (1, 16)), (4096, 12288, 128, (1, 16)), (4096, 22016, 128, (1, 16)),
                        (11008, 4096, 128, (1, 8, 16)), (8192, 8192, 64, (1, 8, 16)),
                        # layers of other models: deep K, or fewer column tiles than compute units (K split across CTAs)
                        (13824, 5120, 128, (1, 16)), (18944, 3584, 128, (1, 16)),
                        # more column tiles than eight per compute unit: two whole rounds of strips
                        (3584, 37888, 128, (1, 16))):
        qw = torch.zeros((K, N // 8), dtype=torch.int32, device="cuda")
        s = torch.ones((K // g, N), dtype=torch.float16, device="cuda")
        packed = tm.tm_pack_w4(qw, s, None, K, N, g)
        for M in Ms:
            plan = tm.tm_get_plan(packed, M)
            _say(f"decode plan K={K} N={N} M={M}: {plan}")
            assert plan["one_shot_units_per_wave"] > 0, (K, N, M, plan)
        packed.close()


def test_very_deep_decode_layer_splits_k(tm, oracle):
    """K so deep that no split of eight or less brings a CTA's slice of X into LDS, on an output wider than one strip per
    compute unit: the ring-buffered kernel with K split across CTAs.  Integer-valued inputs with power-of-two scales and
    sparse activation rows keep every product and partial sum exact, so the result must equal the oracle's bit for bit."""
    rng = np.random.default_rng(77)
    M, K, N, g = 12, 24576, 4352, 128
    q = rng.integers(0, 16, (K, N), dtype=np.uint8)
    z = rng.integers(0, 16, (K // g, N)).astype(np.float16)
    s = np.exp2(rng.integers(-3, 2, (K // g, N))).astype(np.float16)
    X = np.zeros((M, K), dtype=np.float16)
    for m in range(M):
        X[m, rng.choice(K, 64, replace=False)] = rng.integers(-2, 3, 64).astype(np.float16)
    d = {"q": q, "s": s, "z": z, "X": X, "qweight": wl.pack_interchange(q)}
    packed = gu.pack(d, g)
    plan = tm.tm_get_plan(packed, M)
    _say(f"very deep decode layer K={K} N={N} M={M}: {plan}")
    assert plan["one_shot_units_per_wave"] == 0 and plan["split_k"] >= 2 and plan["name"] == "skinny16x64", plan
    Y = gu.gemm(packed, X)
    Yref = oracle.gemm(X, q, s, z, g)
    assert np.array_equal(Y.view(np.uint16), Yref.view(np.uint16))
    Y2 = gu.gemm(packed, X)
    assert np.array_equal(Y.view(np.uint16), Y2.view(np.uint16))
    packed.close()


# (variant, waves per CTA): 128-column tiles with two or four sets of four waves, 96-column tiles with two or four
# sets of two waves; the 128-row tiles are built with two sets only (the 128 x 256 one hands its set tile over in two parts)
WAVE_SETS = [(13, 8), (13, 16), (9, 8), (9, 16), (10, 8), (7, 8), (20, 4), (20, 8), (21, 4), (21, 8), (22, 4), (22, 8), (23, 4), (23, 8)]


@pytest.mark.parametrize("variant,waves", WAVE_SETS)
@pytest.mark.parametrize("stage", [2, 4, 8])
@pytest.mark.parametrize("g,split", [(32, 1), (64, 2), (128, 1), (128, 3)])
def test_tile_wave_sets(tm, oracle, variant, waves, stage, g, split):
    """Tile kernels with several wave sets per CTA, each set multiplying its own slice of every K stage."""
    M = {13: 33, 9: 70, 10: 150, 7: 200, 20: 31, 21: 50, 22: 59, 23: 128}[variant]
    K, N = 1536, 336                         # 12 packed units: whole stages for every depth up to four units
    d = _random_problem(variant * 100 + waves + stage + split, M, K, N, g)
    packed = gu.pack(d, g)
    tm.tm_set_launch(waves, stage)
    tm.tm_set_variant(variant, split)
    plan = tm.tm_get_plan(packed, M)
    _say(f"wave sets variant={variant} waves={waves} stage={stage} g={g} split={split} plan={plan}")
    assert plan["variant"] == variant
    assert plan["block"] == waves * 64
    Y = gu.gemm(packed, d["X"])
    Y2 = gu.gemm(packed, d["X"])
    tm.tm_set_variant(-1, 0)
    tm.tm_set_launch(0, 0)
    Yref = oracle.gemm(d["X"], d["q"], d["s"], d["z"], g)
    ok, worst, fro = acceptance(Y, Yref)
    assert ok, (worst, fro)
    assert np.array_equal(Y.view(np.uint16), Y2.view(np.uint16))


@pytest.mark.parametrize("variant,M", [(22, 100), (22, 250), (23, 130), (13, 40), (9, 120)])
@pytest.mark.parametrize("split", [1, 2])
def test_tile_sets_when_k_is_no_multiple_of_the_full_stage(tm, oracle, variant, M, split):
    """22 packed units along K (a multiple of two, not of four): the tiles that would take four wave sets with 128-deep
    stages must shrink the stage; the two-wave tiles give up two of their sets and keep the depth."""
    K, N, g = 22 * 128, 1040, 128
    d = _random_problem(4100 + variant + M + split, M, K, N, g)
    packed = gu.pack(d, g)
    tm.tm_set_variant(variant, split)
    plan = tm.tm_get_plan(packed, M)
    _say(f"odd stage count variant={variant} M={M} split={split} plan={plan}")
    assert plan["variant"] == variant
    if variant == 22:
        assert plan["block"] == 256, plan               # two sets of two waves (the 128-row tile's stages are 64 deep anyway)
    Y = gu.gemm(packed, d["X"])
    Y2 = gu.gemm(packed, d["X"])
    tm.tm_set_variant(-1, 0)
    Yref = oracle.gemm(d["X"], d["q"], d["s"], d["z"], g)
    ok, worst, fro = acceptance(Y, Yref)
    assert ok, (worst, fro)
    assert np.array_equal(Y.view(np.uint16), Y2.view(np.uint16))


def test_caller_workspace_entry_point(tm, oracle):
    import torch
    M, K, N, g = 20, 1152, 336, 128
    d = _random_problem(77, M, K, N, g)
    packed = gu.pack(d, g)
    tm.tm_set_variant(4, 3)
    need = tm.tm_gemm_workspace_bytes(packed, M)
    ws = torch.zeros(need + 256, dtype=torch.uint8, device="cuda")
    off = (-ws.data_ptr()) % 256
    ws = ws[off:off + need]
    Xd = gu.to_dev(d["X"])
    Y = torch.empty((M, N), dtype=torch.float16, device="cuda")
    for _ in range(2):                       # second call checks the workspace was left ready
        Y.fill_(float("nan"))
        tm.tm_gemm_w4a16_ws(Xd, packed, Y, ws)
        torch.cuda.synchronize()
        ok, worst, fro = acceptance(Y.cpu().numpy(), oracle.gemm(d["X"], d["q"], d["s"], d["z"], g))
        assert ok, (worst, fro)
    with pytest.raises(tm.TmError):
        tm.tm_gemm_w4a16_ws(Xd, packed, Y, ws[:256])
    # counters left part-way by a launch that died are put right by the reset call
    ws[:64].fill_(1)
    tm.tm_reset_workspace(ws)
    Y.fill_(float("nan"))
    tm.tm_gemm_w4a16_ws(Xd, packed, Y, ws)
    torch.cuda.synchronize()
    ok, worst, fro = acceptance(Y.cpu().numpy(), oracle.gemm(d["X"], d["q"], d["s"], d["z"], g))
    assert ok, (worst, fro)
    tm.tm_reset_workspace()                       # the library's own: a no-op on clean counters
    tm.tm_set_variant(-1, 0)


def test_edge_cases(tm, oracle):
    import torch
    d = _random_problem(3, 2, 128, 16, 128)
    packed = gu.pack(d, 128)
    # M = 0 is a no-op
    X0 = torch.empty((0, 128), dtype=torch.float16, device="cuda")
    Y0 = torch.empty((0, 16), dtype=torch.float16, device="cuda")
    tm.tm_gemm_w4a16(X0, packed, Y0)
    # misaligned X is rejected, not launched
    buf = torch.zeros(2 * 128 + 8, dtype=torch.float16, device="cuda")
    Xmis = buf[1:1 + 256].view(2, 128)
    with pytest.raises(tm.TmError):
        tm.tm_gemm_w4a16(Xmis, packed, torch.empty((2, 16), dtype=torch.float16, device="cuda"))
    # M*K beyond the 32-bit byte offsets the kernels use is rejected before anything is launched
    import ctypes
    lib = tm.load_library()
    big = ctypes.c_void_p(buf.data_ptr())
    assert lib.tm_gemm_w4a16(big, packed.handle, big, 1 << 24, None) == -1      # M itself out of range
    assert lib.tm_gemm_w4a16(big, packed.handle, big, -3, None) == -1
    # a freed handle is refused, not dereferenced as valid
    p3 = gu.pack(d, 128)
    h3 = p3.handle
    p3.close()
    with pytest.raises(ValueError):
        _ = p3.handle
    # extreme codes and zero-points: q in {0, 15}, z in {0, 15}
    K, N, g = 256, 32, 64
    rng = np.random.default_rng(0)
    q = (rng.integers(0, 2, (K, N)) * 15).astype(np.uint8)
    z = (rng.integers(0, 2, (K // g, N)) * 15).astype(np.float16)
    s = rng.uniform(0.001, 0.02, (K // g, N)).astype(np.float16)
    X = rng.standard_normal((5, K)).astype(np.float16)
    dd = {"q": q, "s": s, "z": z, "qweight": wl.pack_interchange(q)}
    p2 = gu.pack(dd, g)
    ok, worst, fro = acceptance(gu.gemm(p2, X), oracle.gemm(X, q, s, z, g))
    assert ok, (worst, fro)
    assert lib.tm_gemm_w4a16(big, p2.handle, big, 1 << 23, None) == -1          # M*K = 2^31 with K = 256
    assert "2^31" in tm.tm_last_error()


# ------------------------------------------------------------------ GEMM: the benchmark configurations

def _plan_tile(plan):
    """(rows, columns) of the output tile one CTA of the planned kernel owns, read from the variant's name
    ("tile128x256", "skinny16x48"); a decode strip is dealt in 16-column tiles, so 16 columns is its granule."""
    kind, dims = ("tile", plan["name"][4:]) if plan["name"].startswith("tile") else ("skinny", plan["name"][6:])
    bm, bn = (int(v) for v in dims.split("x"))
    return bm, (bn if kind == "tile" else 16)


def _check_case(tm, oracle, case, d=None, packed=None, full_limit=2.5e10):
    d = d or wl.make(case)
    own = packed is None
    packed = packed or gu.pack(d, case.group)
    X = d["X"][:case.M]
    plan = tm.tm_get_plan(packed, case.M)
    _say(f"{case.name}: M={case.M} K={case.K} N={case.N} g={case.group} plan={plan}")
    Y = gu.gemm(packed, X)
    assert not np.isnan(Y).any()
    # same launch again: the reduction over K splits and wave sets has a fixed order, so the bits must repeat
    Y_again = gu.gemm(packed, X)
    assert np.array_equal(Y.view(np.uint16), Y_again.view(np.uint16)), (case.name, "not run-to-run identical")
    work = float(case.M) * case.K * case.N
    if work <= full_limit:
        Yref = oracle.gemm(X, d["q"], d["s"], d["z"], case.group)
        ok, worst, fro = acceptance(Y, Yref)
        assert ok, (case.name, worst, fro)
    else:
        # Sampled outputs that still meet EVERY output tile of the planned kernel (and with it every K split, since
        # an output sums over all of K): one complete row through each row of tiles and one complete column through
        # each column of tiles, at a random place inside the tile, plus the four edges.  A tile written to the wrong
        # place, or not at all, therefore fails whichever tile it is.
        bm, bn = _plan_tile(plan)
        rng = np.random.default_rng(1)
        starts = np.arange(0, case.M, bm)
        rows = np.unique(np.concatenate([[0, case.M - 1], starts + rng.integers(0, np.minimum(bm, case.M - starts))]))
        Yref_rows = oracle.gemm(X[rows], d["q"], d["s"], d["z"], case.group)
        ok, worst, fro = acceptance(Y[rows], Yref_rows)
        assert ok, (case.name, "rows", worst, fro)
        starts = np.arange(0, case.N, bn)
        cols = np.unique(np.concatenate([[0, case.N - 1], starts + rng.integers(0, np.minimum(bn, case.N - starts))]))
        _say(f"   sampled: {rows.size} rows (one per {bm}-row tile), {cols.size} columns (one per {bn}-column tile)")
        ms = np.repeat(np.arange(case.M), cols.size)
        ns = np.tile(cols, case.M)
        Yref_cols = oracle.gemm_sampled(X, d["q"], d["s"], d["z"], case.group, ms, ns)
        ok, worst, fro = acceptance(Y[ms, ns], Yref_cols)
        assert ok, (case.name, "cols", worst, fro)
    if own:
        packed.close()
    return d


def test_config1_tiny(tm, oracle):
    _check_case(tm, oracle, wl.case_by_name("cfg1_tiny_M1"))


@pytest.mark.parametrize("layer,Ms", [("cfg2_attn_out", (1, 4, 8, 16)), ("cfg2_qkv", (1, 4, 8, 16)),
                                      ("cfg3_gate_up", (1, 16, 32, 64)), ("cfg3_down", (1, 16, 32, 64))])
def test_config2_3_decode_layers(tm, oracle, layer, Ms):
    big = wl.case_by_name(f"{layer}_M{max(Ms)}")
    d = wl.make(big)                           # one weight matrix per layer; X rows are shared by the smaller M
    packed = gu.pack(d, big.group)
    for M in Ms:
        case = wl.Case(f"{layer}_M{M}", M, big.K, big.N, big.group, big.sigma, big.outlier_frac, big.seed)
        _check_case(tm, oracle, case, d=d, packed=packed)
    packed.close()


def test_config5_dispatch_sweep(tm, oracle):
    big = wl.case_by_name("cfg5_sweep_M1024")
    d = wl.make(big)
    packed = gu.pack(d, big.group)
    seen = set()
    for M in (1, 2, 4, 8, 32, 128, 256, 1024):
        case = wl.Case(f"cfg5_sweep_M{M}", M, big.K, big.N, big.group, big.sigma, big.outlier_frac, big.seed)
        _check_case(tm, oracle, case, d=d, packed=packed, full_limit=1e10)
        seen.add(tm.tm_get_plan(packed, M)["variant"])
    assert len(seen) >= 3, "the dispatch should switch kernel variants across the M sweep"
    packed.close()


def test_config4_prefill_sampled(tm, oracle):
    case = wl.case_by_name("cfg4_prefill_70b_mlp")
    _check_case(tm, oracle, case)


def test_hip_graph_replay_matches_eager(tm, oracle):
    """The GEMM allocates nothing and clears its split-K counters itself, so it can be captured into a HIP graph;
    every replay, with eager work in between, must reproduce the eager bits."""
    import torch
    M, K, N, g = 12, 1152, 336, 128
    d = _random_problem(91, M, K, N, g)
    packed = gu.pack(d, g)
    tm.tm_set_variant(0, 3)                       # split-K path: workspace + arrival counters
    Xd = gu.to_dev(d["X"])
    Y_eager = torch.empty((M, N), dtype=torch.float16, device="cuda")
    tm.tm_gemm_w4a16(Xd, packed, Y_eager)
    torch.cuda.synchronize()
    ok, worst, fro = acceptance(Y_eager.cpu().numpy(), oracle.gemm(d["X"], d["q"], d["s"], d["z"], g))
    assert ok, (worst, fro)
    Y_graph = torch.empty_like(Y_eager)
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            tm.tm_gemm_w4a16(Xd, packed, Y_graph)
            tm.tm_gemm_w4a16(Xd, packed, Y_graph)
    for rep in range(4):
        Y_graph.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y_graph.view(torch.int16), Y_eager.view(torch.int16)), f"replay {rep}"
        Y2 = torch.empty_like(Y_eager)
        tm.tm_gemm_w4a16(Xd, packed, Y2)           # eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(Y2.view(torch.int16), Y_eager.view(torch.int16))
    tm.tm_set_variant(-1, 0)


# ------------------------------------------------------------------ grouped (mixture-of-experts) GEMM

def _make_experts(tm, rng, E, K, N, g):
    host, dev = [], []
    for e in range(E):
        q = rng.integers(0, 16, (K, N), dtype=np.uint8)
        s = rng.uniform(0.001, 0.02, (K // g, N)).astype(np.float16)
        z = rng.integers(0, 16, (K // g, N)).astype(np.float16)
        host.append((q, s, z))
        dev.append(gu.pack({"q": q, "qweight": wl.pack_interchange(q), "s": s, "z": z}, g))
    return host, dev


GROUPED_CASES = [
    # E, K, N, g, rows per expert, rows before the first / after the last expert, forced variant (-1: library's choice)
    (4, 512, 272, 128, [0, 1, 17, 5], 0, 0, -1),
    (8, 1024, 2064, 64, [3, 0, 16, 2, 0, 0, 9, 1], 2, 3, -1),
    (3, 256, 48, 32, [40, 0, 70], 0, 1, -1),            # average load picks the 64-row kernels; 70 rows = two passes
    (3, 256, 48, 32, [40, 0, 70], 1, 0, 0),             # 16-row kernel: five passes for the last expert
    (3, 384, 336, 128, [33, 2, 18], 0, 0, 1),
    (2, 512, 1040, 64, [16, 15], 0, 0, 2),
    (2, 512, 1040, 128, [7, 31], 0, 0, 16),
    (5, 256, 528, 128, [20, 0, 0, 45, 1], 0, 0, 4),
    (64, 256, 96, 128, [0] * 20 + [2] + [0] * 30 + [1, 5] + [0] * 11, 0, 0, -1),
    (6, 2048, 512, 128, [1, 1, 1, 1, 1, 1], 0, 0, -1),
    # skewed routing: one expert holds nearly all rows, so the kernel chosen from the average load takes it in passes
    (8, 512, 272, 128, [200, 1, 0, 2, 0, 3, 1, 0], 0, 0, -1),
    (8, 512, 272, 64, [0, 0, 0, 0, 0, 0, 0, 150], 2, 0, -1),
    # prefill-sized loads go through the CTA-tile kernels (64x128, 128x256), also forced on small loads
    (3, 512, 528, 128, [200, 0, 70], 0, 0, -1),
    (2, 256, 272, 64, [300, 260], 3, 2, -1),
    (4, 384, 144, 32, [130, 1, 0, 129], 0, 5, 9),
    (5, 256, 528, 128, [20, 0, 0, 45, 1], 1, 0, 7),
    (70, 256, 96, 128, [0] * 30 + [65] + [0] * 34 + [3, 0, 64, 0, 130], 0, 0, 9),
    (3, 1024, 1040, 64, [257, 128, 1], 0, 0, 7),
]


@pytest.mark.parametrize("E,K,N,g,counts,lead,trail,variant", GROUPED_CASES)
def test_grouped_gemm_against_oracle(tm, oracle, E, K, N, g, counts, lead, trail, variant):
    import torch
    _say(f"grouped E={E} K={K} N={N} g={g} counts={counts} lead={lead} trail={trail} variant={variant}")
    assert len(counts) == E
    rng = np.random.default_rng(E * 1000 + K + N)
    host, dev = _make_experts(tm, rng, E, K, N, g)
    offsets = (lead + np.concatenate([[0], np.cumsum(counts)])).astype(np.int32)
    R = int(offsets[-1]) + trail
    X = rng.standard_normal((R, K)).astype(np.float16)
    group = tm.tm_group_experts(dev)
    Xd, od = gu.to_dev(X), torch.from_numpy(offsets).cuda()
    Yref = oracle.gemm_grouped(X, host, offsets, g)
    owned = ~np.isnan(Yref[:, 0])
    assert owned.sum() == sum(counts)
    # decode-sized loads take the one-shot form of the decode kernels where it fits (stage 0) and their ring-buffered
    # form otherwise, or when asked to (stage 1); both stay under test
    for stage in (0, 1):
        tm.tm_set_variant(variant, 0)
        tm.tm_set_launch(0, stage)
        try:
            outs = []
            for _ in range(2):
                Y = torch.full((R, N), float("nan"), dtype=torch.float16, device="cuda")
                tm.tm_gemm_w4a16_grouped(Xd, group, od, Y)
                torch.cuda.synchronize()
                outs.append(Y.cpu().numpy())
        finally:
            tm.tm_set_variant(-1, 0)
            tm.tm_set_launch(0, 0)
        assert np.array_equal(outs[0].view(np.uint16), outs[1].view(np.uint16))    # run-to-run identical
        assert np.isnan(outs[0][~owned]).all()                                      # unowned rows untouched
        ok, worst, fro = acceptance(outs[0][owned], Yref[owned])
        assert ok, (stage, worst, fro)
    group.close()
    for p in dev:
        p.close()


# the same launch over 8-bit integer and FP8 experts: decode-sized loads (every strip width the dispatcher picks), loads
# taken in passes, prefill-sized loads on both CTA tiles
GROUPED_8BIT_CASES = [
    (4, 512, 272, 128, [0, 1, 17, 5], 0, 0, -1),
    (8, 1024, 2064, 64, [3, 0, 16, 2, 0, 0, 9, 1], 2, 3, -1),
    (3, 256, 48, 32, [40, 0, 70], 0, 1, -1),
    (2, 512, 1040, 128, [7, 31], 0, 0, 16),
    (5, 256, 528, 128, [20, 0, 0, 45, 1], 0, 0, 4),
    (6, 2048, 512, 128, [1, 1, 1, 1, 1, 1], 0, 0, -1),
    (3, 512, 528, 128, [200, 0, 70], 0, 0, -1),
    (2, 256, 272, 64, [300, 260], 3, 2, -1),
    (4, 384, 144, 32, [130, 1, 0, 129], 0, 5, 9),
]


@pytest.mark.parametrize("fmt", ["int8", "fp8"])
@pytest.mark.parametrize("E,K,N,g,counts,lead,trail,variant", GROUPED_8BIT_CASES)
def test_grouped_gemm_8bit_formats_against_oracle(tm, oracle, E, K, N, g, counts, lead, trail, variant, fmt):
    import torch
    _say(f"grouped {fmt} E={E} K={K} N={N} g={g} counts={counts} lead={lead} trail={trail} variant={variant}")
    rng = np.random.default_rng(E * 1000 + K + N + (1 if fmt == "fp8" else 0))
    host, dev = [], []
    for e in range(E):
        if fmt == "int8":
            q, s, z = _w8_case(rng, K, N, g)
            host.append((q, s, z))
            dev.append(_pack_w8(tm, q, s, z, g))
        else:
            q, s = _fp8_case(rng, K, N, g)
            host.append((q, s))
            dev.append(tm.tm_pack_w8_fp8(gu.to_dev(wl.pack_interchange8(q)), gu.to_dev(s), K, N, g))
    offsets = (lead + np.concatenate([[0], np.cumsum(counts)])).astype(np.int32)
    R = int(offsets[-1]) + trail
    X = (rng.standard_normal((R, K)) * (0.25 if fmt == "fp8" else 1.0)).astype(np.float16)
    group = tm.tm_group_experts(dev)
    Xd, od = gu.to_dev(X), torch.from_numpy(offsets).cuda()
    tm.tm_set_variant(variant, 0)
    try:
        outs = []
        for _ in range(2):
            Y = torch.full((R, N), float("nan"), dtype=torch.float16, device="cuda")
            tm.tm_gemm_w4a16_grouped(Xd, group, od, Y)
            torch.cuda.synchronize()
            outs.append(Y.cpu().numpy())
    finally:
        tm.tm_set_variant(-1, 0)
    assert np.array_equal(outs[0].view(np.uint16), outs[1].view(np.uint16))
    # the definition: the plain GEMM of every expert on its own rows, nothing written elsewhere
    owned = np.zeros(R, bool)
    for e in range(E):
        r0, r1 = int(offsets[e]), int(offsets[e + 1])
        if r1 > r0:
            ref = oracle.gemm(X[r0:r1], *host[e], g) if fmt == "int8" else oracle.gemm_fp8(X[r0:r1], *host[e], g)
            ok, worst, fro = acceptance(outs[0][r0:r1], ref)
            assert ok, (e, worst, fro)
            owned[r0:r1] = True
    assert np.isnan(outs[0][~owned]).all()
    group.close()
    for p in dev:
        p.close()


def test_grouped_gemm_rejects_mixed_formats(tm, oracle):
    rng = np.random.default_rng(9)
    _, dev4 = _make_experts(tm, rng, 1, 256, 32, 128)
    q, s, z = _w8_case(rng, 256, 32, 128)
    dev8 = [_pack_w8(tm, q, s, z, 128)]
    qf, sf = _fp8_case(rng, 256, 32, 128)
    devf = [tm.tm_pack_w8_fp8(gu.to_dev(wl.pack_interchange8(qf)), gu.to_dev(sf), 256, 32, 128)]
    for mix in (dev4 + dev8, dev8 + devf):
        with pytest.raises(tm.TmError):
            tm.tm_group_experts(mix)
    for p in dev4 + dev8 + devf:
        p.close()


def test_grouped_gemm_clamps_offsets_and_rejects_mismatched_experts(tm, oracle):
    import torch
    _say("grouped: offsets beyond the buffers, mismatched experts")
    rng = np.random.default_rng(3)
    host, dev = _make_experts(tm, rng, 2, 256, 32, 128)
    other = _make_experts(tm, rng, 1, 256, 48, 128)[1]
    with pytest.raises(tm.TmError):
        tm.tm_group_experts(dev + other)
    group = tm.tm_group_experts(dev)
    R = 6
    X = rng.standard_normal((R, 256)).astype(np.float16)
    offsets = np.array([-4, 2, 50], np.int32)             # reads as [0, 2, 6]
    Y = torch.full((R, 32), float("nan"), dtype=torch.float16, device="cuda")
    tm.tm_gemm_w4a16_grouped(gu.to_dev(X), group, torch.from_numpy(offsets).cuda(), Y)
    torch.cuda.synchronize()
    Yref = oracle.gemm_grouped(X, host, np.array([0, 2, 6]), 128)
    ok, worst, fro = acceptance(Y.cpu().numpy(), Yref)
    assert ok, (worst, fro)
    group.close()
    for p in dev + other:
        p.close()


# ------------------------------------------------------------------ 8-bit weight codes (W8A16)

def _w8_case(rng, K, N, g, symmetric=False):
    q = rng.integers(0, 256, (K, N), dtype=np.uint8)
    s = rng.uniform(0.0001, 0.002, (K // g, N)).astype(np.float16)
    z = np.full((K // g, N), 128, np.float16) if symmetric else rng.integers(0, 256, (K // g, N)).astype(np.float16)
    return q, s, z


def _pack_w8(tm, q, s, z, g, symmetric=False):
    K, N = q.shape
    return tm.tm_pack_w8(gu.to_dev(wl.pack_interchange8(q)), gu.to_dev(s), None if symmetric else gu.to_dev(z), K, N, g)


@pytest.mark.parametrize("K,N,g", [(128, 16, 128), (256, 48, 32), (384, 2064, 64), (1024, 272, 128), (512, 32, 512)])
def test_w8_pack_bit_exact(tm, oracle, K, N, g):
    _say(f"w8 pack K={K} N={N} g={g}")
    rng = np.random.default_rng(K * 13 + N)
    kk, nn = np.meshgrid(np.arange(K), np.arange(N), indexing="ij")
    for q in (rng.integers(0, 256, (K, N), dtype=np.uint8), ((kk * 37 + nn * 11 + (kk >> 2) + (nn >> 4)) & 255).astype(np.uint8)):
        _, s, z = _w8_case(rng, K, N, g)
        packed = _pack_w8(tm, q, s, z, g)
        assert packed.bits == 8 and tm.load_library().tm_packed_bits(packed.handle) == 8
        wbuf, szbuf = tm.tm_packed_raw(packed)
        gs = min(g, 128)
        q2, s2, z2 = oracle.unpack_packed(wbuf, szbuf, K, N, gs, bits=8)
        assert np.array_equal(q2, q)
        assert np.array_equal(s2.view(np.uint16), np.repeat(s, g // gs, axis=0).view(np.uint16))
        assert np.array_equal(z2.view(np.uint16), np.repeat(z, g // gs, axis=0).view(np.uint16))
        packed.close()


W8_VARIANTS = [-1, 0, 1, 14, 2, 15, 16, 4, 19, 13, 9, 7]


@pytest.mark.parametrize("variant", W8_VARIANTS)
def test_w8_one_hot_rows_return_dequantised_weights_bit_exactly(tm, oracle, variant):
    """X = one-hot rows: Y[m] must equal row k_m of (q - z) * s rounded once to fp16, whatever the kernel."""
    _say(f"w8 one-hot variant={variant}")
    K, N, g, M = 512, 272, 64, 16
    rng = np.random.default_rng(31 + variant)
    q, s, z = _w8_case(rng, K, N, g)
    packed = _pack_w8(tm, q, s, z, g)
    X = np.zeros((M, K), np.float16)
    ks = rng.integers(0, K, M)
    X[np.arange(M), ks] = 1.0
    tm.tm_set_variant(variant, 0)
    try:
        Y = gu.gemm(packed, X)
    finally:
        tm.tm_set_variant(-1, 0)
    What = oracle.dequant(q, s, z, g)
    assert np.array_equal(Y.view(np.uint16), What[ks].astype(np.float16).view(np.uint16))
    packed.close()


@pytest.mark.parametrize("g", [32, 64, 128])
@pytest.mark.parametrize("M,K,N,variant,split", [
    (1, 1024, 528, -1, 0), (7, 768, 4112, -1, 0), (16, 2048, 1040, -1, 0), (16, 512, 48, 0, 0), (9, 1280, 336, 1, 2),
    (13, 1024, 1552, 14, 0), (16, 1024, 1040, 2, 3), (5, 896, 1552, 15, 0), (16, 640, 2064, 16, 0),
    (23, 1024, 1040, -1, 0), (32, 1536, 528, 4, 2), (33, 1024, 272, -1, 0), (64, 768, 1040, 19, 0),
    (100, 512, 272, -1, 0), (300, 1024, 528, -1, 0),
    # CTA-tile kernels of the 8-bit formats: forced shapes, ragged M and N, split-K
    (200, 1024, 1040, 7, 0), (70, 768, 528, 9, 2), (130, 512, 272, 13, 3), (257, 1536, 2064, 7, 2), (96, 2048, 336, 9, 0)])
def test_w8_gemm_against_oracle(tm, oracle, M, K, N, variant, split, g):
    _say(f"w8 gemm M={M} K={K} N={N} g={g} variant={variant} split={split}")
    rng = np.random.default_rng(M + K + N + g)
    q, s, z = _w8_case(rng, K, N, g)
    X = rng.standard_normal((M, K)).astype(np.float16)
    packed = _pack_w8(tm, q, s, z, g)
    tm.tm_set_variant(variant, split)
    try:
        for waves in (0, 8, 16):     # decode kernels: waves per CTA; CTA tiles: two and four wave sets
            tm.tm_set_launch(waves, 0)
            Y = gu.gemm(packed, X)
            ok, worst, fro = acceptance(Y, oracle.gemm(X, q, s, z, g))
            assert ok, (waves, worst, fro)
    finally:
        tm.tm_set_variant(-1, 0)
        tm.tm_set_launch(0, 0)
    packed.close()


def test_w8_quantised_weights_symmetric_and_per_channel(tm, oracle):
    """End to end from fp32 weights through the 8-bit recipe; symmetric packing without a zeros tensor; one scale per
    output channel; and the handle kinds that take 4-bit weights only."""
    _say("w8 recipe / symmetric / per-channel")
    rng = np.random.default_rng(77)
    K, N, M = 1024, 528, 12
    W = (0.02 * rng.standard_normal((K, N))).astype(np.float32)
    X = rng.standard_normal((M, K)).astype(np.float16)
    for g in (128, K):
        q, s, z = wl.quantise_recipe(W, g, bits=8)
        packed = _pack_w8(tm, q, s, z, g)
        Yref = oracle.gemm(X, q, s, z, g)
        ok, worst, fro = acceptance(gu.gemm(packed, X), Yref)
        assert ok, (g, worst, fro)
        # the 8-bit codes reproduce the fp32 product far better than the tolerance of the 4-bit path
        exact = X.astype(np.float64) @ W.astype(np.float64)
        assert np.linalg.norm(Yref.astype(np.float64) - exact) / np.linalg.norm(exact) < (2e-2 if g == K else 1e-2)
        packed.close()
    q, s, _ = _w8_case(rng, K, N, 128)
    packed = _pack_w8(tm, q, s, None, 128, symmetric=True)
    ok, worst, fro = acceptance(gu.gemm(packed, X), oracle.gemm(X, q, s, np.full((K // 128, N), 128, np.float16), 128))
    assert ok, (worst, fro)
    with pytest.raises(tm.TmError):
        tm.tm_unpack_w4(packed)
    packed.close()


# ------------------------------------------------------------------ FP8 (E4M3) weight codes

def _fp8_case(rng, K, N, g):
    q = rng.integers(0, 256, (K, N), dtype=np.uint8)
    q[(q & 0x7F) == 0x7F] = 0x30                                          # no NaN codes
    s = rng.uniform(0.0005, 0.005, (K // g, N)).astype(np.float16)
    return q, s


def test_fp8_every_code_converts_exactly(tm, oracle):
    """One-hot rows against a weight matrix that holds all 254 finite codes: Y must be fp16(fp8(q) * s), bit for bit,
    for the bias-free MFMA route (16- and 32-row kernels) and the ALU route (64-row kernel)."""
    _say("fp8 all codes")
    K, N, g = 256, 16, 128
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], np.uint8)
    q = np.zeros((K, N), np.uint8)
    q[:len(codes), :] = codes[:, None]
    s = np.array([[1.0, 0.5, 0.25, 3.0, 0.0078125, 1.5, 0.001, 0.37] * 2] * (K // g), np.float16)
    packed = tm.tm_pack_w8_fp8(gu.to_dev(wl.pack_interchange8(q)), gu.to_dev(s), K, N, g)
    wbuf, szbuf = tm.tm_packed_raw(packed)
    q2, s2, z2 = oracle.unpack_packed(wbuf, szbuf, K, N, g, bits=8)
    assert np.array_equal(q2, q) and np.array_equal(s2.view(np.uint16), s.view(np.uint16)) and not z2.view(np.uint16).any()
    What = oracle.dequant_fp8(q, s, g)
    for variant in (0, 1, 2, 4, 19, 13, 7):
        tm.tm_set_variant(variant, 0)
        try:
            for k0 in range(0, K, 16):
                X = np.zeros((16, K), np.float16)
                X[np.arange(16), k0 + np.arange(16)] = 1.0
                Y = gu.gemm(packed, X)
                # numeric equality: a sum that starts at +0 returns +0 for the code -0, on both sides
                assert np.array_equal(Y, What[k0:k0 + 16].astype(np.float16)), (variant, k0)
        finally:
            tm.tm_set_variant(-1, 0)
    packed.close()


@pytest.mark.parametrize("g", [32, 64, 128])
@pytest.mark.parametrize("M,K,N,variant,split", [
    (1, 1024, 528, -1, 0), (8, 768, 4112, -1, 0), (16, 2048, 1040, -1, 0), (11, 1280, 336, 1, 2), (16, 1024, 1552, 14, 0),
    (6, 896, 1552, 15, 0), (16, 640, 2064, 16, 0), (29, 1024, 1040, -1, 0), (64, 768, 1040, 19, 3), (150, 512, 272, -1, 0),
    (200, 1024, 1040, 7, 0), (70, 768, 528, 9, 2), (130, 512, 272, 13, 3), (300, 1024, 528, -1, 0)])
def test_fp8_gemm_against_oracle(tm, oracle, M, K, N, variant, split, g):
    _say(f"fp8 gemm M={M} K={K} N={N} g={g} variant={variant} split={split}")
    rng = np.random.default_rng(M + K + N + g + 1)
    q, s = _fp8_case(rng, K, N, g)
    # codes are uniform over the exponent range, so a few huge weights dominate: scale X down to keep fp16 outputs finite
    X = (rng.standard_normal((M, K)) * 0.25).astype(np.float16)
    packed = tm.tm_pack_w8_fp8(gu.to_dev(wl.pack_interchange8(q)), gu.to_dev(s), K, N, g)
    tm.tm_set_variant(variant, split)
    try:
        for waves in (0, 8, 16):     # decode kernels: waves per CTA; CTA tiles: two and four wave sets
            tm.tm_set_launch(waves, 0)
            ok, worst, fro = acceptance(gu.gemm(packed, X), oracle.gemm_fp8(X, q, s, g))
            assert ok, (waves, worst, fro)
    finally:
        tm.tm_set_variant(-1, 0)
        tm.tm_set_launch(0, 0)
    packed.close()


def test_fp8_quantised_weights_end_to_end(tm, oracle):
    _say("fp8 recipe end to end")
    rng = np.random.default_rng(99)
    K, N, M = 1024, 528, 12
    W = (0.02 * rng.standard_normal((K, N))).astype(np.float32)
    X = rng.standard_normal((M, K)).astype(np.float16)
    for g in (128, K):
        q, s = wl.quantise_fp8_recipe(W, g)
        packed = tm.tm_pack_w8_fp8(gu.to_dev(wl.pack_interchange8(q)), gu.to_dev(s), K, N, g)
        Yref = oracle.gemm_fp8(X, q, s, g)
        ok, worst, fro = acceptance(gu.gemm(packed, X), Yref)
        assert ok, (g, worst, fro)
        exact = X.astype(np.float64) @ W.astype(np.float64)
        assert np.linalg.norm(Yref.astype(np.float64) - exact) / np.linalg.norm(exact) < 5e-2     # 3 mantissa bits
        packed.close()


# ------------------------------------------------------------------ activation-order checkpoints

@pytest.mark.parametrize("layout", [0, 1, 2])
@pytest.mark.parametrize("M,K,N,g", [(1, 512, 272, 128), (16, 1024, 528, 64), (40, 768, 1040, 32), (300, 1024, 272, 128),
                                     (5, 512, 48, 256)])
def test_act_order_checkpoints(tm, oracle, M, K, N, g, layout):
    """Rows carry their group in g_idx: the pack sorts rows by group, the GEMM regroups X; Y must match the oracle that
    reads the checkpoint as it is."""
    import torch
    _say(f"act-order M={M} K={K} N={N} g={g} layout={layout}")
    rng = np.random.default_rng(M + K + N + g + layout)
    q = rng.integers(0, 16, (K, N), dtype=np.uint8)
    s = rng.uniform(0.001, 0.02, (K // g, N)).astype(np.float16)
    z = rng.integers(0, 16, (K // g, N)).astype(np.float16)
    gi = wl.draw_act_order(K, g, rng)
    X = rng.standard_normal((M, K)).astype(np.float16)
    qw, zs = wl.encode_layout(q, z, layout)
    zt = gu.to_dev(zs) if layout == 0 else torch.from_numpy(zs.view(np.int32)).cuda()
    packed = tm.tm_pack_w4_actorder(torch.from_numpy(qw.view(np.int32)).cuda(), gu.to_dev(s), zt,
                                    torch.from_numpy(gi).cuda(), K, N, g, layout)
    # the packed buffer holds the rows sorted by group (stable)
    perm = np.argsort(gi, kind="stable")
    wbuf, szbuf = tm.tm_packed_raw(packed)
    gs = min(g, 128)
    q2, s2, z2 = oracle.unpack_packed(wbuf, szbuf, K, N, gs)
    assert np.array_equal(q2, q[perm])
    assert np.array_equal(s2.view(np.uint16), np.repeat(s, g // gs, axis=0).view(np.uint16))
    Yref = oracle.gemm_gidx(X, q, s, z, gi)
    ok, worst, fro = acceptance(gu.gemm(packed, X), Yref)
    assert ok, (worst, fro)
    # caller-workspace entry point: regroup area inside the workspace
    nbytes = tm.tm_gemm_workspace_bytes(packed, M)
    assert nbytes >= M * K * 2
    ws = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    Y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
    tm.tm_gemm_w4a16_ws(gu.to_dev(X), packed, Y, ws)
    torch.cuda.synchronize()
    ok, worst, fro = acceptance(Y.cpu().numpy(), Yref)
    assert ok, (worst, fro)
    packed.close()


def test_act_order_rejects_bad_group_index(tm):
    import torch
    _say("act-order bad g_idx")
    K, N, g = 256, 16, 128
    qw = torch.zeros((K // 8, N), dtype=torch.int32, device="cuda")
    s = torch.ones((K // g, N), dtype=torch.float16, device="cuda")
    zq = torch.zeros((K // g, N // 8), dtype=torch.int32, device="cuda")
    for bad in (np.zeros(K, np.int32), np.full(K, 2, np.int32), np.concatenate([np.zeros(129), np.ones(127)]).astype(np.int32)):
        with pytest.raises(tm.TmError):
            tm.tm_pack_w4_actorder(qw, s, zq, torch.from_numpy(bad).cuda(), K, N, g, 2)
