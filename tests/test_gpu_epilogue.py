"""GPU parity of the fused epilogue (bias, silu(gate)*up, residual) against the oracle, through the C ABI.

Every mode, the activation included, is held to the acceptance rule of the plain product: |Y - Yref| <= 1e-2 + 5e-3*|Yref|
and relative Frobenius error <= 2e-3."""
import sys

import numpy as np
import pytest

from workloads import w4a16 as wl
from helpers import acceptance
import gpu_util as gu

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, file=sys.stderr, flush=True)


@pytest.fixture(scope="module")
def tm():
    import torch
    import paper_2508_15601_amd as tm
    assert torch.cuda.is_available(), "GPU tests need a device"
    tm.load_library()
    yield tm
    tm.tm_set_variant(-1, 0)
    tm.tm_set_launch(0, 0)


def _run(tm, oracle, d, g, M, mode, variant=-1, split=0, waves=0, stage=0):
    import torch
    K, N = d["q"].shape
    rng = np.random.default_rng(N + M)
    act = "silu_mul" in mode
    n_out = N // 2 if act else N
    bias = rng.standard_normal(N).astype(np.float16) if "bias" in mode else None
    res = rng.standard_normal((M, n_out)).astype(np.float16) if "residual" in mode else None
    if act:
        packed = tm.tm_pack_w4_gate_up(gu.to_dev(d["qweight"]), gu.to_dev(d["s"]), gu.to_dev(d["z"]), K, N, g)
    else:
        packed = gu.pack(d, g)
    tm.tm_set_launch(waves, stage)
    tm.tm_set_variant(variant, split)
    plan = tm.tm_get_plan(packed, M)
    _say(f"epilogue {mode} M={M} K={K} N={N} g={g} plan={plan}")
    if variant >= 0:
        assert plan["variant"] == variant
    X = d["X"][:M]
    outs = []
    for _ in range(2):
        Y = torch.full((M, n_out), float("nan"), dtype=torch.float16, device="cuda")
        tm.tm_gemm_w4a16_ex(gu.to_dev(X), packed, Y, bias=None if bias is None else gu.to_dev(bias),
                            residual=None if res is None else gu.to_dev(res),
                            act=tm.TM_ACT_SILU_MUL if act else tm.TM_ACT_NONE)
        torch.cuda.synchronize()
        outs.append(Y.cpu().numpy())
    tm.tm_set_variant(-1, 0)
    tm.tm_set_launch(0, 0)
    assert np.array_equal(outs[0].view(np.uint16), outs[1].view(np.uint16))
    _, Yd = oracle.gemm(X, d["q"], d["s"], d["z"], g, want_fp64=True)
    Yref = oracle.epilogue(Yd, bias, res, "silu_mul" if act else "none")
    # one rule for every mode: |Y - Yref| <= 1e-2 + 5e-3 |Yref| and relative Frobenius error <= 2e-3 (with the activation the
    # observed worst ratio to that bound is 0.16 and the Frobenius error 2.2e-4 over all cases of this file)
    ok, worst, fro = acceptance(outs[0], Yref)
    assert ok, (mode, worst, fro)
    packed.close()


MODES = ["bias", "residual", "bias+residual", "silu_mul", "silu_mul+bias+residual"]
# (variant, split, waves, M): decode strips with and without split-K, CTA tiles with and without split-K and wave sets,
# the 128-row tile; -1 = the library's own choice
LAUNCHES = [(-1, 0, 0, 1), (-1, 0, 0, 16), (-1, 0, 0, 40), (-1, 0, 0, 300), (0, 1, 8, 13), (0, 3, 16, 13), (3, 1, 8, 29),
            (4, 2, 8, 32), (5, 3, 0, 30), (8, 1, 0, 300), (9, 2, 0, 70), (11, 1, 0, 200), (13, 1, 8, 33), (20, 1, 4, 30)]


@pytest.mark.parametrize("variant,split,waves,M", LAUNCHES)
@pytest.mark.parametrize("mode", MODES)
def test_epilogue_against_oracle(tm, oracle, variant, split, waves, M, mode):
    K, N, g = 1152, 352, 128
    d = wl.make(wl.Case(f"epi_{M}", max(M, 1), K, N, g, seed=(variant + 2) * 7 + split + M))
    _run(tm, oracle, d, g, M, mode, variant, split, waves)


@pytest.mark.parametrize("M", [4, 96])
def test_epilogue_small_groups_and_real_shape(tm, oracle, M):
    """Group 32 on a ragged shape, and the gated MLP's fused projection at a real width (sampled rows keep the oracle
    within seconds)."""
    d = wl.make(wl.Case("epi_g32", M, 640, 416, 32, seed=5))
    _run(tm, oracle, d, 32, M, "silu_mul+bias+residual")
    d = wl.make(wl.Case("epi_mlp", min(M, 8), 4096, 2 * 11008, 128, seed=6))
    _run(tm, oracle, d, 128, min(M, 8), "silu_mul+residual")


def test_epilogue_argument_checks(tm, oracle):
    import torch
    d = wl.make(wl.Case("epi_args", 4, 256, 64, 128, seed=1))
    plain = gu.pack(d, 128)
    fused = tm.tm_pack_w4_gate_up(gu.to_dev(d["qweight"]), gu.to_dev(d["s"]), gu.to_dev(d["z"]), 256, 64, 128)
    X = gu.to_dev(d["X"])
    Yh = torch.empty((4, 32), dtype=torch.float16, device="cuda")
    Yf = torch.empty((4, 64), dtype=torch.float16, device="cuda")
    with pytest.raises(tm.TmError):                       # a plain handle has no interleaved columns
        tm.tm_gemm_w4a16_ex(X, plain, Yh, act=tm.TM_ACT_SILU_MUL)
    with pytest.raises(tm.TmError):                       # an interleaved handle only serves the activation
        tm.tm_gemm_w4a16(X, fused, Yf)
    with pytest.raises(tm.TmError):
        tm.tm_pack_w4_gate_up(gu.to_dev(d["qweight"][:, :6]), gu.to_dev(d["s"][:, :48]), None, 256, 48, 128)   # N % 32
    # no epilogue fields set: identical to the plain call
    tm.tm_gemm_w4a16_ex(X, plain, Yf)
    Y0 = torch.empty_like(Yf)
    tm.tm_gemm_w4a16(X, plain, Y0)
    torch.cuda.synchronize()
    assert torch.equal(Yf, Y0)
    plain.close()
    fused.close()


@pytest.mark.parametrize("E,K,N,g,counts,variant", [
    (4, 512, 288, 128, [0, 1, 17, 5], -1),                  # decode-sized loads
    (3, 256, 96, 32, [40, 0, 70], 0),                       # several passes per expert
    (2, 512, 1056, 64, [16, 15], 2),
    (3, 512, 544, 128, [200, 0, 70], -1),                   # CTA tiles
    (4, 384, 160, 32, [130, 1, 0, 129], 9),
])
def test_grouped_gemm_with_fused_activation(tm, oracle, E, K, N, g, counts, variant):
    """All experts of a mixture-of-experts layer in one launch, silu(gate)*up fused: per expert the oracle's product on
    that expert's rows, then the oracle's epilogue."""
    import torch
    _say(f"grouped silu_mul E={E} K={K} N={N} g={g} counts={counts} variant={variant}")
    rng = np.random.default_rng(E * 100 + N)
    host, dev = [], []
    for e in range(E):
        q = rng.integers(0, 16, (K, N), dtype=np.uint8)
        s = rng.uniform(0.001, 0.02, (K // g, N)).astype(np.float16)
        z = rng.integers(0, 16, (K // g, N)).astype(np.float16)
        host.append((q, s, z))
        dev.append(tm.tm_pack_w4_gate_up(gu.to_dev(wl.pack_interchange(q)), gu.to_dev(s), gu.to_dev(z), K, N, g))
    offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    R = int(offsets[-1]) + 2                                 # two rows no expert owns
    X = rng.standard_normal((R, K)).astype(np.float16)
    group = tm.tm_group_experts(dev)
    Y = torch.full((R, N // 2), float("nan"), dtype=torch.float16, device="cuda")
    tm.tm_set_variant(variant, 0)
    try:
        tm.tm_gemm_w4a16_grouped_act(gu.to_dev(X), group, torch.from_numpy(offsets).cuda(), Y, tm.TM_ACT_SILU_MUL)
        torch.cuda.synchronize()
        with pytest.raises(tm.TmError):                      # interleaved experts serve the activation only
            tm.tm_gemm_w4a16_grouped(gu.to_dev(X), group, torch.from_numpy(offsets).cuda(),
                                     torch.empty((R, N), dtype=torch.float16, device="cuda"))
    finally:
        tm.tm_set_variant(-1, 0)
    Y = Y.cpu().numpy()
    assert np.isnan(Y[offsets[-1]:]).all()
    for e in range(E):
        r0, r1 = offsets[e], offsets[e + 1]
        if r1 == r0:
            continue
        _, Yd = oracle.gemm(X[r0:r1], *host[e], g, want_fp64=True)
        ok, worst, fro = acceptance(Y[r0:r1], oracle.epilogue(Yd, act="silu_mul"))
        assert ok, (e, worst, fro)
    group.close()
    for p in dev:
        p.close()


@pytest.mark.parametrize("K,N,g,symmetric", [(256, 64, 128, False), (384, 416, 32, False), (1024, 2080 * 2, 64, True)])
def test_gate_up_pack_is_the_column_interleave_bit_for_bit(tm, oracle, K, N, g, symmetric):
    """The packed buffer of a gate/up handle holds kernel column 2j = gate column j and 2j + 1 = up column N/2 + j:
    undone by the oracle's inverse of the packed layout and compared with the input codes, scales and zero-points."""
    rng = np.random.default_rng(K + N)
    q = rng.integers(0, 16, (K, N), dtype=np.uint8)
    s = rng.uniform(0.001, 0.02, (K // g, N)).astype(np.float16)
    z = rng.integers(0, 16, (K // g, N)).astype(np.float16)
    fused = tm.tm_pack_w4_gate_up(gu.to_dev(wl.pack_interchange(q)), gu.to_dev(s), None if symmetric else gu.to_dev(z), K, N, g)
    wbuf, szbuf = tm.tm_packed_raw(fused)
    q2, s2, z2 = oracle.unpack_packed(wbuf, szbuf, K, N, g)
    src = np.empty(N, np.int64)
    src[0::2] = np.arange(N // 2)
    src[1::2] = N // 2 + np.arange(N // 2)
    assert np.array_equal(q2, q[:, src])
    assert np.array_equal(s2.view(np.uint16), s[:, src].view(np.uint16))
    want_z = np.full_like(z, 8.0) if symmetric else z
    assert np.array_equal(z2.view(np.uint16), want_z[:, src].view(np.uint16))
    fused.close()
