"""Repeat-determinism of the cross-CTA hand-overs at full size: the split-K merge of the GEMM kernels and the in-kernel /
second-kernel merge of split attention contexts.  Partial results cross CTAs (and L2 caches) through write-through stores,
a wave-level wait for their completion, a CTA barrier and a relaxed arrival counter; a hand-over that reads a partial
before it has landed would show up as a changed bit somewhere in a few hundred launches.  Every launch is followed by
unrelated work that sweeps more than the L2 capacity on the same stream, and the output must equal the first launch's bit
for bit.  The loop stops at the first mismatch."""
import sys

import numpy as np
import pytest

from workloads import w4a16 as wl
import gpu_util as gu

pytestmark = pytest.mark.gpu
LAUNCHES = 300


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _repeat(torch, launch, out, thrash, what):
    """launch() writes `out`; returns nothing, asserts that LAUNCHES launches reproduce the first bits."""
    launch()
    torch.cuda.synchronize()
    first = out.clone()
    bad = torch.zeros((), dtype=torch.int32, device="cuda")
    for it in range(LAUNCHES):
        out.fill_(float("nan"))
        thrash()
        launch()
        bad += (out.view(torch.int16) != first.view(torch.int16)).any().to(torch.int32)
        if it % 25 == 24:
            assert int(bad.item()) == 0, f"{what}: output changed within launches {it - 24}..{it}"
    assert int(bad.item()) == 0, what


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2508_15601_amd as tm
    tm.load_library()
    src = torch.empty(96 << 20, dtype=torch.uint8, device="cuda").random_(0, 256)      # 96 MB: every L2 several times over
    dst = torch.empty_like(src)
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    turn = [0]

    def thrash():
        turn[0] += 1
        if turn[0] & 1:
            tm.tm_bench_read(src, sink)
        else:
            tm.tm_bench_copy(dst[:32 << 20], src[:32 << 20])
    return torch, tm, thrash


# (layer, M, forced split): 0 = the split the dispatcher picks by itself; the 8192 x 8192 layer at M = 32 runs unsplit by
# default and is split here, so that its kernel's hand-over is covered as well
@pytest.mark.parametrize("layer,M,split", [("cfg3_down", 16, 0), ("cfg3_down", 32, 0), ("cfg3_down", 64, 0), ("cfg5_sweep", 32, 2),
                                           ("cfg5_sweep", 64, 2)])
def test_split_k_merge_repeats_bit_for_bit(env, layer, M, split):
    torch, tm, thrash = env
    big = wl.case_by_name({"cfg3_down": "cfg3_down_M64", "cfg5_sweep": "cfg5_sweep_M1024"}[layer])
    d = wl.make(big)
    packed = gu.pack(d, big.group)
    tm.tm_set_variant(-1, split)
    try:
        plan = tm.tm_get_plan(packed, M)
        _say(f"stress split-K {layer} M={M} plan={plan}")
        assert plan["split_k"] > 1, "the case is meant to cross CTAs"
        X = gu.to_dev(d["X"][:M])
        Y = torch.empty((M, big.N), dtype=torch.float16, device="cuda")
        _repeat(torch, lambda: tm.tm_gemm_w4a16(X, packed, Y), Y, thrash, f"{layer} M={M}")
    finally:
        tm.tm_set_variant(-1, 0)
    packed.close()


@pytest.mark.parametrize("bits,B,T", [(8, 1, 32768), (4, 1, 32768), (8, 8, 8192), (4, 4, 8192)])
def test_attention_split_merge_repeats_bit_for_bit(env, bits, B, T):
    torch, tm, thrash = env
    Hq, Hkv = 32, 8
    _say(f"stress attention merge KV{bits} batch {B} context {T}")
    cache = tm.tm_kv_create(B, Hkv, T, bits)
    k, v, pairs, cb, pb = tm.tm_kv_raw(cache)
    rng = np.random.default_rng(bits + B)
    n = B * Hkv * cache.capacity
    words = (rng.uniform(0.005, 0.05, 2 * n).astype(np.float16).view(np.uint16).astype(np.uint32)
             | (rng.integers(0, 1 << bits, 2 * n).astype(np.float16).view(np.uint16).astype(np.uint32) << 16))
    for ptr in (k, v):
        t = torch.randint(0, 256, (cb,), dtype=torch.uint8, device="cuda")
        tm.tm_bench_copy_raw(ptr, t.data_ptr(), cb)
    t = torch.from_numpy(words.view(np.uint8)).cuda()
    tm.tm_bench_copy_raw(pairs, t.data_ptr(), pb)
    torch.cuda.synchronize()
    Q = torch.randn((B, Hq, 128), device="cuda").to(torch.float16)
    O = torch.empty_like(Q)
    lens = torch.full((B,), T, dtype=torch.int32, device="cuda")
    _repeat(torch, lambda: tm.tm_attn_decode(Q, cache, lens, O, 128 ** -0.5, max_len=T), O, thrash, f"KV{bits} {B}x{T}")
    cache.close()


def test_measurement_helpers_mfma_loop_and_clock_probe(env):
    """The two measurement kernels end by themselves and report plausible counters: the MFMA-only loop issues 16-clock
    instructions back to back (16-20 clocks per MFMA and SIMD with one wave per SIMD), and the clock probe sees a shader
    clock between 0.5 and 3 GHz over the stretch it was asked to watch."""
    torch, tm, _ = env
    out = torch.zeros(16, dtype=torch.int32, device="cuda")
    iters = 2000
    tm.tm_bench_mfma(out, 256, 256, iters, 2)
    torch.cuda.synchronize()
    ticks = out.cpu().numpy().astype("uint32")
    assert 15.0 <= ticks[0] / (iters * 8) <= 24.0, ticks[:2]
    assert ticks[1] > 0
    out.zero_()
    khz = tm.tm_bench_clock(out, 500, delay_micros=200)
    torch.cuda.synchronize()
    ticks = out.cpu().numpy().astype("uint32")
    assert khz > 0
    watched_us = ticks[1] / (khz * 1e3) * 1e6
    assert 500 <= watched_us < 2500, watched_us
    ghz = ticks[0] / (watched_us * 1e3)
    assert 0.5 < ghz < 3.0, ghz
    for bad in (lambda: tm.tm_bench_clock(out, 0), lambda: tm.tm_bench_clock(out, 30000), lambda: tm.tm_bench_clock(out, 100, delay_micros=-1),
                lambda: tm.tm_bench_mfma(out, 0, 256, 10), lambda: tm.tm_bench_mfma(out, 256, 100, 10),
                lambda: tm.tm_bench_mfma(out, 256, 256, 0), lambda: tm.tm_bench_mfma(out, 256, 256, 10, 3)):
        with pytest.raises(tm.TmError):
            bad()
