"""GPU parity of the attention path (tm_attn.h) against the oracle: the quantise-and-store kernel bit for bit, the decode
attention within  |O - Oref| <= 2e-3 + 5e-3*|Oref|  and relative Frobenius error <= 2e-3  (the probabilities enter the
second matrix product as fp16, and O is rounded to fp16 once)."""
import sys

import numpy as np
import pytest

from oracle import oracle_attn as oa
from workloads import attn as wa

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tm():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import paper_2508_15601_amd as tm
    tm.load_library()
    return tm


def _say(msg):
    print(msg, file=sys.stderr, flush=True)


def _close(O, Oref):
    o, r = O.astype(np.float64), Oref.astype(np.float64)
    worst = float((np.abs(o - r) / (2e-3 + 5e-3 * np.abs(r))).max())
    fro = float(np.linalg.norm(o - r) / max(np.linalg.norm(r), 1e-30))
    return worst <= 1.0 and fro <= 2e-3, worst, fro


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("B,Hkv,T,chunks", [(1, 1, 32, [32]), (2, 3, 70, [40, 1, 1, 28]), (3, 2, 97, [97]), (2, 1, 33, [1] * 33),
                                             (2, 2, 300, [5, 200, 15, 80])])
@pytest.mark.parametrize("bits", [8, 4])
def test_kv_append_bit_exact(tm, B, Hkv, T, chunks, bits):
    """Keys and values appended in chunks land in the cache layout with exactly the oracle's codes and pairs."""
    import torch
    _say(f"kv append B={B} Hkv={Hkv} T={T} chunks={chunks[:4]} bits={bits}")
    cbytes = 128 * bits // 8
    _, K, V, _ = wa.draw(B, Hkv, Hkv, T, seed=T)
    K[0, 0, 0, :] = 1.5                                   # a constant row: scale falls back to 1
    V[-1, -1, -1, :64] = 0.0
    cache = tm.tm_kv_create(B, Hkv, T, bits)
    cap = cache.capacity
    tm.tm_kv_upload(cache, np.zeros(B * Hkv * cap * cbytes, np.uint8), np.zeros(B * Hkv * cap * cbytes, np.uint8),
                    np.zeros(B * Hkv * cap * 2, np.uint32))
    pos = 0
    for n in chunks:
        Kn = np.ascontiguousarray(K[:, :, pos:pos + n].transpose(0, 2, 1, 3))      # [B, n, Hkv, 128]
        Vn = np.ascontiguousarray(V[:, :, pos:pos + n].transpose(0, 2, 1, 3))
        tm.tm_kv_append(cache, _dev(Kn), _dev(Vn), torch.full((B,), pos, dtype=torch.int32, device="cuda"))
        pos += n
    kbuf, vbuf, szbuf = tm.tm_kv_download(cache)
    Kq, Ks, Kz, Vq, Vs, Vz = oa.kv_cache_unpack(kbuf, vbuf, szbuf, B, Hkv, cap, bits)
    for got, want in zip((Kq, Ks, Kz), oa.kv_quantise(K, bits)):
        g, w = got[:, :, :T], want
        assert np.array_equal(g.view(np.uint16) if g.dtype == np.float16 else g, w.view(np.uint16) if w.dtype == np.float16 else w)
    for got, want in zip((Vq, Vs, Vz), oa.kv_quantise(V, bits)):
        g, w = got[:, :, :T], want
        assert np.array_equal(g.view(np.uint16) if g.dtype == np.float16 else g, w.view(np.uint16) if w.dtype == np.float16 else w)
    assert not Kq[:, :, T:].any() and not Vq[:, :, T:].any()                       # nothing written past the tokens
    # tokens that would fall outside the cache are dropped
    tm.tm_kv_append(cache, _dev(Kn), _dev(Vn), torch.full((B,), cap, dtype=torch.int32, device="cuda"))
    k2, v2, s2 = tm.tm_kv_download(cache)
    assert np.array_equal(k2, kbuf) and np.array_equal(v2, vbuf) and np.array_equal(s2, szbuf)
    cache.close()


@pytest.mark.parametrize("bits", [8, 4])
def test_kv_append_ragged_positions(tm, bits):
    """Sequences at different positions, runs that start and end inside a 32-token block (the block-wise kernel merges with
    what the cache holds), a run cut off by the capacity, and a run that starts before position 0."""
    import torch
    B, Hkv, cap = 3, 2, 192
    _say(f"kv append ragged positions bits={bits}")
    cbytes = 128 * bits // 8
    _, K, V, _ = wa.draw(B, Hkv, Hkv, cap, seed=11)
    cache = tm.tm_kv_create(B, Hkv, cap, bits)
    assert cache.capacity == cap
    tm.tm_kv_upload(cache, np.zeros(B * Hkv * cap * cbytes, np.uint8), np.zeros(B * Hkv * cap * cbytes, np.uint8),
                    np.zeros(B * Hkv * cap * 2, np.uint32))
    filled = np.zeros((B, cap), bool)
    # (count, positions per sequence): first lays single tokens and short runs, then long runs over and between them
    for n, pos in [(3, [0, 30, 189]), (20, [5, 40, 100]), (70, [25, 64, 150]), (33, [-7, 129, 10]), (17, [95, 0, 175])]:
        Kn = np.zeros((B, n, Hkv, 128), np.float16)
        Vn = np.zeros((B, n, Hkv, 128), np.float16)
        for b in range(B):
            for j in range(n):
                t = pos[b] + j
                if 0 <= t < cap:
                    Kn[b, j], Vn[b, j] = K[b, :, t], V[b, :, t]
                    filled[b, t] = True
                else:
                    Kn[b, j], Vn[b, j] = 7.0, -3.0              # must never reach the cache
        tm.tm_kv_append(cache, _dev(Kn), _dev(Vn), torch.tensor(pos, dtype=torch.int32, device="cuda"))
    kbuf, vbuf, szbuf = tm.tm_kv_download(cache)
    got = oa.kv_cache_unpack(kbuf, vbuf, szbuf, B, Hkv, cap, bits)
    want = oa.kv_quantise(K, bits) + oa.kv_quantise(V, bits)
    m = filled[:, None, :]
    assert filled.any() and not filled.all()
    for g, w in zip(got, want):
        g = g.view(np.uint16) if g.dtype == np.float16 else g
        w = w.view(np.uint16) if w.dtype == np.float16 else w
        mm = np.broadcast_to(m[..., None] if g.ndim == 4 else m, g.shape)
        assert np.array_equal(g[mm], w[mm])
        assert not g[~mm].any()                                  # untouched tokens still hold the zeros uploaded
    cache.close()


ATTN_CASES = [
    # B, Hq, Hkv, T, lens (None: drawn)
    (1, 1, 1, 1, [1]),
    (2, 4, 4, 31, None),
    (2, 8, 2, 32, [32, 17]),
    (3, 8, 1, 33, None),
    (2, 16, 1, 100, None),
    (1, 32, 8, 257, None),
    (4, 12, 3, 1000, None),                # several blocks per wave
    (1, 8, 2, 5000, [5000]),               # split context, merged by the second kernel
    (2, 8, 8, 4100, [4100, 1300]),         # splits of which some are empty for the short sequence
    (1, 64, 8, 640, None),
    (2, 4, 2, 64, [33, 64]),               # a 4-bit block whose second half holds one token / is full
    (1, 8, 2, 8200, [8161]),               # split context ending in the first half of a 64-token block
    # more than sixteen query heads per KV head: one pass per sixteen heads (a last pass of 16, of 4, of 8 heads)
    (2, 32, 1, 300, None),
    (1, 40, 2, 5000, [5000]),              # 20 per KV head, split context merged by the second kernel
    (2, 48, 2, 700, [700, 90]),            # 24 per KV head, split context merged in the kernel
]


@pytest.mark.parametrize("B,Hq,Hkv,T,lens", ATTN_CASES)
@pytest.mark.parametrize("bits", [8, 4])
def test_attn_decode_against_oracle(tm, B, Hq, Hkv, T, lens, bits):
    import torch
    _say(f"attn decode B={B} Hq={Hq} Hkv={Hkv} T={T} lens={lens} bits={bits}")
    Q, K, V, drawn = wa.draw(B, Hq, Hkv, T, seed=B * 100 + Hq + T)
    lens = np.array(lens, np.int32) if lens is not None else drawn
    Kq, Ks, Kz = oa.kv_quantise(K, bits)
    Vq, Vs, Vz = oa.kv_quantise(V, bits)
    cache = tm.tm_kv_create(B, Hkv, T, bits)
    cap = cache.capacity
    # the cache is filled by the library's own kernel; positions past T keep whatever the allocation held
    tm.tm_kv_append(cache, _dev(np.ascontiguousarray(K.transpose(0, 2, 1, 3))), _dev(np.ascontiguousarray(V.transpose(0, 2, 1, 3))),
                    torch.zeros(B, dtype=torch.int32, device="cuda"))
    scale = 1.0 / np.sqrt(128.0)
    outs = []
    for _ in range(2):
        O = torch.full((B, Hq, 128), float("nan"), dtype=torch.float16, device="cuda")
        tm.tm_attn_decode(_dev(Q), cache, _dev(lens), O, scale, max_len=int(lens.max()))
        torch.cuda.synchronize()
        outs.append(O.cpu().numpy())
    assert np.array_equal(outs[0].view(np.uint16), outs[1].view(np.uint16))        # run-to-run identical
    Oref = oa.attn_decode(Q, Kq, Ks, Kz, Vq, Vs, Vz, lens, scale)
    ok, worst, fro = _close(outs[0], Oref)
    assert ok, (worst, fro)
    cache.close()


@pytest.mark.parametrize("bits", [8, 4])
def test_attn_decode_special_cases(tm, bits):
    """Sharp softmax (one token takes all the weight), a sequence without tokens, cache bytes past the context that hold
    NaN pairs, and max_len left at 0."""
    import torch
    _say(f"attn special cases bits={bits}")
    B, Hq, Hkv, T = 2, 8, 2, 128
    Q, K, V, _ = wa.draw(B, Hq, Hkv, T, seed=5)
    Kq, Ks, Kz = oa.kv_quantise(K, bits)
    Vq, Vs, Vz = oa.kv_quantise(V, bits)
    Kd = oa.kv_dequant(Kq, Ks, Kz)
    Q[0, :4] = (Kd[0, 0, 70] * 1.0).astype(np.float16)     # heads 0..3 (KV head 0) point at token 70
    lens = np.array([80, 0], np.int32)
    cache = tm.tm_kv_create(B, Hkv, T, bits)
    cap = cache.capacity
    assert cap == T
    kbuf, vbuf, szbuf = wa.encode_cache(*[np.ascontiguousarray(a) for a in (Kq, Ks, Kz, Vq, Vs, Vz)], bits=bits)
    sz = szbuf.reshape(B, Hkv, cap, 2).copy()
    sz[:, :, 80:] = 0x7E007E00                              # NaN scale and zero-point past the context
    tm.tm_kv_upload(cache, kbuf, vbuf, sz.reshape(-1))
    O = torch.full((B, Hq, 128), float("nan"), dtype=torch.float16, device="cuda")
    tm.tm_attn_decode(_dev(Q), cache, _dev(lens), O, 4.0)   # max_len = 0: the capacity
    torch.cuda.synchronize()
    O = O.cpu().numpy()
    assert not O[1].any()                                   # no tokens: zeros
    Oref = oa.attn_decode(Q[:1], Kq[:1], Ks[:1], Kz[:1], Vq[:1], Vs[:1], Vz[:1], lens[:1], 4.0)
    ok, worst, fro = _close(O[:1], Oref)
    assert ok, (worst, fro)
    assert np.allclose(O[0, 0].astype(np.float64), oa.kv_dequant(Vq, Vs, Vz)[0, 0, 70], rtol=1e-2, atol=2e-3)
    # a max_len below the sequence's length cuts the context at a block boundary instead of dropping blocks in the middle
    tm.tm_kv_upload(cache, kbuf, vbuf, szbuf)
    lens2 = np.array([128, 100], np.int32)
    O2 = torch.full((B, Hq, 128), float("nan"), dtype=torch.float16, device="cuda")
    tm.tm_attn_decode(_dev(Q), cache, _dev(lens2), O2, 0.1, max_len=64)
    torch.cuda.synchronize()
    Oref2 = oa.attn_decode(Q, Kq, Ks, Kz, Vq, Vs, Vz, np.array([64, 64], np.int32), 0.1)
    ok, worst, fro = _close(O2.cpu().numpy(), Oref2)
    assert ok, (worst, fro)
    cache.close()


@pytest.mark.parametrize("bits", [8, 4])
def test_attn_decode_full_size_sampled(tm, bits):
    """The benchmark's largest shape in its own launch configuration (batch 128 x context 2048, 32 query / 8 KV heads, the
    prompt stored by one block-wise append, one decode launch without splits); the oracle recomputes a sample of the
    sequences from the same keys and values."""
    import torch
    B, Hq, Hkv, T = 128, 32, 8, 2048
    _say(f"attn full size B={B} T={T} bits={bits}")
    g = torch.Generator(device="cuda").manual_seed(1234 + bits)
    K = torch.randn((B, T, Hkv, 128), generator=g, device="cuda").to(torch.float16)
    V = torch.randn((B, T, Hkv, 128), generator=g, device="cuda").to(torch.float16)
    Q = torch.randn((B, Hq, 128), generator=g, device="cuda").to(torch.float16)
    lens = torch.randint(1, T + 1, (B,), generator=g, device="cuda").to(torch.int32)
    lens[0] = T
    lens[5] = 1
    cache = tm.tm_kv_create(B, Hkv, T, bits)
    tm.tm_kv_append(cache, K, V, torch.zeros(B, dtype=torch.int32, device="cuda"))
    O = torch.full((B, Hq, 128), float("nan"), dtype=torch.float16, device="cuda")
    scale = 1.0 / np.sqrt(128.0)
    tm.tm_attn_decode(Q, cache, lens, O, scale, max_len=T)
    torch.cuda.synchronize()
    assert not torch.isnan(O).any()
    sample = [0, 5, 17, 64, 127]
    Ks = K[sample].permute(0, 2, 1, 3).contiguous().cpu().numpy()           # [n, Hkv, T, 128]
    Vs = V[sample].permute(0, 2, 1, 3).contiguous().cpu().numpy()
    Oref = oa.attn_decode(Q[sample].cpu().numpy(), *oa.kv_quantise(Ks, bits), *oa.kv_quantise(Vs, bits),
                          lens[sample].cpu().numpy(), scale)
    ok, worst, fro = _close(O[sample].cpu().numpy(), Oref)
    assert ok, (worst, fro)
    cache.close()


def _random_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        Hkv = int(rng.choice([1, 2, 3, 8]))
        G = int(rng.choice([1, 2, 4, 5, 8, 9, 16]))
        B = int(rng.choice([1, 2, 5, 9]))
        T = int(rng.choice([1, 40, 64, 65, 130, 700, 2100, 6000]))
        cases.append((i, B, Hkv * G, Hkv, T, int(rng.choice([4, 8]))))
    return cases


@pytest.mark.parametrize("i,B,Hq,Hkv,T,bits", _random_cases(24, 2024))
def test_attn_decode_random_shapes(tm, i, B, Hq, Hkv, T, bits):
    """Seeded random shapes: group sizes on both sides of the shared-pass limit (8), odd batch and head counts, contexts
    from one token to several splits, ragged lengths (some sequences empty), both code widths."""
    import torch
    _say(f"attn random {i}: B={B} Hq={Hq} Hkv={Hkv} T={T} bits={bits}")
    Q, K, V, lens = wa.draw(B, Hq, Hkv, T, seed=1000 + i, min_len=0)
    if B > 2:
        lens[1] = 0
    cache = tm.tm_kv_create(B, Hkv, T, bits)
    tm.tm_kv_append(cache, _dev(np.ascontiguousarray(K.transpose(0, 2, 1, 3))), _dev(np.ascontiguousarray(V.transpose(0, 2, 1, 3))),
                    torch.zeros(B, dtype=torch.int32, device="cuda"))
    O = torch.full((B, Hq, 128), float("nan"), dtype=torch.float16, device="cuda")
    scale = 1.0 / np.sqrt(128.0)
    tm.tm_attn_decode(_dev(Q), cache, _dev(lens), O, scale, max_len=int(max(lens.max(), 1)))
    torch.cuda.synchronize()
    O = O.cpu().numpy()
    some = lens > 0                                          # the oracle defines attention over at least one token
    assert not O[~some].any()                                # an empty sequence gets zeros
    kq, vq = oa.kv_quantise(K[some], bits), oa.kv_quantise(V[some], bits)
    Oref = oa.attn_decode(Q[some], *kq, *vq, lens[some], scale)
    ok, worst, fro = _close(O[some], Oref)
    assert ok, (worst, fro)
    cache.close()


@pytest.mark.parametrize("bits,T", [(8, 3000), (4, 3000), (8, 40000)])
def test_attn_hip_graph_replay_matches_eager(tm, bits, T):
    """A decoding step - append of the newest token, then attention over split contexts (merged in the kernel through
    the arrival counters at 3000 tokens, by the merge kernel at 40000) - allocates nothing and leaves its counters at
    zero, so it can be captured into a HIP graph; every replay, with eager work between, reproduces the eager bits."""
    import torch
    B, Hq, Hkv = 2, 8, 2
    _say(f"attn graph replay bits={bits} T={T}")
    g = torch.Generator(device="cuda").manual_seed(7)
    K = torch.randn((B, T, Hkv, 128), generator=g, device="cuda").to(torch.float16)
    V = torch.randn((B, T, Hkv, 128), generator=g, device="cuda").to(torch.float16)
    Q = torch.randn((B, Hq, 128), generator=g, device="cuda").to(torch.float16)
    cache = tm.tm_kv_create(B, Hkv, T, bits)
    zero = torch.zeros(B, dtype=torch.int32, device="cuda")
    tm.tm_kv_append(cache, K[:, :T - 1].contiguous(), V[:, :T - 1].contiguous(), zero)
    last_k, last_v = K[:, T - 1:].contiguous(), V[:, T - 1:].contiguous()
    pos = torch.full((B,), T - 1, dtype=torch.int32, device="cuda")
    lens = torch.tensor([T, T - 700], dtype=torch.int32, device="cuda")

    def step(out):
        tm.tm_kv_append(cache, last_k, last_v, pos)
        tm.tm_attn_decode(Q, cache, lens, out, 0.09, max_len=T)

    O_eager = torch.empty((B, Hq, 128), dtype=torch.float16, device="cuda")
    step(O_eager)
    torch.cuda.synchronize()
    O_graph = torch.empty_like(O_eager)
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            step(O_graph)
            step(O_graph)
    for rep in range(3):
        O_graph.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(O_graph.view(torch.int16), O_eager.view(torch.int16)), f"replay {rep}"
        O2 = torch.empty_like(O_eager)
        step(O2)                                             # eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(O2.view(torch.int16), O_eager.view(torch.int16))
    # and the eager result is the right one (sampled against the oracle on the first sequence)
    Ks = K[:1].permute(0, 2, 1, 3).contiguous().cpu().numpy()
    Vs = V[:1].permute(0, 2, 1, 3).contiguous().cpu().numpy()
    Oref = oa.attn_decode(Q[:1].cpu().numpy(), *oa.kv_quantise(Ks, bits), *oa.kv_quantise(Vs, bits), np.array([T]), 0.09)
    ok, worst, fro = _close(O_eager[:1].cpu().numpy(), Oref)
    assert ok, (worst, fro)
    cache.close()


# ------------------------------------------------------------------ a chunk of prompt tokens (prefill)

PREFILL_CASES = [
    # B, Hq, Hkv, cached tokens T, positions, counts (None: all), query rows n
    (1, 4, 1, 40, [0], None, 40),                         # whole prompt, G = 4
    (3, 8, 2, 96, [0, 0, 0], [70, 1, 33], 70),            # ragged prompt lengths in one call
    (2, 4, 4, 50, [0, 0], [50, 17], 50),                  # G = 1: sixteen tokens per CTA
    (2, 16, 1, 45, [0, 0], None, 45),                     # G = 16: one token per CTA
    (2, 6, 2, 37, [0, 0], [37, 20], 37),                  # G = 3: five tokens per CTA, one column idle
    (2, 8, 1, 64, [0, 0], None, 64),                      # G = 8
    (3, 8, 2, 130, [40, 0, 100], [20, 5, 17], 20),        # later chunks of longer prompts (chunked prefill)
    (2, 8, 2, 300, [0, 150], [300, 150], 300),            # several blocks per wave, ragged tail
    (2, 40, 2, 90, [0, 30], [60, 33], 60),                # G = 20: a pass of sixteen heads and one of four
]


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("B,Hq,Hkv,T,positions,counts,n", PREFILL_CASES)
def test_attn_prefill_against_oracle(tm, B, Hq, Hkv, T, positions, counts, n, bits):
    import torch
    _say(f"attn prefill B={B} Hq={Hq} Hkv={Hkv} T={T} positions={positions} counts={counts} n={n} bits={bits}")
    rng = np.random.default_rng(B * 1000 + Hq * 10 + T + bits)
    _, K, V, _ = wa.draw(B, Hq, Hkv, T, seed=T + Hq)
    Q = rng.standard_normal((B, n, Hq, 128)).astype(np.float16)
    kq, vq = oa.kv_quantise(K, bits), oa.kv_quantise(V, bits)
    cache = tm.tm_kv_create(B, Hkv, T, bits)
    tm.tm_kv_append(cache, _dev(np.ascontiguousarray(K.transpose(0, 2, 1, 3))), _dev(np.ascontiguousarray(V.transpose(0, 2, 1, 3))),
                    torch.zeros(B, dtype=torch.int32, device="cuda"))
    pos = np.array(positions, np.int32)
    cnt = np.full(B, n, np.int32) if counts is None else np.array(counts, np.int32)
    scale = 1.0 / np.sqrt(128.0)
    outs = []
    for _ in range(2):
        O = torch.full((B, n, Hq, 128), float("nan"), dtype=torch.float16, device="cuda")
        tm.tm_attn_prefill(_dev(Q), cache, _dev(pos), O, scale, counts=None if counts is None else _dev(cnt))
        torch.cuda.synchronize()
        outs.append(O.cpu().numpy())
    assert np.array_equal(outs[0].view(np.uint16), outs[1].view(np.uint16))        # run-to-run identical
    Oref = oa.attn_prefill(Q, *kq, *vq, pos, cnt, scale)
    for b in range(B):
        assert np.isnan(outs[0][b, cnt[b]:]).all()                                 # rows past the count are left alone
        ok, worst, fro = _close(outs[0][b, :cnt[b]], Oref[b, :cnt[b]])
        assert ok, (b, worst, fro)
    cache.close()


@pytest.mark.parametrize("bits", [8, 4])
def test_attn_prefill_long_prompt_sampled(tm, bits):
    """A 2048-token prompt in the benchmark's head geometry (32 query / 8 KV heads), as bench.py launches it; the oracle
    checks sampled query rows, the first and last of them included."""
    import torch
    _say(f"attn prefill long prompt bits={bits}")
    B, Hq, Hkv, T = 1, 32, 8, 2048
    rng = np.random.default_rng(bits)
    _, K, V, _ = wa.draw(B, Hq, Hkv, T, seed=3)
    Q = rng.standard_normal((B, T, Hq, 128)).astype(np.float16)
    kq, vq = oa.kv_quantise(K, bits), oa.kv_quantise(V, bits)
    cache = tm.tm_kv_create(B, Hkv, T, bits)
    tm.tm_kv_append(cache, _dev(np.ascontiguousarray(K.transpose(0, 2, 1, 3))), _dev(np.ascontiguousarray(V.transpose(0, 2, 1, 3))),
                    torch.zeros(B, dtype=torch.int32, device="cuda"))
    O = torch.full((B, T, Hq, 128), float("nan"), dtype=torch.float16, device="cuda")
    tm.tm_attn_prefill(_dev(Q), cache, torch.zeros(B, dtype=torch.int32, device="cuda"), O, 128 ** -0.5)
    torch.cuda.synchronize()
    O = O.cpu().numpy()
    assert not np.isnan(O).any()
    rows = np.unique(np.concatenate([[0, 1, 31, 32, 33, 63, 64, T - 1], rng.integers(0, T, 24)]))
    for i in rows:                                          # row i as a one-token chunk at position i
        ref = oa.attn_prefill(Q[:, i:i + 1], *kq, *vq, np.array([i], np.int32), np.array([1], np.int32), 128 ** -0.5)
        ok, worst, fro = _close(O[:, i:i + 1], ref)
        assert ok, (int(i), worst, fro)
    cache.close()


def test_attn_prefill_argument_checks(tm):
    import torch
    cache = tm.tm_kv_create(1, 2, 64, 8)
    Q = torch.zeros((1, 4, 8, 128), dtype=torch.float16, device="cuda")
    pos = torch.zeros(1, dtype=torch.int32, device="cuda")
    with pytest.raises(tm.TmError):
        tm.tm_attn_prefill(Q, cache, pos, torch.empty_like(Q), 0.0)               # scale
    with pytest.raises(tm.TmError):
        tm.tm_attn_prefill(torch.zeros((1, 4, 7, 128), dtype=torch.float16, device="cuda"), cache, pos,
                           torch.zeros((1, 4, 7, 128), dtype=torch.float16, device="cuda"), 0.1)   # heads not a multiple
    # positions outside the cache: nothing is written, nothing faults
    O = torch.full((1, 4, 8, 128), float("nan"), dtype=torch.float16, device="cuda")
    tm.tm_attn_prefill(Q, cache, torch.full((1,), 64, dtype=torch.int32, device="cuda"), O, 0.1)
    tm.tm_attn_prefill(Q, cache, torch.full((1,), -9, dtype=torch.int32, device="cuda"), O, 0.1)
    torch.cuda.synchronize()
    assert torch.isnan(O).all()
    cache.close()
