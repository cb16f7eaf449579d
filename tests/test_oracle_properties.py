"""Property tests (hypothesis) of the oracle's layout functions: round trips of every interchange word order and of the
fragment-ordered layout over random shapes and contents, and the quantiser's invariants over random groups.  CPU only."""
import numpy as np
from hypothesis import given, settings, strategies as st, HealthCheck

from test_oracle_pins import _pack_fragment_order_numpy

COMMON = dict(deadline=None, max_examples=40, suppress_health_check=[HealthCheck.function_scoped_fixture, HealthCheck.too_slow])


@st.composite
def code_matrices(draw, k_quantum=8, n_quantum=8, kmax=6, nmax=6):
    K = k_quantum * draw(st.integers(1, kmax))
    N = n_quantum * draw(st.integers(1, nmax))
    seed = draw(st.integers(0, 2 ** 32 - 1))
    return np.random.default_rng(seed).integers(0, 16, (K, N), dtype=np.uint8)


@settings(**COMMON)
@given(q=code_matrices())
def test_interchange_orders_round_trip(oracle, q):
    K, N = q.shape
    assert np.array_equal(oracle.unpack_canonical(oracle.pack_canonical(q), N), q)
    assert np.array_equal(oracle.unpack_n8i(oracle.pack_n8i(q), N), q)
    assert np.array_equal(oracle.unpack_k8(oracle.pack_k8(q), K), q)
    # the three orders hold the same nibbles: every word's population of nibble values agrees along its own axis
    can, n8i = oracle.pack_canonical(q), oracle.pack_n8i(q)
    nib = lambda w: np.sort(np.stack([(w >> (4 * t)) & 15 for t in range(8)], axis=-1), axis=-1)
    assert np.array_equal(nib(can), nib(n8i))


@settings(**COMMON)
@given(data=st.data())
def test_fragment_layout_inverts_the_forward_statement(oracle, data):
    g = data.draw(st.sampled_from([32, 64, 128]))
    K = 128 * data.draw(st.integers(1, 4))
    N = 16 * data.draw(st.integers(1, 6))
    rng = np.random.default_rng(data.draw(st.integers(0, 2 ** 32 - 1)))
    q = rng.integers(0, 16, (K, N), dtype=np.uint8)
    s = rng.standard_normal((K // g, N)).astype(np.float16)
    z = rng.integers(0, 16, (K // g, N)).astype(np.float16)
    wbuf, szbuf = _pack_fragment_order_numpy(q, s, z, g)
    q2, s2, z2 = oracle.unpack_packed(wbuf, szbuf, K, N, g)
    assert np.array_equal(q2, q)
    assert np.array_equal(s2.view(np.uint16), s.view(np.uint16)) and np.array_equal(z2.view(np.uint16), z.view(np.uint16))
    # moving one nibble of the buffer changes exactly one code
    i, t = int(rng.integers(0, wbuf.size)), int(rng.integers(0, 8))
    w2 = wbuf.copy()
    w2[i] ^= np.uint32(1) << np.uint32(4 * t)
    q3, _, _ = oracle.unpack_packed(w2, szbuf, K, N, g)
    assert int((q3 != q).sum()) == 1


@settings(**COMMON)
@given(data=st.data())
def test_quantiser_invariants(oracle, data):
    g = data.draw(st.sampled_from([32, 64, 128]))
    N = 8 * data.draw(st.integers(1, 3))
    rng = np.random.default_rng(data.draw(st.integers(0, 2 ** 32 - 1)))
    spread = 10.0 ** data.draw(st.integers(-3, 1))
    W = (rng.standard_normal((g, N)) * spread + rng.standard_normal((1, N)) * spread).astype(np.float32)
    q, s, z = oracle.quantise(W, g)
    sf, zf = s.astype(np.float64), z.astype(np.float64)
    assert q.min() >= 0 and q.max() <= 15 and (zf >= 0).all() and (zf <= 15).all() and (sf > 0).all()
    # codes that were not clamped reproduce their weight to half a step (of the rounded scale)
    what = (q.astype(np.float64) - zf) * sf
    free = (q > 0) & (q < 15)
    assert (np.abs(what - W)[free] <= 0.5 * np.broadcast_to(sf, W.shape)[free] * (1 + 1e-6) + 1e-12).all()
    # the column minimum lands on code 0 or the zero-point was clamped at 0; the maximum on 15 or below
    assert ((q.min(axis=0) == 0) | (zf[0] == 0) | (zf[0] == 15)).all()
