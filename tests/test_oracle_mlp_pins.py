"""Pins for the chunk-MLP compressor oracle (CPU only): closed forms for the
chunk plan, both activations against tabulated values of the normal
distribution function and of tanh, a network whose output is known in closed
form (chunk means), scalar brute force, pool bookkeeping."""

import math

import numpy as np
import pytest

from oracle import fastcache_oracle as fo
from oracle import mlp_compressor_oracle as mo


def test_chunk_plan_closed_form():
    assert mo.chunk_plan(12, 3, 9, 5) == [(0, 3, 0), (3, 9, 1), (8, 9, 1), (9, 12, 0)]
    for L, a, b, k in [(640, 35, 611, 5), (100, 0, 100, 5), (100, 0, 0, 4), (7, 7, 7, 3), (1, 0, 1, 8)]:
        plan = mo.chunk_plan(L, a, b, k)
        want = math.ceil(a / k) + math.ceil((b - a) / k) + math.ceil((L - b) / k)
        assert len(plan) == want == mo.compressed_length(L, a, b, k)
        starts = [p[0] for p in plan]
        assert starts == sorted(starts) and len(set(starts)) == len(starts)
        covered = set()
        for s, e, m in plan:
            covered |= set(range(s, min(s + k, e)))
            assert m == (1 if a <= s < b else 0)
        assert covered == set(range(L))                 # every token in exactly one chunk


# Standard normal distribution function at fixed points, from a table of the
# normal distribution (Phi(0.5), Phi(1), Phi(2), Phi(3)); GELU(v) = v * Phi(v).
PHI_TABLE = {0.5: 0.6914624612740131, 1.0: 0.8413447460685429, 2.0: 0.9772498680518208,
             3.0: 0.9986501019683699}
# textbook values of tanh
TANH_HALF, TANH_ONE = 0.46211715726000974, 0.7615941559557649


def test_gelu_erf_is_v_times_normal_cdf():
    """The definition of GELU against tabulated Phi values (both signs:
    Phi(-v) = 1 - Phi(v)) and against math.erf at other points."""
    for v, phi in PHI_TABLE.items():
        assert abs(float(mo.gelu_erf(v)) - v * phi) < 1e-15
        assert abs(float(mo.gelu_erf(-v)) + v * (1.0 - phi)) < 1e-15
    for v in (-6.0, -2.5, -0.1, 0.3, 1.7, 4.2, 7.0):
        assert abs(float(mo.gelu_erf(v)) - 0.5 * v * math.erfc(-v / math.sqrt(2.0))) < 1e-15
    v = np.linspace(-8, 8, 81)
    np.testing.assert_allclose(mo.gelu_erf(v) - mo.gelu_erf(-v), v, rtol=0, atol=1e-14)
    assert float(mo.gelu_erf(0.0)) == 0.0
    assert abs(float(mo.gelu_erf(30.0)) - 30.0) < 1e-12 and abs(float(mo.gelu_erf(-30.0))) < 1e-12
    # monotone above its minimum near v = -0.7518, whose value is about -0.17
    g = mo.gelu_erf(np.linspace(-0.75, 8, 500))
    assert (np.diff(g) > 0).all()
    assert abs(float(mo.gelu_erf(-0.7517915246935645)) + 0.16997120747) < 1e-9


def _solve_tanh_argument(target):
    """v with sqrt(2/pi) * (v + 0.044715 v^3) = target (bisection, plain floats)."""
    lo, hi = 0.0, 4.0
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if math.sqrt(2 / math.pi) * (mid + 0.044715 * mid ** 3) < target:
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


def test_gelu_tanh_at_textbook_tanh_points():
    """Where the cubic argument equals 1/2 or 1 the tanh form is v/2 * (1 +
    tanh(1/2)) or v/2 * (1 + tanh(1)); fixed literal values besides."""
    for target, th in ((0.5, TANH_HALF), (1.0, TANH_ONE)):
        v = _solve_tanh_argument(target)
        assert abs(float(mo.gelu_tanh(v)) - 0.5 * v * (1.0 + th)) < 1e-14
        assert abs(float(mo.gelu_tanh(-v)) + 0.5 * v * (1.0 - th)) < 1e-14
    for v, want in ((-3.0, -0.0036373920817729943), (-1.0, -0.15880800939172324),
                    (0.5, 0.34571400982514394), (1.0, 0.8411919906082768),
                    (2.0, 1.954597694087775), (3.0, 2.996362607918227)):
        assert abs(float(mo.gelu_tanh(v)) - want) < 1e-15
    v = np.linspace(-8, 8, 81)
    np.testing.assert_allclose(mo.gelu_tanh(v) - mo.gelu_tanh(-v), v, rtol=0, atol=1e-14)
    # the two named options are different functions, close to each other
    diff = np.abs(mo.gelu_tanh(v) - mo.gelu_erf(v))
    assert 1e-4 < diff.max() < 5e-4


def test_activation_is_an_argument():
    rng = np.random.default_rng(7)
    d, k, hid = 4, 2, 5
    rows = rng.standard_normal((6, d)).astype(np.float16).astype(np.float64)
    w = _random_weights(rng, d, k, hid)
    plan = mo.chunk_plan(6, 2, 4, k)
    ye = mo.compress_rows(rows, plan, w, k, "gelu_erf")
    yt = mo.compress_rows(rows, plan, w, k, "gelu_tanh")
    assert ye.dtype == np.float64 and (ye == mo.compress_rows(rows, plan, w, k)).all()
    assert 0 < np.abs(ye - yt).max() < 5e-3
    with pytest.raises(KeyError):
        mo.compress_rows(rows, plan, w, k, "relu")


def _random_weights(rng, d, k, hid):
    return {"w1": [rng.standard_normal((hid, k * d)).astype(np.float16) * np.float16(0.5) for _ in range(2)],
            "b1": [rng.standard_normal(hid).astype(np.float32) for _ in range(2)],
            "w2": [rng.standard_normal((d, hid)).astype(np.float16) * np.float16(0.5) for _ in range(2)],
            "b2": [rng.standard_normal(d).astype(np.float32) for _ in range(2)]}


def _mean_network(d, k, scale_text, scale_image, c=12.0):
    """hidden = d; unit u averages channel u over the k tokens of the chunk,
    shifted by +c so that gelu acts as the identity; the output removes c."""
    w1 = []
    for s in (scale_text, scale_image):
        w = np.zeros((d, k * d), dtype=np.float16)
        for t in range(k):
            w[np.arange(d), t * d + np.arange(d)] = s / k
        w1.append(w)
    eye = np.eye(d, dtype=np.float16)
    return {"w1": w1, "b1": [np.full(d, c, np.float32)] * 2, "w2": [eye, eye],
            "b2": [np.full(d, -c, np.float32)] * 2}


def test_mean_network_closed_form():
    """With the averaging network the compressed rows are the chunk means
    (zero-padded tails divide by k too), scaled x1 for text and x2 for image:
    pins chunk boundaries, padding, modality routing and output order."""
    rng = np.random.default_rng(0)
    L, d, k, a, b = 23, 8, 4, 5, 18
    rows = rng.standard_normal((L, d)).astype(np.float16).astype(np.float64)
    plan = mo.chunk_plan(L, a, b, k)
    for act in ("gelu_erf", "gelu_tanh"):
        y = mo.compress_rows(rows, plan, _mean_network(d, k, 1.0, 2.0), k, act)
        assert y.shape == (len(plan), d) and y.dtype == np.float64
        for o, (s, e, m) in enumerate(plan):
            want = rows[s:min(s + k, e)].sum(axis=0) / k * (2.0 if m else 1.0)
            # nothing is rounded on the way; gelu(v) = v to 1e-13 for v > 8
            np.testing.assert_allclose(y[o], want, atol=1e-12)


def test_against_scalar_brute_force():
    rng = np.random.default_rng(1)
    L, d, k, hid = 11, 4, 3, 6
    rows = rng.standard_normal((L, d)).astype(np.float16).astype(np.float64)
    w = _random_weights(rng, d, k, hid)
    plan = mo.chunk_plan(L, 2, 9, k)
    hidden = []
    y = mo.compress_rows(rows, plan, w, k, "gelu_erf", hidden_out=hidden)
    assert len(hidden) == len(plan)
    for o, (s, e, m) in enumerate(plan):
        x = []
        for t in range(k):
            x += [float(v) for v in rows[s + t]] if s + t < e else [0.0] * d
        hvals = []
        for u in range(hid):
            z = sum(float(w["w1"][m][u][c]) * x[c] for c in range(k * d)) + float(w["b1"][m][u])
            hvals.append(z * 0.5 * math.erfc(-z / math.sqrt(2.0)))    # z * Phi(z)
            assert abs(hvals[u] - hidden[o][u]) < 1e-14
        for c in range(d):
            z = sum(float(w["w2"][m][c][u]) * hvals[u] for u in range(hid)) + float(w["b2"][m][c])
            assert abs(float(y[o][c]) - z) < 1e-13


def test_batch_bookkeeping_and_transparent_copy():
    """k = 1 with the averaging network is a copy: pins the data movement
    through block tables; the pool bookkeeping matches the pruning stage's."""
    rng = np.random.default_rng(2)
    n_layers, n_heads, bs, d, nb = 2, 2, 4, 8, 32
    kv = rng.standard_normal((n_layers, nb, 2, n_heads, bs, d)).astype(np.float16)
    st = fo.FreeStack(nb)
    lens = np.array([10, 7, 13], dtype=np.int32)
    bt = np.full((3, 4), -1, dtype=np.int32)
    for r in range(3):
        n = fo.blocks_for(int(lens[r]), bs)
        bt[r, :n] = st.alloc(n)
    kv0, bt0, lens0 = kv.copy(), bt.copy(), lens.copy()
    img_b, img_e = np.array([2, 0, 13]), np.array([8, 7, 13])
    status = mo.compress_batch_mlp(kv, st, bt, lens, img_b, img_e, [1, 0, 1],
                                   _mean_network(d, 1, 1.0, 1.0), 1)
    assert status is None and lens.tolist() == [10, 7, 13]
    for r in (0, 2):
        for l in range(n_layers):
            for h in range(n_heads):
                for c in (0, 1):
                    for t in range(int(lens[r])):
                        new = kv[l, bt[r, t // bs], c, h, t % bs].astype(np.float64)
                        old = kv0[l, bt0[r, t // bs], c, h, t % bs].astype(np.float64)
                        # nothing but the store rounds, and old is an fp16 value already
                        np.testing.assert_allclose(new, old, rtol=0, atol=1e-12)
    assert (bt[1] == bt0[1]).all()
    live = []
    for r in range(3):
        live += bt[r, :fo.blocks_for(int(lens[r]), bs)].tolist()
    assert sorted(st.stack[:st.top].tolist() + live) == list(range(nb))
    # k = 5 shrinks the lengths to the chunk counts; errors leave state untouched
    snap = (kv.copy(), bt.copy(), lens.copy(), st.export())
    assert mo.compress_batch_mlp(kv, st, bt, lens, np.array([2, 0, 14]), img_e, [1, 1, 1],
                                 _mean_network(d, 5, 1.0, 1.0), 5) == "EINVAL"
    small = fo.FreeStack(nb)
    small.top = 1
    assert mo.compress_batch_mlp(kv, small, bt, lens, img_b, img_e, [1, 1, 1],
                                 _mean_network(d, 5, 1.0, 1.0), 5) == "ENOMEM"
    assert (kv == snap[0]).all() and (bt == snap[1]).all() and (lens == snap[2]).all()
    assert mo.compress_batch_mlp(kv, st, bt, lens, img_b, img_e, [1, 1, 1],
                                 _mean_network(d, 5, 1.0, 1.0), 5) is None
    assert lens.tolist() == [1 + 2 + 1, 2, 3]
