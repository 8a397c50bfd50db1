"""Pins for the chunk-MLP compressor oracle (CPU only): closed forms for the
chunk plan, a network whose output is known in closed form (chunk means),
scalar brute force, pool bookkeeping."""

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


def test_gelu_against_scalar_tanh_form():
    v = np.linspace(-6, 6, 49)
    ref = [0.5 * x * (1 + math.tanh(math.sqrt(2 / math.pi) * (x + 0.044715 * x ** 3))) for x in v]
    np.testing.assert_allclose(mo.gelu(v), ref, rtol=1e-12, atol=1e-15)
    assert mo.gelu(np.array([0.0]))[0] == 0 and abs(mo.gelu(np.array([30.0]))[0] - 30) < 1e-12
    assert abs(mo.gelu(np.array([-30.0]))[0]) < 1e-12
    # the tanh form stays within 5e-4 of the erf form everywhere
    erf_form = [0.5 * x * (1 + math.erf(x / math.sqrt(2))) for x in v]
    assert np.abs(mo.gelu(v) - erf_form).max() < 5e-4


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
    y = mo.compress_rows(rows, plan, _mean_network(d, k, 1.0, 2.0), k).astype(np.float64)
    assert y.shape == (len(plan), d)
    for o, (s, e, m) in enumerate(plan):
        want = rows[s:min(s + k, e)].sum(axis=0) / k * (2.0 if m else 1.0)
        # the hidden value (mean + 12) is held in fp16: spacing 2^-7 in [8, 16)
        np.testing.assert_allclose(y[o], want, atol=2 ** -7)


def test_against_scalar_brute_force():
    rng = np.random.default_rng(1)
    L, d, k, hid = 11, 4, 3, 6
    rows = rng.standard_normal((L, d)).astype(np.float16).astype(np.float64)
    w = {"w1": [rng.standard_normal((hid, k * d)).astype(np.float16) * np.float16(0.5) for _ in range(2)],
         "b1": [rng.standard_normal(hid).astype(np.float32) for _ in range(2)],
         "w2": [rng.standard_normal((d, hid)).astype(np.float16) * np.float16(0.5) for _ in range(2)],
         "b2": [rng.standard_normal(d).astype(np.float32) for _ in range(2)]}
    plan = mo.chunk_plan(L, 2, 9, k)
    y = mo.compress_rows(rows, plan, w, k)
    for o, (s, e, m) in enumerate(plan):
        x = []
        for t in range(k):
            x += [float(v) for v in rows[s + t]] if s + t < e else [0.0] * d
        hvals = []
        for u in range(hid):
            z = sum(float(w["w1"][m][u][c]) * x[c] for c in range(k * d)) + float(w["b1"][m][u])
            g = 0.5 * z * (1 + math.tanh(math.sqrt(2 / math.pi) * (z + 0.044715 * z ** 3)))
            hvals.append(float(np.float16(g)))
        for c in range(d):
            z = sum(float(w["w2"][m][c][u]) * hvals[u] for u in range(hid)) + float(w["b2"][m][c])
            assert float(y[o][c]) == float(np.float16(z))


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
                        np.testing.assert_allclose(new, old, atol=2 ** -7)
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
