"""The argument behind the pruned second pass of the SnapKV-style score, checked
on the CPU in fp64 with a small model of what the kernel keeps (host logic, no
GPU): one pass over the keys that only knows, for every token, the sum of its
soft-max numerators over the window rows and the sum of their squares, taken
against a reference of the row sums that is renewed at fixed steps, must

  * enclose every exact column sum between the two bounds it forms at the end
    from the factors between reference and final sum of the rows: a centre times
    the sum, plus the root of the squares times the root of the squared
    excesses of the factors over the centre (no numerator is negative, so only
    the excesses count; Cauchy-Schwarz), likewise downwards, for three centres
    around the factors' mean; and the sum times the smallest and the largest
    factor,
  * and lead to exactly the oracle's kept set when the tokens that can still
    decide the selection are re-scored exactly and all others keep their
    upper bound (Algorithm 1, batch compression: the top-budget set with the
    lower index winning ties).

The model follows the kernel's schedule (64 tokens per step, a new reference
before steps 1 and 2 and then every 4 steps, trivial bounds for the tokens of
the first step, which has no reference) but none of its code; exact scores and
the selection come from the oracle.
"""

import numpy as np
import pytest

from oracle import fastcache_oracle as fo


STEP = 64          # tokens of one step (four blocks of 16)


def _epoch_of_step(t):
    return t if t < 2 else (2 if t < 4 else 2 + t // 4)


def _bounds(logits, lse, W):
    """logits [W][L] (-inf where masked), lse [W]: (lo, hi) of the column sums of the L - W prefix tokens."""
    L = logits.shape[1]
    n_prefix = L - W
    lo, hi = np.zeros(n_prefix), np.full(n_prefix, float(W))
    n_steps = (L + STEP - 1) // STEP
    run = np.full(W, -np.inf)            # log of every row's sum over the steps before this one
    ref = np.zeros(W)
    epoch = 0
    for t in range(n_steps):
        j0, j1 = t * STEP, min(L, (t + 1) * STEP)
        if _epoch_of_step(t) != epoch:   # renewal: the reference becomes the running sum
            epoch = _epoch_of_step(t)
            ref = np.where(np.isneginf(run), 0.0, run)
        if epoch >= 1 and j0 < n_prefix:
            jj = np.arange(j0, min(j1, n_prefix))
            num = np.exp(logits[:, jj] - ref[:, None])            # numerators against the reference
            rho = np.exp(ref - lse)                               # factor to the exact weight, per row
            c = num.sum(axis=0)
            s = np.sqrt((num ** 2).sum(axis=0))
            l, h = c * rho.min(), c * rho.max()
            for t in (-0.5, 0.0, 0.5):
                up = max(rho.mean() + t * rho.std(), 0.0)
                dn = max(rho.mean() - t * rho.std(), 0.0)
                h = np.minimum(h, up * c + s * np.sqrt((np.maximum(rho - up, 0.0) ** 2).sum()))
                l = np.maximum(l, dn * c - s * np.sqrt((np.maximum(dn - rho, 0.0) ** 2).sum()))
            lo[jj], hi[jj] = np.maximum(l, 0.0), np.minimum(h, float(W))
        run = np.logaddexp(run, np.logaddexp.reduce(logits[:, j0:j1], axis=1))
    return lo, hi


def _kept_through_bounds(keys, q, budget, pool_kernel):
    L, W = keys.shape[0], q.shape[0]
    scale = 1.0 / np.sqrt(keys.shape[1])
    logits = fo.window_logits(keys, q, scale)
    lse = fo.window_lse(keys, q, scale)
    exact = np.exp(logits - lse[:, None]).sum(axis=0)[:L - W]
    lo, hi = _bounds(logits, lse, W)
    assert (lo <= exact * (1 + 1e-12) + 1e-300).all(), "a lower bound exceeds the exact column sum"
    assert (hi >= exact * (1 - 1e-12)).all(), "an upper bound is below the exact column sum"
    n_sel, k_sel = L - W, budget - W
    value = hi.copy()
    marked = np.zeros(n_sel, dtype=bool)
    if 0 < k_sel < n_sel:
        plo, phi = fo.maxpool_same(lo, pool_kernel), fo.maxpool_same(hi, pool_kernel)
        t_lo = np.sort(plo)[-k_sel]      # the k-th largest pooled score lies between these two
        t_hi = np.sort(phi)[-k_sel]
        h = pool_kernel // 2
        for j in np.nonzero((phi >= t_lo) & (plo <= t_hi))[0]:
            a, b = max(0, j - h), min(n_sel, j + h + 1)
            marked[a:b] |= hi[a:b] >= plo[j]     # only these can carry the maximum of j's window
        value[marked] = exact[marked]
    pooled = fo.maxpool_same(value, pool_kernel) if n_sel else value
    kept = fo.select_topk(np.concatenate([pooled, np.full(W, np.inf)]), budget)
    return kept, marked.mean() if n_sel else 0.0


def _unit(rng, L, W, d, kind):
    keys = rng.standard_normal((L, d))
    q = rng.standard_normal((W, d))
    u = np.zeros(d)
    u[:8] = 1.0
    if kind == "outlier_channels":
        keys[:, rng.choice(d, 4, replace=False)] *= 8.0
    elif kind == "ramp":
        keys += u * (6.0 * np.arange(L) / L)[:, None]
        q += 2.0 * u
    elif kind == "sinks":
        keys[:4] += 8.0 * u
        q += 2.0 * u
    elif kind == "late_and_uneven":
        keys[L - 200:] += 5.0 * u
        q[::2] += 2.5 * u
    elif kind == "heavy_tail":
        keys[rng.random(L) < 0.01] += 4.0 * u
        q += 2.0 * u
    elif kind == "all_ties":
        q[:] = 0.0
    elif kind == "two_values":
        keys = np.where(rng.random((L, 1)) < 0.5, 0.25, 0.25 + 1.0 / 1024) * np.ones((L, d))
    return (keys.astype(np.float16).astype(np.float64), q.astype(np.float16).astype(np.float64))


@pytest.mark.parametrize("kind", ["gaussian", "outlier_channels", "ramp", "sinks", "late_and_uneven",
                                  "heavy_tail", "all_ties", "two_values"])
@pytest.mark.parametrize("L,W,pct,pool_kernel", [(2304, 64, 20, 7), (2111, 33, 45, 1), (2600, 16, 5, 15)])
def test_bounds_enclose_and_the_kept_set_is_the_oracles(kind, L, W, pct, pool_kernel):
    rng = np.random.default_rng(1000 * sum(map(ord, kind)) + L)
    keys, q = _unit(rng, L, W, 64, kind)
    budget = max(W, L * pct // 100)
    want = fo.select_topk(fo.snapkv_scores(keys, q, 1.0 / np.sqrt(64), pool_kernel), budget)
    got, frac = _kept_through_bounds(keys, q, budget, pool_kernel)
    assert (got == want).all(), (kind, np.setxor1d(got, want))
    assert 0.0 <= frac <= 1.0


def test_budget_edges_need_no_second_look():
    rng = np.random.default_rng(5)
    keys, q = _unit(rng, 2100, 64, 64, "gaussian")
    for budget in (64, 2100):
        want = fo.select_topk(fo.snapkv_scores(keys, q, 0.125, 7), budget)
        got, frac = _kept_through_bounds(keys, q, budget, 7)
        assert (got == want).all() and frac == 0.0
