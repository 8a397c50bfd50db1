"""Side-by-side harness: runs one workload through the HIP library (via the
C ABI binding) and through the CPU oracle on the same seeded bytes, and
compares them by the parity rules:

  * scores: |gpu - oracle| <= 2e-3*|oracle| + 1e-9 on finite entries, +inf
    must match exactly;
  * kept sets: identical, except that indices whose oracle score lies within
    2e-3*|T| of the oracle's budget-th largest score T may be swapped; and,
    with no tolerance, the GPU's kept list must be exactly the top-budget of
    the GPU's own fp32 scores under (score descending, index ascending);
  * gathered K/V bytes: bit-exact against the oracle's copy step applied to
    the GPU's kept lists (which is the oracle's full output wherever the kept
    lists agree);
  * block tables (valid entries), lengths, free stack [0, top) and top:
    bit-exact.
"""

import numpy as np

from oracle import fastcache_oracle as fo
from paper_2503_08461_amd import synth

REL_TOL = 2e-3
ABS_TOL = 1e-9


def check_scores(g, o, where=""):
    g = np.asarray(g, dtype=np.float64)
    inf_o = np.isposinf(o)
    assert (np.isposinf(g) == inf_o).all(), "forced-window (+inf) pattern differs " + where
    fin = ~inf_o
    assert np.isfinite(g[fin]).all(), "non-finite GPU score " + where
    err = np.abs(g[fin] - o[fin])
    bound = REL_TOL * np.abs(o[fin]) + ABS_TOL
    if not (err <= bound).all():
        k = int(np.argmax(err - bound))
        raise AssertionError("score mismatch %s: gpu %r oracle %r (worst of %d)" % (
            where, g[fin][k], o[fin][k], int((err > bound).sum())))
    return float((err / np.maximum(np.abs(o[fin]), 1e-300)).max()) if fin.any() else 0.0


def check_kept(gk, g_scores, ok, o_scores, budget, where=""):
    gk = np.asarray(gk)
    assert gk.shape[0] == budget, "kept count != budget " + where
    assert (np.diff(gk) > 0).all(), "kept not strictly ascending " + where
    assert gk.min() >= 0 and gk.max() < o_scores.shape[0], "kept index out of range " + where
    # self-consistency with no tolerance: top-budget of the GPU's own fp32 scores
    gs = np.asarray(g_scores, dtype=np.float32)
    own = np.sort(np.argsort(-gs, kind="stable")[:budget])
    assert (own == gk).all(), "kept list is not the exact top-budget of the GPU scores " + where
    if (gk == ok).all():
        return True
    # band around the oracle's threshold
    T = np.sort(o_scores)[::-1][budget - 1]
    sym = np.setxor1d(gk, ok)
    band = np.abs(o_scores[sym] - T) <= REL_TOL * abs(T) + ABS_TOL
    assert band.all(), "kept sets differ outside the threshold band %s: %s" % (where, sym[~band])
    return False


def check_kept_without_scores(gk, ok, o_scores, budget, where=""):
    """For a call that produces no scores (pruned second pass): the kept list
    against the oracle's, identical except inside the band around the oracle's
    threshold.  (The no-tolerance check of check_kept needs the GPU's own
    scores; here the same selection code runs on bounds and exact values, and
    the kept set is compared with the oracle's directly.)"""
    gk = np.asarray(gk)
    assert gk.shape[0] == budget, "kept count != budget " + where
    assert (np.diff(gk) > 0).all(), "kept not strictly ascending " + where
    assert gk.min() >= 0 and gk.max() < o_scores.shape[0], "kept index out of range " + where
    if (gk == ok).all():
        return True
    T = np.sort(o_scores)[::-1][budget - 1]
    sym = np.setxor1d(gk, ok)
    band = np.abs(o_scores[sym] - T) <= REL_TOL * abs(T) + ABS_TOL
    assert band.all(), "kept sets differ outside the threshold band %s: %s" % (where, sym[~band])
    return False


class SideBySide:
    """Small workloads only: the whole pool lives on the host too."""

    def __init__(self, wl, device="cuda:0", kv_host=None, q_host=None, score_mode=None,
                 in_place=False):
        import torch
        from paper_2503_08461_amd import fastcache as fc
        self.torch, self.fc, self.wl = torch, fc, wl
        self.dev = torch.device(device)
        self.kv_host = synth.fill_pool_host(wl) if kv_host is None else kv_host
        self.q_host = synth.fill_q_window_host(wl) if q_host is None else q_host
        self.kv_dev = torch.from_numpy(self.kv_host.copy()).to(self.dev)
        self.q_dev = torch.from_numpy(self.q_host.copy()).to(self.dev)
        self.pool = fc.fc_pool_create(self.kv_dev, wl.n_blocks, wl.n_layers, wl.n_heads,
                                      wl.head_dim)
        if score_mode is not None:
            fc.fc_set_score_mode(self.pool, score_mode)
        self.in_place = in_place
        fc.fc_set_compaction_mode(self.pool, 1 if in_place else 0)
        self.stack = fo.FreeStack(wl.n_blocks)
        # block tables through the public calls of each pool
        rows_o = synth.build_block_tables(wl, self.stack.alloc, self.stack.free,
                                          lambda ids, ix: ids[ix])
        rows_g = synth.build_block_tables(
            wl, lambda n: fc.fc_pool_alloc(self.pool, n),
            lambda ids: fc.fc_pool_free(self.pool, ids),
            lambda ids, ix: ids[torch.from_numpy(ix).to(self.dev)].contiguous())
        mb = wl.max_blocks + int(wl.extra.get("table_slack", 0))  # room for caches that grow
        self.bt_host = np.full((wl.n_req, mb), -1, dtype=np.int32)
        self.bt_dev = torch.full((wl.n_req, mb), -1, dtype=torch.int32, device=self.dev)
        for r in range(wl.n_req):
            self.bt_host[r, :rows_o[r].shape[0]] = rows_o[r]
            self.bt_dev[r, :rows_g[r].shape[0]] = rows_g[r]
        assert (self.bt_dev.cpu().numpy() == self.bt_host).all(), "pools hand out different ids"
        self.lens_o = wl.seq_lens.copy()
        self.lens_g = wl.seq_lens.copy()

    def close(self):
        self.fc.fc_pool_destroy(self.pool)

    def assert_pool_state_equal(self):
        stack_g, top_g = self.fc.fc_pool_export_state(self.pool)
        assert top_g == self.stack.top == self.fc.fc_pool_num_free(self.pool)
        assert (stack_g[:top_g] == self.stack.stack[:top_g]).all(), "free stacks differ"

    def compress_and_compare(self, methods=None, budgets=None, window=None, pool_kernel=None,
                             scale=0.0, n_sink=4, q_list=None, lse=None, scores=True):
        """One fc_compress_batch on both sides + full comparison.  Returns stats.
        lse = "oracle": the window rows' log-sum-exp comes from the oracle, is
        rounded to fp32 and handed to both sides (fc_compress_batch_lse);
        lse = "library": fc_window_lse computes it (checked against the oracle's)
        and the oracle runs the plain two-pass definition.
        With q_list (per request: fp16 array [n_layers][n_heads][window_r][d] or
        None), window and pool_kernel are int32 arrays and the call is
        fc_compress_batch_var.  scores=False: the call does not ask for the
        scores (which lets the library prune its second pass); kept lists,
        bytes and pool state are compared as always."""
        torch, fc, wl = self.torch, self.fc, self.wl
        methods = wl.methods if methods is None else methods
        budgets = wl.budgets if budgets is None else budgets
        window = wl.window if window is None else window
        pool_kernel = wl.pool_kernel if pool_kernel is None else pool_kernel
        n_lh = wl.n_layers * wl.n_heads
        comp = methods != fo.METHOD_NONE
        lens_before = self.lens_g.copy()
        n_scores = int(lens_before[comp].astype(np.int64).sum()) * n_lh
        n_kept = int(budgets[comp].astype(np.int64).sum()) * n_lh
        scores_dev = torch.full((max(n_scores, 1),), float("nan"), dtype=torch.float32,
                                device=self.dev)
        kept_dev = torch.full((max(n_kept, 1),), -7, dtype=torch.int32, device=self.dev)
        fc.fc_set_streaming_sinks(self.pool, n_sink)
        q_host = self.q_host
        lse_host = None
        if lse is not None:
            assert q_list is None
            lse_o = fo.window_lse_batch(self.kv_host, self.bt_host, lens_before, q_host, window,
                                        methods, scale if scale > 0 else None)
            if lse == "oracle":
                lse_host = lse_o.astype(np.float32)
                lse_dev = torch.from_numpy(lse_host).to(self.dev)
            else:
                lse_dev = torch.full(lse_o.shape, float("nan"), dtype=torch.float32,
                                     device=self.dev)
                fc.fc_window_lse(self.pool, self.bt_dev, lens_before, self.q_dev, window, methods,
                                 lse_dev, scale)
                got = lse_dev.cpu().numpy()
                snap = methods == fo.METHOD_SNAPKV
                assert np.isnan(got[~snap]).all(), "rows of other requests were written"
                # same bar as the scores: exp(logit - lse) moves by the absolute error of lse
                assert np.abs(got[snap] - lse_o[snap]).max() <= REL_TOL, "log-sum-exp differs"
                lse_dev[torch.from_numpy(~snap).to(self.dev)] = 0.0
            fc.fc_compress_batch_lse(self.pool, self.bt_dev, self.lens_g, self.q_dev, lse_dev,
                                     window, methods, budgets, pool_kernel, scale, scores_dev,
                                     kept_dev)
        elif q_list is None:
            fc.fc_compress_batch(self.pool, self.bt_dev, self.lens_g, self.q_dev, window,
                                 methods, budgets, pool_kernel, scale,
                                 scores_dev if scores else None, kept_dev)
        else:
            q_host = q_list
            packed = [q.reshape(-1) for r, q in enumerate(q_list)
                      if methods[r] == fo.METHOD_SNAPKV]
            q_flat = (torch.from_numpy(np.concatenate(packed)).to(self.dev) if packed else None)
            fc.fc_compress_batch_var(self.pool, self.bt_dev, self.lens_g, q_flat, window, methods,
                                     budgets, pool_kernel, scale, scores_dev if scores else None,
                                     kept_dev)
        torch.cuda.synchronize()
        scores_g = scores_dev.cpu().numpy()
        kept_g = kept_dev.cpu().numpy()

        # oracle: its own selection (scores + kept) on a scratch copy ...
        kv_a, st_a = self.kv_host.copy(), fo.FreeStack(wl.n_blocks)
        st_a.stack[:], st_a.top = self.stack.stack, self.stack.top
        bt_a, lens_a = self.bt_host.copy(), self.lens_o.copy()
        status, scores_o, kept_o = fo.compress_batch(
            kv_a, st_a, bt_a, lens_a, q_host, window, methods, budgets, pool_kernel,
            scale if scale > 0 else None, n_sink=n_sink, in_place=self.in_place,
            lse_window=lse_host)
        assert status is None, status

        # ... compared unit by unit
        stats = {"max_rel_err": 0.0, "units": 0, "units_kept_identical": 0}
        kept_g_lists = [None] * wl.n_req
        so = ko = 0
        for r in range(wl.n_req):
            if not comp[r]:
                continue
            L, B = int(lens_before[r]), int(budgets[r])
            sg = scores_g[so:so + n_lh * L].reshape(wl.n_layers, wl.n_heads, L)
            kg = kept_g[ko:ko + n_lh * B].reshape(wl.n_layers, wl.n_heads, B)
            so += n_lh * L
            ko += n_lh * B
            kept_g_lists[r] = kg
            for l in range(wl.n_layers):
                for h in range(wl.n_heads):
                    where = "(req %d layer %d head %d L %d B %d)" % (r, l, h, L, B)
                    if scores:
                        e = check_scores(sg[l, h], scores_o[r][l, h], where)
                        stats["max_rel_err"] = max(stats["max_rel_err"], e)
                        same = check_kept(kg[l, h], sg[l, h], kept_o[r][l, h],
                                          scores_o[r][l, h], B, where)
                    else:
                        same = check_kept_without_scores(kg[l, h], kept_o[r][l, h],
                                                         scores_o[r][l, h], B, where)
                    stats["units"] += 1
                    stats["units_kept_identical"] += int(same)

        # oracle copy step applied to the GPU's kept lists = expected final state
        status, _, _ = fo.compress_batch(
            self.kv_host, self.stack, self.bt_host, self.lens_o, q_host, window,
            methods, budgets, pool_kernel, scale if scale > 0 else None,
            kept_override=kept_g_lists, n_sink=n_sink, in_place=self.in_place)
        assert status is None
        self.compare_state()
        return stats

    def compare_state(self):
        wl = self.wl
        assert (self.lens_g == self.lens_o).all(), "lengths differ"
        bt_g = self.bt_dev.cpu().numpy()
        kv_g = self.kv_dev.cpu().numpy()
        bs = wl.block_size
        for r in range(wl.n_req):
            L = int(self.lens_o[r])
            n = fo.blocks_for(L, bs)
            assert (bt_g[r, :n] == self.bt_host[r, :n]).all(), "block table row %d differs" % r
            for i in range(n):
                b = self.bt_host[r, i]
                valid = min(bs, L - i * bs)
                a = kv_g[:, b, :, :, :valid, :].view(np.uint16)
                e = self.kv_host[:, b, :, :, :valid, :].view(np.uint16)
                assert (a == e).all(), "K/V bytes differ in request %d block %d" % (r, i)
        self.assert_pool_state_equal()
        # conservation: every id exactly once across free stack and live tables
        live = []
        for r in range(wl.n_req):
            live += bt_g[r, :fo.blocks_for(int(self.lens_g[r]), bs)].tolist()
        stack_g, top_g = self.fc.fc_pool_export_state(self.pool)
        assert sorted(stack_g[:top_g].tolist() + live) == list(range(wl.n_blocks))


def check_unit_on_device(kv_dev, q_unit, old_ids, new_ids, layer, head, L, B, method, window,
                         pool_kernel, scores_g, kept_g, where=""):
    """Full-size workloads: checks ONE (request, layer, head) unit of a finished
    fc_compress_batch against the oracle.  The unit's old blocks are downloaded
    (they are intact after the call: compaction writes only into blocks that
    were free), the oracle scores / selects / copies on a private mini pool,
    and the new blocks are downloaded for the byte comparison.

    kv_dev: device pool tensor; q_unit: [window][d] fp16 numpy (or None);
    old_ids / new_ids: int numpy arrays; scores_g fp32 [L], or None for a call
    that did not ask for the scores (the kept list is then checked against the
    oracle's scores alone); kept_g int32 [B].
    Returns (max relative score error, kept lists identical?)."""
    import torch
    bs, d = kv_dev.shape[4], kv_dev.shape[5]
    n_old, n_new = len(old_ids), len(new_ids)
    dev = kv_dev.device
    mini = np.zeros((1, n_old + n_new, 2, 1, bs, d), dtype=np.float16)
    oi = torch.from_numpy(np.asarray(old_ids, dtype=np.int64)).to(dev)
    ni = torch.from_numpy(np.asarray(new_ids, dtype=np.int64)).to(dev)
    mini[0, :n_old, :, 0] = kv_dev[layer, oi, :, head].cpu().numpy()
    table = np.arange(n_old)
    s_o = fo.unit_scores(mini, 0, table, 0, L, method, q_unit, None, pool_kernel)
    k_o = fo.select_topk(s_o, B)
    if scores_g is None:
        err = 0.0
        same = check_kept_without_scores(kept_g, k_o, s_o, B, where)
    else:
        err = check_scores(scores_g, s_o, where)
        same = check_kept(kept_g, scores_g, k_o, s_o, B, where)
    fo.copy_rows(mini, 0, 0, table, n_old + np.arange(n_new), kept_g)
    got = kv_dev[layer, ni, :, head].cpu().numpy()            # [n_new][2][bs][d]
    for i in range(n_new):
        valid = min(bs, B - i * bs)
        a = got[i, :, :valid].view(np.uint16)
        e = mini[0, n_old + i, :, 0, :valid].view(np.uint16)
        assert (a == e).all(), "gathered K/V bytes differ %s new block %d" % (where, i)
    return err, same


# ---- chunk-MLP compressor: error bound of the kernel's arithmetic ---------------

U16 = 2.0 ** -11          # unit round-off of fp16
H_ABS = 1e-4              # fp32 accumulation of k*d products + fast-math activation, absolute


def mlp_error_bound(y, hidden, w2):
    """What the kernel's arithmetic may differ from the exact row by, element
    by element.  The kernel holds the hidden activations as the fp16 operand
    of its second matrix product and stores fp16 rows:
        |h~_u - h_u| <= U16 |h_u| + H_ABS
        |y~_c - y_c| <= U16 |y_c| + sum_u |W2_cu| |h~_u - h_u|   (+ fp32 sums, << the rest)
    y [rows][d], hidden [rows][hidden] from the oracle, w2 [d][hidden]."""
    dh = U16 * np.abs(hidden) + H_ABS
    return U16 * np.abs(y) * 1.01 + dh @ np.abs(w2.astype(np.float64)).T + 1e-6
