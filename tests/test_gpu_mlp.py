"""GPU parity of the chunk-MLP compressor (fc_compress_batch_mlp) against its
CPU oracle (plain fp64, nothing rounded on the way) on seeded inputs: output
rows within the bound derived below, pool state bit-exact."""

import numpy as np
import pytest

from oracle import fastcache_oracle as fo
from oracle import mlp_compressor_oracle as mo
from paper_2503_08461_amd import synth
from parity_util import mlp_error_bound

pytestmark = pytest.mark.gpu

def make_weights(d, k, hidden, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    w = {"w1": [], "b1": [], "w2": [], "b2": []}
    for _ in range(2):
        w["w1"].append((rng.standard_normal((hidden, k * d)) / np.sqrt(k * d)).astype(np.float16))
        w["b1"].append((0.1 * rng.standard_normal(hidden)).astype(np.float32))
        w["w2"].append((rng.standard_normal((d, hidden)) / np.sqrt(hidden)).astype(np.float16))
        w["b2"].append((0.1 * rng.standard_normal(d)).astype(np.float32))
    return w


def run_case(lens, img_b, img_e, enable, d, k, hidden, n_layers=1, n_heads=2, seed=0,
             activation="gelu_erf", row_scale=1.0):
    import torch
    from paper_2503_08461_amd import fastcache as fc
    lens = np.array(lens, dtype=np.int32)
    nb = int(sum(synth.blocks_for(int(x)) for x in lens) * 2 + 8)
    wl = synth.Workload("mlp", n_layers, n_heads, d, nb, 16, 7, lens, np.zeros(len(lens), np.int32),
                        np.ones(len(lens), np.int32), seed, False, True)
    kv_host = synth.fill_pool_host(wl)
    if row_scale != 1.0:
        kv_host = (kv_host.astype(np.float32) * row_scale).astype(np.float16)
    w = make_weights(d, k, hidden, seed + 1)
    dev = torch.device("cuda:0")
    kv_dev = torch.from_numpy(kv_host.copy()).to(dev)
    pool = fc.fc_pool_create(kv_dev, nb, n_layers, n_heads, d)
    st = fo.FreeStack(nb)
    try:
        rows_o = synth.build_block_tables(wl, st.alloc, st.free, lambda ids, ix: ids[ix])
        rows_g = synth.build_block_tables(
            wl, lambda n: fc.fc_pool_alloc(pool, n), lambda ids: fc.fc_pool_free(pool, ids),
            lambda ids, ix: ids[torch.from_numpy(ix).to(dev)].contiguous())
        mb = wl.max_blocks
        bt_o = np.full((len(lens), mb), -1, dtype=np.int32)
        bt_g = torch.full((len(lens), mb), -1, dtype=torch.int32, device=dev)
        for r in range(len(lens)):
            bt_o[r, :rows_o[r].shape[0]] = rows_o[r]
            bt_g[r, :rows_g[r].shape[0]] = rows_g[r]
        tw = {key: [torch.from_numpy(a).to(dev) for a in w[key]] for key in w}
        fc.fc_mlp_set_weights(pool, k, tw["w1"], tw["b1"], tw["w2"], tw["b2"],
                              {"gelu_erf": fc.FC_ACT_GELU_ERF, "gelu_tanh": fc.FC_ACT_GELU_TANH}[activation])
        img_b = np.array(img_b, dtype=np.int32)
        img_e = np.array(img_e, dtype=np.int32)
        en = np.array(enable, dtype=np.int32)
        lens_g, lens_o = lens.copy(), lens.copy()
        fc.fc_compress_batch_mlp(pool, bt_g, lens_g, img_b, img_e, en)
        torch.cuda.synchronize()
        exact = {}
        status = mo.compress_batch_mlp(kv_host, st, bt_o, lens_o, img_b, img_e, en, w, k,
                                       activation, exact)
        assert status is None
        lens_before = lens
        assert (lens_g == lens_o).all()
        btg = bt_g.cpu().numpy()
        kvg = kv_dev.cpu().numpy()
        worst = 0.0
        for r in range(len(lens)):
            n = fo.blocks_for(int(lens_o[r]), 16)
            assert (btg[r, :n] == bt_o[r, :n]).all()
            if not en[r]:
                for i in range(n):
                    b = bt_o[r, i]
                    assert (kvg[:, b].view(np.uint16) == kv_host[:, b].view(np.uint16)).all()
                continue
            plan = mo.chunk_plan(int(lens_before[r]), int(img_b[r]), int(img_e[r]), k)
            w2_of_row = np.array([m for (_, _, m) in plan])
            for (rr, l, h, c), (y, hid) in exact.items():
                if rr != r:
                    continue
                g = np.stack([kvg[l, bt_o[r, o // 16], c, h, o % 16] for o in range(len(plan))])
                g = g.astype(np.float64)
                bound = np.empty_like(y)
                for m in (0, 1):
                    sel = w2_of_row == m
                    if sel.any():
                        bound[sel] = mlp_error_bound(y[sel], hid[sel], w["w2"][m])
                ratio = np.abs(g - y) / bound
                worst = max(worst, float(ratio.max()))
                assert (ratio <= 1.0).all(), "request %d unit (%d,%d,%d): error %.3g x the bound" % (
                    r, l, h, c, ratio.max())
        sg, tg = fc.fc_pool_export_state(pool)
        assert tg == st.top and (sg[:tg] == st.stack[:tg]).all()
        return worst
    finally:
        fc.fc_pool_destroy(pool)


@pytest.mark.parametrize("activation", ["gelu_erf", "gelu_tanh"])
def test_single_image_request_k5(activation):
    # LLaVA-like: 35 text, 576 image, 29 text tokens; k = 5 -> 7 + 116 + 6 rows
    run_case([640], [35], [611], [1], d=128, k=5, hidden=256, activation=activation)


@pytest.mark.parametrize("activation", ["gelu_erf", "gelu_tanh"])
@pytest.mark.parametrize("d,hidden,k", [(128, 256, 5), (128, 128, 4), (64, 256, 8), (64, 128, 1),
                                        (128, 256, 3)])
def test_shapes_and_factors(d, hidden, k, activation):
    run_case([333, 77, 1200], [10, 0, 1200], [300, 77, 1200], [1, 1, 1], d=d, k=k, hidden=hidden,
             n_layers=2, n_heads=3, seed=5, activation=activation)


def test_large_pre_activations_both_signs():
    """Rows scaled so that the pre-activations reach far into both tails of the
    activation (|v| up to about 12), where the erf form is v * (a tiny number)
    on one side and v itself on the other."""
    for activation in ("gelu_erf", "gelu_tanh"):
        run_case([200], [20], [180], [1], d=64, k=4, hidden=128, seed=21, activation=activation,
                 row_scale=6.0)


def test_pass_through_and_degenerate_spans():
    # disabled request untouched; all-text, all-image, single-token requests; ragged tails
    run_case([50, 64, 19, 1, 23], [0, 0, 19, 0, 11], [0, 64, 19, 1, 12], [1, 0, 1, 1, 1],
             d=128, k=5, hidden=256, seed=9)


def test_errors_leave_everything_untouched():
    import torch
    from paper_2503_08461_amd import fastcache as fc
    kv = torch.zeros((1, 8, 2, 1, 16, 64), dtype=torch.float16, device="cuda:0")
    pool = fc.fc_pool_create(kv, 8, 1, 1, 64)
    try:
        bt = torch.full((1, 8), -1, dtype=torch.int32, device="cuda:0")
        bt[0, :7] = fc.fc_pool_alloc(pool, 7)
        lens = np.array([100], np.int32)
        zero, full = np.array([0], np.int32), np.array([100], np.int32)
        with pytest.raises(fc.FastCacheError) as ei:          # weights not set
            fc.fc_compress_batch_mlp(pool, bt, lens, zero, full)
        assert ei.value.code == fc.FC_EINVAL
        w = make_weights(64, 2, 128, 0)
        tw = {key: [torch.from_numpy(a).cuda() for a in w[key]] for key in w}
        with pytest.raises(fc.FastCacheError) as ei:          # unknown activation
            fc.fc_mlp_set_weights(pool, 2, tw["w1"], tw["b1"], tw["w2"], tw["b2"], activation=7)
        assert ei.value.code == fc.FC_EINVAL
        fc.fc_mlp_set_weights(pool, 2, tw["w1"], tw["b1"], tw["w2"], tw["b2"])
        with pytest.raises(fc.FastCacheError) as ei:          # 50 rows need 4 blocks, 1 free
            fc.fc_compress_batch_mlp(pool, bt, lens, zero, full)
        assert ei.value.code == fc.FC_ENOMEM and lens[0] == 100
        with pytest.raises(fc.FastCacheError) as ei:
            fc.fc_compress_batch_mlp(pool, bt, lens, np.array([60], np.int32), np.array([50], np.int32))
        assert ei.value.code == fc.FC_EINVAL
        assert fc.fc_pool_num_free(pool) == 1
    finally:
        fc.fc_pool_destroy(pool)
