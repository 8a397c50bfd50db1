"""High-concurrency stress (config 5): repeated admit -> compress -> decode
append -> free cycles on a pool kept near 90% occupancy, with the oracle's
free stack driven by the same operations.  After every cycle the pool state
must be bit-exact with the oracle's and every block id must be owned exactly
once; sampled units of every compression call are checked element by element.

The full LLaVA-1.5-7B layer count would need about 1 TiB for 256 resident
requests of up to 16384 tokens, so the layer count is 2 here; the per-layer
kernel shapes (32 heads x 128, fp16, lengths up to 16384) are the real ones."""

import numpy as np
import pytest

from oracle import fastcache_oracle as fo
from paper_2503_08461_amd import synth

pytestmark = pytest.mark.gpu

N_CYCLES = 50
SAMPLES_PER_CALL = 3


def test_config5_alloc_compress_append_free_cycles():
    import torch
    from paper_2503_08461_amd import fastcache as fc
    from parity_util import check_unit_on_device

    wl = synth.make_workload(5)
    dev = torch.device("cuda:0")
    if wl.pool_bytes() + (10 << 30) > torch.cuda.get_device_properties(0).total_memory:
        pytest.skip("pool does not fit this device")
    R, bs, W = wl.n_req, wl.block_size, wl.window
    n_lh = wl.n_layers * wl.n_heads
    max_blocks = 16384 // bs + 2
    rng = np.random.Generator(np.random.PCG64(wl.seed + 77))

    kv = torch.empty(wl.pool_shape(), dtype=torch.float16, device=dev)
    synth.fill_pool_device(wl, kv)
    q = synth.fill_q_window_device(wl, dev)
    pool = fc.fc_pool_create(kv, wl.n_blocks, wl.n_layers, wl.n_heads, wl.head_dim)
    st = fo.FreeStack(wl.n_blocks)
    skeleton = np.zeros((0, wl.n_blocks, 2, wl.n_heads, bs, wl.head_dim), np.float16)

    bt_g = torch.full((R, max_blocks), -1, dtype=torch.int32, device=dev)
    bt_o = np.full((R, max_blocks), -1, dtype=np.int32)
    lens_g = np.zeros(R, dtype=np.int32)       # 0 = slot empty
    lens_o = np.zeros(R, dtype=np.int32)
    compressed = np.zeros(R, dtype=bool)
    new_len = iter(rng.integers(512, 16385, size=100000).tolist())
    pct_of = wl.extra["pct"]

    def admit(r, L):
        n = fo.blocks_for(L, bs)
        ids = fc.fc_pool_alloc(pool, n)
        bt_g[r, :n] = ids
        bt_o[r, :n] = st.alloc(n)
        lens_g[r] = lens_o[r] = L
        compressed[r] = False

    def check_state(tag):
        stack_g, top_g = fc.fc_pool_export_state(pool)
        assert top_g == st.top == fc.fc_pool_num_free(pool), tag
        assert (stack_g[:top_g] == st.stack[:top_g]).all(), tag + ": free stacks differ"
        btg = bt_g.cpu().numpy()
        live = []
        for r in range(R):
            n = fo.blocks_for(int(lens_o[r]), bs) if lens_o[r] else 0
            assert (btg[r, :n] == bt_o[r, :n]).all(), tag + ": table row %d" % r
            live += bt_o[r, :n].tolist()
        assert (lens_g == lens_o).all()
        assert top_g + len(live) == wl.n_blocks, tag + ": blocks not conserved"
        assert sorted(stack_g[:top_g].tolist() + live) == list(range(wl.n_blocks)), \
            tag + ": a block is owned twice or lost"

    try:
        # initial residents: the configured 256 requests fill the pool to 90%
        for r in range(R):
            admit(r, int(wl.seq_lens[r]))
        check_state("initial")
        n_calls = n_sampled = 0
        worst = 0.0
        for cycle in range(N_CYCLES):
            # ---- compress: uncompressed requests, trimmed to what fits -------------
            methods = np.zeros(R, dtype=np.int32)
            budgets = np.ones(R, dtype=np.int32)
            free = fc.fc_pool_num_free(pool)
            picked = []
            for r in rng.permutation(R):
                if lens_o[r] == 0 or compressed[r] or len(picked) >= 48:
                    continue
                m = int(wl.methods[r])
                B = synth.budget_from_pct(int(lens_o[r]), int(pct_of[r]), m, W)
                need = fo.blocks_for(B, bs)
                if need <= free:
                    free -= need
                    methods[r], budgets[r] = m, B
                    picked.append(int(r))
            if cycle == 1 and picked:
                # over-ask on purpose: every live uncompressed request at once
                m2, b2 = methods.copy(), budgets.copy()
                for r in range(R):
                    if lens_o[r] and not compressed[r]:
                        m2[r] = int(wl.methods[r])
                        b2[r] = max(int(lens_o[r]) - 1, W)
                lens_try = lens_g.copy()
                with pytest.raises(fc.FastCacheError) as ei:
                    fc.fc_compress_batch(pool, bt_g, lens_try, q, W, m2, b2, wl.pool_kernel)
                assert ei.value.code == fc.FC_ENOMEM
                assert (lens_try == lens_g).all()
                check_state("after refused call")
            if picked:
                lens_before = lens_g.copy()
                old_tables = bt_o.copy()
                comp = methods != 0
                n_s = int(lens_before[comp].astype(np.int64).sum()) * n_lh
                n_k = int(budgets[comp].astype(np.int64).sum()) * n_lh
                scores = torch.empty(n_s, dtype=torch.float32, device=dev)
                kept = torch.empty(n_k, dtype=torch.int32, device=dev)
                fc.fc_compress_batch(pool, bt_g, lens_g, q, W, methods, budgets, wl.pool_kernel,
                                     0.0, scores, kept)
                status, _, _ = fo.compress_batch(skeleton, st, bt_o, lens_o, None, W, methods,
                                                 budgets, wl.pool_kernel)
                assert status is None
                torch.cuda.synchronize()
                n_calls += 1
                compressed[picked] = True
                # sampled units of this call
                offs, so, ko = {}, 0, 0
                for r in range(R):
                    if comp[r]:
                        offs[r] = (so, ko)
                        so += n_lh * int(lens_before[r])
                        ko += n_lh * int(budgets[r])
                for r in rng.choice(picked, size=min(SAMPLES_PER_CALL, len(picked)), replace=False):
                    r = int(r)
                    l, h = int(rng.integers(wl.n_layers)), int(rng.integers(wl.n_heads))
                    L, B = int(lens_before[r]), int(budgets[r])
                    lh = l * wl.n_heads + h
                    so, ko = offs[r]
                    sg = scores[so + lh * L: so + (lh + 1) * L].cpu().numpy()
                    kg = kept[ko + lh * B: ko + (lh + 1) * B].cpu().numpy()
                    qu = q[r, l, h].cpu().numpy() if methods[r] == fo.METHOD_SNAPKV else None
                    err, _ = check_unit_on_device(
                        kv, qu, old_tables[r, :fo.blocks_for(L, bs)],
                        bt_o[r, :fo.blocks_for(B, bs)], l, h, L, B, int(methods[r]), W,
                        wl.pool_kernel, sg, kg, "(cycle %d req %d layer %d head %d)" % (cycle, r, l, h))
                    worst = max(worst, err)
                    n_sampled += 1
            # ---- decode: append one token to some compressed requests -------------
            for r in range(R):
                if compressed[r] and rng.random() < 0.5 and fc.fc_pool_num_free(pool) > 0:
                    L = int(lens_o[r])
                    if L % bs == 0:
                        n = L // bs
                        bt_g[r, n:n + 1] = fc.fc_pool_alloc(pool, 1)
                        bt_o[r, n] = st.alloc(1)[0]
                    lens_g[r] = lens_o[r] = L + 1
            # ---- finish some compressed requests, admit new ones -------------------
            for r in range(R):
                if compressed[r] and rng.random() < 0.35:
                    n = fo.blocks_for(int(lens_o[r]), bs)
                    fc.fc_pool_free(pool, bt_g[r, :n].contiguous())
                    st.free(bt_o[r, :n])
                    bt_g[r, :] = -1
                    bt_o[r, :] = -1
                    lens_g[r] = lens_o[r] = 0
                    compressed[r] = False
            for r in range(R):
                if lens_o[r] == 0:
                    L = next(new_len)
                    # keep the pool near 90% occupancy
                    if fo.blocks_for(L, bs) <= fc.fc_pool_num_free(pool) - wl.n_blocks // 10:
                        admit(r, L)
            check_state("cycle %d" % cycle)
            print("cycle %d: %d picked, free %d/%d" % (cycle, len(picked), st.top, wl.n_blocks),
                  flush=True)
        assert n_calls >= N_CYCLES - 2 and n_sampled >= 20
        print("calls %d sampled units %d worst rel err %.2e" % (n_calls, n_sampled, worst))
        assert worst < 2e-3
    finally:
        fc.fc_pool_destroy(pool)
