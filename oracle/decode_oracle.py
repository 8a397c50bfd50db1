"""CPU oracle of the decode-side pool traffic (test infrastructure; shares no
code with the library).

Algorithm 1, ExecuteDecoding: every decode step reads the (compressed) cache
of each request of the batch (M.Generate) and appends the new token's K and V
(UpdateKVCache).  The paper gives no formulas for either; what is computed
here is their plain definition on the paged pool:

  * append: request r's new K and V rows (one per layer and head) go to token
    position L_r, i.e. slot L_r % 16 of the block in table entry L_r // 16;
    when L_r is a multiple of 16 a block is popped first (requests in batch
    order); L_r becomes L_r + 1;
  * single-query attention of a decode step over the paged cache, per request,
    layer and head: out = softmax(scale * K q) . V over the request's L_r
    cached tokens (fp64 here).
"""

import numpy as np

from .fastcache_oracle import blocks_for, fetch_rows


def append_batch(kv_pool, stack, block_tables, seq_lens, new_kv, enable=None):
    """new_kv: float16 [n_req][n_layers][2][n_heads][d].  In place.  Returns
    None / 'EINVAL' / 'ENOMEM' (then nothing was modified)."""
    n_layers, _, _, n_heads, bs, d = kv_pool.shape
    n_req = len(seq_lens)
    on = [True] * n_req if enable is None else [bool(e) for e in enable]
    need = 0
    for r in range(n_req):
        if not on[r]:
            continue
        L = int(seq_lens[r])
        if L < 0 or L // bs >= block_tables.shape[1]:
            return "EINVAL"
        need += 1 if L % bs == 0 else 0
    if need > stack.num_free():
        return "ENOMEM"
    for r in range(n_req):
        if on[r] and int(seq_lens[r]) % bs == 0:
            block_tables[r, int(seq_lens[r]) // bs] = stack.alloc(1)[0]
    for r in range(n_req):
        if not on[r]:
            continue
        L = int(seq_lens[r])
        blk, slot = int(block_tables[r, L // bs]), L % bs
        for l in range(n_layers):
            for c in (0, 1):
                kv_pool[l, blk, c, :, slot, :] = new_kv[r, l, c]
        seq_lens[r] = L + 1
    return None


def decode_attention(kv_pool, block_tables, seq_lens, q, scale=None):
    """q: float16 [n_req][n_layers][n_heads][d].  Returns float64
    [n_req][n_layers][n_heads][d] (zeros for a request without tokens)."""
    n_layers, _, _, n_heads, bs, d = kv_pool.shape
    if scale is None or scale <= 0:
        scale = 1.0 / np.sqrt(d)
    out = np.zeros((len(seq_lens), n_layers, n_heads, d), dtype=np.float64)
    for r, L in enumerate(int(x) for x in seq_lens):
        if L == 0:
            continue
        for l in range(n_layers):
            for h in range(n_heads):
                keys = fetch_rows(kv_pool, l, block_tables[r], 0, h, L)
                vals = fetch_rows(kv_pool, l, block_tables[r], 1, h, L)
                z = scale * (keys @ q[r, l, h].astype(np.float64))
                p = np.exp(z - z.max())
                p /= p.sum()
                out[r, l, h] = p @ vals
    return out


def decode_attention_kept(kv_pool, block_tables, seq_lens, kept, q, scale=None):
    """The same attention over a pruned but uncompacted cache: request r, layer
    l, head h attends over the tokens kept[r][l, h] (ascending indices into
    its uncompressed cache).  kept[r]: int array [n_layers][n_heads][B_r]."""
    n_layers, _, _, n_heads, bs, d = kv_pool.shape
    if scale is None or scale <= 0:
        scale = 1.0 / np.sqrt(d)
    out = np.zeros((len(seq_lens), n_layers, n_heads, d), dtype=np.float64)
    for r, L in enumerate(int(x) for x in seq_lens):
        for l in range(n_layers):
            for h in range(n_heads):
                idx = np.asarray(kept[r][l, h], dtype=np.int64)
                if idx.size == 0:
                    continue
                keys = fetch_rows(kv_pool, l, block_tables[r], 0, h, L)[idx]
                vals = fetch_rows(kv_pool, l, block_tables[r], 1, h, L)[idx]
                z = scale * (keys @ q[r, l, h].astype(np.float64))
                p = np.exp(z - z.max())
                p /= p.sum()
                out[r, l, h] = p @ vals
    return out
