"""CPU oracle for the chunk-MLP ("lightweight multimodal") compressor shape
(test infrastructure; shares no code with the HIP library).

What the paper says (FastCache, "Multimodal Compressor" section): the KV-cache
is split at the modality boundary; image and text portions are compressed
independently by their own networks; for a compression factor k a portion of
length n becomes length n/k by reshaping chunks of k consecutive tokens and
processing each chunk; the compressed parts are concatenated in the original
order; two MLPs are used, one per modality.  The paper gives no depth, width,
activation or weights ("Offline Training" is out of scope), so the readings
taken here are:

  * one image span [img_begin, img_end) per request, text before and after it:
    three segments, each chunked on its own into ceil(n/k) chunks of k
    consecutive tokens, the last chunk of a segment zero-padded;
  * a chunk is the concatenation of its k token rows (k*d numbers); the
    network of the chunk's modality maps it to ONE row of d numbers:
        y = W2 . gelu(W1 . x + b1) + b2
    with W1 [hidden][k*d], W2 [d][hidden] and the tanh form of GELU,
        gelu(v) = v/2 * (1 + tanh(sqrt(2/pi) * (v + 0.044715 v^3)));
  * the same two networks serve every layer, every head, and both K and V;
  * precision: rows, W1, W2 are fp16 values; sums are exact (fp64 here); the
    hidden activations are rounded to fp16 before the second product (they are
    the fp16 operand of the second matrix product); the output row is rounded
    to fp16 (the pool's type);
  * pool: as for the pruning stage - new blocks of all requests are popped
    first (batch order), rows written, then all old blocks pushed (batch order,
    table order); the request's length becomes its number of chunks.
"""

import numpy as np

from .fastcache_oracle import blocks_for, fetch_rows


def gelu(v):
    return 0.5 * v * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (v + 0.044715 * v ** 3)))


def chunk_plan(n_tokens, img_begin, img_end, k):
    """[(first token, end of its segment, modality)] per output row, in order;
    modality 0 = text, 1 = image."""
    assert 0 <= img_begin <= img_end <= n_tokens and k >= 1
    plan = []
    for lo, hi, m in ((0, img_begin, 0), (img_begin, img_end, 1), (img_end, n_tokens, 0)):
        for s in range(lo, hi, k):
            plan.append((s, hi, m))
    return plan


def compressed_length(n_tokens, img_begin, img_end, k):
    return len(chunk_plan(n_tokens, img_begin, img_end, k))


def compress_rows(rows, plan, weights, k):
    """rows: [L][d] fp64 holding fp16 values.  weights: dict with w1, b1, w2,
    b2, each a pair (text, image).  Returns float16 [len(plan)][d]."""
    d = rows.shape[1]
    out = np.empty((len(plan), d), dtype=np.float16)
    for o, (s, seg_end, m) in enumerate(plan):
        x = np.zeros(k * d, dtype=np.float64)
        n = min(k, seg_end - s)
        x[:n * d] = rows[s:s + n].reshape(-1)
        h = gelu(weights["w1"][m].astype(np.float64) @ x + weights["b1"][m].astype(np.float64))
        h = h.astype(np.float16).astype(np.float64)
        y = weights["w2"][m].astype(np.float64) @ h + weights["b2"][m].astype(np.float64)
        out[o] = y.astype(np.float16)
    return out


def compress_batch_mlp(kv_pool, stack, block_tables, seq_lens, img_begin, img_end, enable,
                       weights, k):
    """The whole stage for one batch, in place (same pool conventions as the
    pruning stage).  enable[r] == 0 leaves request r untouched.
    Returns status (None / 'EINVAL' / 'ENOMEM')."""
    n_layers, _, _, n_heads, bs, d = kv_pool.shape
    n_req = len(seq_lens)
    need = 0
    for r in range(n_req):
        if not enable[r]:
            continue
        L = int(seq_lens[r])
        if not (0 <= img_begin[r] <= img_end[r] <= L) or L < 1:
            return "EINVAL"
        if blocks_for(L, bs) > block_tables.shape[1]:
            return "EINVAL"
        need += blocks_for(compressed_length(L, int(img_begin[r]), int(img_end[r]), k), bs)
    if need > stack.num_free():
        return "ENOMEM"
    plans, old_rows, new_rows = [None] * n_req, [None] * n_req, [None] * n_req
    for r in range(n_req):
        if not enable[r]:
            continue
        L = int(seq_lens[r])
        plans[r] = chunk_plan(L, int(img_begin[r]), int(img_end[r]), k)
        old_rows[r] = block_tables[r, :blocks_for(L, bs)].copy()
        new_rows[r] = stack.alloc(blocks_for(len(plans[r]), bs))
    for r in range(n_req):
        if plans[r] is None:
            continue
        L = int(seq_lens[r])
        for l in range(n_layers):
            for h in range(n_heads):
                for kv in (0, 1):
                    rows = fetch_rows(kv_pool, l, old_rows[r], kv, h, L)
                    y = compress_rows(rows, plans[r], weights, k)
                    for o in range(y.shape[0]):
                        kv_pool[l, new_rows[r][o // bs], kv, h, o % bs, :] = y[o]
    for r in range(n_req):
        if plans[r] is None:
            continue
        stack.free(old_rows[r])
        block_tables[r, :] = -1
        block_tables[r, :new_rows[r].shape[0]] = new_rows[r]
        seq_lens[r] = len(plans[r])
    return None
