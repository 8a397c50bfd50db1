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
        y = W2 . act(W1 . x + b1) + b2
    with W1 [hidden][k*d], W2 [d][hidden].  The paper says "MLP" and names no
    activation, so it is an argument: "gelu_erf" is GELU by its definition,
        gelu(v) = v * Phi(v) = v/2 * (1 + erf(v / sqrt(2))),
    "gelu_tanh" is the usual tanh approximation of it, a second named option,
        v/2 * (1 + tanh(sqrt(2/pi) * (v + 0.044715 v^3)));
  * the same two networks serve every layer, every head, and both K and V;
  * precision: rows, W1, W2 are fp16 VALUES and biases fp32 values (that is
    what the pool and the caller hold); everything in between is plain fp64
    with no intermediate rounding.  compress_rows returns fp64; only the write
    into the pool rounds, because the pool's storage type is fp16;
  * pool: as for the pruning stage - new blocks of all requests are popped
    first (batch order), rows written, then all old blocks pushed (batch order,
    table order); the request's length becomes its number of chunks.
"""

import math

import numpy as np

from .fastcache_oracle import blocks_for, fetch_rows


_erf = np.vectorize(math.erf, otypes=[np.float64])


def gelu_erf(v):
    """GELU by definition: v times the standard normal distribution function."""
    v = np.asarray(v, dtype=np.float64)
    return 0.5 * v * (1.0 + _erf(v / math.sqrt(2.0)))


def gelu_tanh(v):
    """The tanh approximation of GELU."""
    v = np.asarray(v, dtype=np.float64)
    return 0.5 * v * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (v + 0.044715 * v ** 3)))


ACTIVATIONS = {"gelu_erf": gelu_erf, "gelu_tanh": gelu_tanh}


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


def compress_rows(rows, plan, weights, k, activation="gelu_erf", hidden_out=None):
    """rows: [L][d] fp64 holding fp16 values.  weights: dict with w1, b1, w2,
    b2, each a pair (text, image).  Returns fp64 [len(plan)][d], unrounded.
    hidden_out (optional list) receives the hidden vector of every output row,
    for tests that bound the effect of a reduced-precision hidden operand."""
    act = ACTIVATIONS[activation]
    d = rows.shape[1]
    out = np.empty((len(plan), d), dtype=np.float64)
    for o, (s, seg_end, m) in enumerate(plan):
        x = np.zeros(k * d, dtype=np.float64)
        n = min(k, seg_end - s)
        x[:n * d] = rows[s:s + n].reshape(-1)
        h = act(weights["w1"][m].astype(np.float64) @ x + weights["b1"][m].astype(np.float64))
        out[o] = weights["w2"][m].astype(np.float64) @ h + weights["b2"][m].astype(np.float64)
        if hidden_out is not None:
            hidden_out.append(h)
    return out


def compress_batch_mlp(kv_pool, stack, block_tables, seq_lens, img_begin, img_end, enable,
                       weights, k, activation="gelu_erf", exact_out=None):
    """The whole stage for one batch, in place (same pool conventions as the
    pruning stage).  enable[r] == 0 leaves request r untouched.  The rows are
    rounded to the pool's type when they are stored; exact_out (optional dict)
    receives {(r, layer, head, kv): (unrounded fp64 rows [rows][d], their hidden
    vectors [rows][hidden])}.
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
                    hid = [] if exact_out is not None else None
                    y = compress_rows(rows, plans[r], weights, k, activation, hid)
                    if exact_out is not None:
                        exact_out[(r, l, h, kv)] = (y, np.array(hid))
                    for o in range(y.shape[0]):
                        kv_pool[l, new_rows[r][o // bs], kv, h, o % bs, :] = \
                            y[o].astype(kv_pool.dtype)
    for r in range(n_req):
        if plans[r] is None:
            continue
        stack.free(old_rows[r])
        block_tables[r, :] = -1
        block_tables[r, :new_rows[r].shape[0]] = new_rows[r]
        seq_lens[r] = len(plans[r])
    return None
