"""CPU oracle for the batched KV-cache compression stage (test infrastructure).

This module is TEST INFRASTRUCTURE, not product code.  It is a plain, slow,
fp64 numpy statement of what the stage computes, written so that it can be
checked against the definitions by eye.  Only the tests, the smoke check and
the `cpu_baseline` leg of the benchmark may import it.  It shares no code with
the HIP library and never imports it.

What the stage is (FastCache paper, Algorithm 1, the "batch compression" step
`kv_c <- C(kv, lambda)` between `P.Store(M.Prefill(batch))` and decoding; the
KV-cache memory pool of the "Dynamic Resource Management" section): for every
request of a batch, every layer and every head, score the cached tokens, keep
the `budget` best ones, write the kept K/V rows densely into freshly allocated
pool blocks, and hand the pre-compression ("zombie") blocks back to the pool
right after.  The paper runs existing pruning methods (SnapKV, key-L2-norm)
through this stage (the "existing methods run through FastCache" experiment)
but prints none of their formulas; the readings taken here are:

  * pool layout: kv[layer][block][0=K,1=V][head][slot][channel], fp16;
    a request owns a row of block ids shared by all layers and heads;
  * SnapKV-style score: the last `window` tokens are the observation window;
    query i of the window sits at position L-window+i and sees keys j at
    positions <= its own (causal); logits are scale * q.k with
    scale = 1/sqrt(head_dim); each row is soft-maxed over its visible keys;
    the rows are summed (not averaged) per key; the sums over the prefix
    (keys before the window) are max-pooled with an odd kernel, stride 1,
    same length, neighbours outside the prefix ignored; window tokens get
    score +inf so they are always kept;
  * SnapKV-style score with the row normalisers handed in: a caller whose
    attention kernel already produced, for every window query, the natural
    logarithm of the sum of exp(logit) over its visible keys (the "log-sum-exp"
    that fused attention kernels return) passes it in, and row i of the
    soft-max is then exp(logit - lse_i); with the exact log-sum-exp this is the
    same number as above;
  * key-norm score: minus the Euclidean norm of the key, so that keeping the
    best scores keeps the lowest norms; no pooling, no forced tokens;
  * streaming (StreamingLLM-style, one of the baselines the paper runs): no
    scoring; the first min(n_sink, budget) tokens ("attention sinks") and the
    most recent budget - sinks tokens are kept.  As a score: +inf on those
    tokens and 0 elsewhere, which the common selection rule turns into exactly
    that kept set;
  * selection: sort by (score descending, index ascending), keep the first
    `budget`, emit them in ascending index order;
  * pool: a LIFO stack of free block ids; a fresh pool holds
    stack[i] = n_blocks-1-i so the first pop is block 0;
  * compaction: new blocks for all compressed requests are popped first (in
    batch order), rows are copied, then all old blocks are pushed (in batch
    order, table order) and the request's length becomes its budget.
"""

import numpy as np

METHOD_NONE = 0
METHOD_SNAPKV = 1
METHOD_KNORM = 2
METHOD_STREAMING = 3


# --------------------------------------------------------------------------
# scoring
# --------------------------------------------------------------------------

def fetch_rows(kv_pool, layer, table_row, kv, head, n_tokens):
    """Rows 0..n_tokens-1 of one (layer, head) of a request, as fp64.

    kv_pool: float16 array [n_layers][n_blocks][2][n_heads][block_size][d].
    table_row: the request's block ids; token j lives in block
    table_row[j // block_size], slot j % block_size.
    """
    block_size = kv_pool.shape[4]
    j = np.arange(n_tokens)
    blocks = np.asarray(table_row)[j // block_size]
    return kv_pool[layer, blocks, kv, head, j % block_size, :].astype(np.float64)


def maxpool_same(a, kernel):
    """1-D max-pool, stride 1, output length == input length.

    out[j] = max(a[max(0, j-h)] ... a[min(n-1, j+h)]), h = kernel // 2.
    """
    assert kernel >= 1 and kernel % 2 == 1
    n = a.shape[0]
    h = kernel // 2
    out = np.empty_like(a)
    for j in range(n):
        out[j] = a[max(0, j - h):min(n, j + h + 1)].max()
    return out


def snapkv_scores(keys, q_window, scale, pool_kernel):
    """SnapKV-style observation-window score of every cached token.

    keys: [L][d] fp64, q_window: [W][d] fp64 (queries of the last W tokens).
    Returns fp64 [L]; the last W entries are +inf.
    """
    L = keys.shape[0]
    W = q_window.shape[0]
    assert 1 <= W <= L
    logits = scale * (q_window @ keys.T)                      # [W][L]
    q_pos = L - W + np.arange(W)                              # position of query i
    visible = np.arange(L)[None, :] <= q_pos[:, None]         # causal
    logits = np.where(visible, logits, -np.inf)
    row_max = logits.max(axis=1, keepdims=True)
    e = np.exp(logits - row_max)                              # exp(-inf) = 0
    p = e / e.sum(axis=1, keepdims=True)                      # row softmax
    col = p.sum(axis=0)                                       # sum over queries
    prefix = maxpool_same(col[:L - W], pool_kernel) if L > W else col[:0]
    return np.concatenate([prefix, np.full(W, np.inf)])


def window_logits(keys, q_window, scale):
    """Logits of the window queries against every key, -inf where key j lies
    after query i (query i sits at position L-W+i).  [W][L] fp64."""
    L = keys.shape[0]
    W = q_window.shape[0]
    assert 1 <= W <= L
    logits = scale * (q_window @ keys.T)
    q_pos = L - W + np.arange(W)
    visible = np.arange(L)[None, :] <= q_pos[:, None]
    return np.where(visible, logits, -np.inf)


def window_lse(keys, q_window, scale):
    """Natural log of the soft-max denominator of every window row:
    lse_i = log(sum over visible keys j of exp(logit_ij)).  fp64 [W]."""
    logits = window_logits(keys, q_window, scale)
    row_max = logits.max(axis=1)
    return row_max + np.log(np.exp(logits - row_max[:, None]).sum(axis=1))


def snapkv_scores_given_lse(keys, q_window, scale, pool_kernel, lse):
    """The SnapKV-style score when the caller supplies the rows' log-sum-exp:
    p_ij = exp(logit_ij - lse_i); column sums, pooling and the forced window
    as in snapkv_scores.  lse: [W]."""
    L = keys.shape[0]
    W = q_window.shape[0]
    lse = np.asarray(lse, dtype=np.float64)
    assert lse.shape == (W,)
    p = np.exp(window_logits(keys, q_window, scale) - lse[:, None])   # exp(-inf) = 0
    col = p.sum(axis=0)
    prefix = maxpool_same(col[:L - W], pool_kernel) if L > W else col[:0]
    return np.concatenate([prefix, np.full(W, np.inf)])


def knorm_scores(keys):
    """Key-norm score: minus the L2 norm of each key row.  keys: [L][d]."""
    return -np.sqrt((keys * keys).sum(axis=1))


def streaming_scores(n_tokens, budget, n_sink):
    """Sinks-plus-recent rule written as a score: +inf on the first
    min(n_sink, budget) tokens and on the last budget - sinks tokens, else 0."""
    sinks = min(int(n_sink), int(budget))
    recent = int(budget) - sinks
    s = np.zeros(n_tokens, dtype=np.float64)
    s[:sinks] = np.inf
    if recent > 0:
        s[n_tokens - recent:] = np.inf
    return s


def unit_scores(kv_pool, layer, table_row, head, n_tokens, method,
                q_window_unit=None, scale=None, pool_kernel=7, budget=None, n_sink=4,
                lse_unit=None):
    """Scores of one (request, layer, head) unit read through its block table.
    lse_unit: the window rows' log-sum-exp, if the caller supplies it."""
    if method == METHOD_STREAMING:
        return streaming_scores(n_tokens, budget, n_sink)
    keys = fetch_rows(kv_pool, layer, table_row, 0, head, n_tokens)
    if method == METHOD_SNAPKV:
        d = keys.shape[1]
        if scale is None or scale <= 0:
            scale = 1.0 / np.sqrt(d)
        q = np.asarray(q_window_unit, dtype=np.float64)
        if lse_unit is not None:
            return snapkv_scores_given_lse(keys, q, scale, pool_kernel, lse_unit)
        return snapkv_scores(keys, q, scale, pool_kernel)
    if method == METHOD_KNORM:
        return knorm_scores(keys)
    raise ValueError("unknown method")


# --------------------------------------------------------------------------
# selection
# --------------------------------------------------------------------------

def select_topk(scores, budget):
    """Indices of the `budget` largest scores, ties to the lower index,
    returned in ascending index order."""
    L = scores.shape[0]
    assert 1 <= budget <= L
    assert not np.isnan(scores).any()
    order = np.argsort(-scores, kind="stable")   # descending, stable => lower index first
    return np.sort(order[:budget]).astype(np.int32)


# --------------------------------------------------------------------------
# pool
# --------------------------------------------------------------------------

class FreeStack:
    """LIFO stack of free block ids; stack[0..top) are free."""

    def __init__(self, n_blocks):
        self.stack = (n_blocks - 1 - np.arange(n_blocks)).astype(np.int32)
        self.top = int(n_blocks)

    def num_free(self):
        return self.top

    def alloc(self, n):
        if n < 0 or n > self.top:
            raise MemoryError("pool exhausted")
        ids = self.stack[self.top - n:self.top][::-1].copy()   # ids[i] = stack[top-1-i]
        self.top -= n
        return ids

    def free(self, ids):
        ids = np.asarray(ids, dtype=np.int32)
        n = ids.shape[0]
        assert self.top + n <= self.stack.shape[0]
        self.stack[self.top:self.top + n] = ids
        self.top += n

    def export(self):
        return self.stack.copy(), self.top


def blocks_for(n_tokens, block_size):
    return (n_tokens + block_size - 1) // block_size


def copy_rows(kv_pool, layer, head, old_row, new_row, kept):
    """Compaction copy of one (layer, head): slot t of the new blocks receives
    the K and V rows of original token kept[t]."""
    bs = kv_pool.shape[4]
    for t, idx in enumerate(kept):
        for kv in (0, 1):
            kv_pool[layer, new_row[t // bs], kv, head, t % bs, :] = \
                kv_pool[layer, old_row[idx // bs], kv, head, idx % bs, :]


def window_lse_batch(kv_pool, block_tables, seq_lens, q_window, window, method, scale=None):
    """Log-sum-exp of the window rows of every SnapKV request of a batch:
    fp64 [n_req][n_layers][n_heads][window], zero for the other requests."""
    n_layers, _, _, n_heads, _, d = kv_pool.shape
    n_req = len(seq_lens)
    if scale is None or scale <= 0:
        scale = 1.0 / np.sqrt(d)
    out = np.zeros((n_req, n_layers, n_heads, int(window)), dtype=np.float64)
    for r in range(n_req):
        if int(method[r]) != METHOD_SNAPKV:
            continue
        for l in range(n_layers):
            for h in range(n_heads):
                keys = fetch_rows(kv_pool, l, block_tables[r], 0, h, int(seq_lens[r]))
                out[r, l, h] = window_lse(keys, np.asarray(q_window[r][l, h], dtype=np.float64),
                                          scale)
    return out


def per_request(value, n_req):
    """An int (the same for every request) or a sequence of n_req ints."""
    if np.ndim(value) == 0:
        return [int(value)] * n_req
    assert len(value) == n_req
    return [int(v) for v in value]


def validate_batch(stack, block_tables, seq_lens, window, method, budget,
                   pool_kernel, block_size, in_place=False):
    """Returns None if the batch is acceptable, else 'EINVAL' / 'ENOMEM'.
    window and pool_kernel: one int, or one per request (only looked at for
    SnapKV requests)."""
    n_req = len(seq_lens)
    if np.ndim(pool_kernel) == 0 and (pool_kernel < 1 or pool_kernel % 2 == 0):
        return "EINVAL"   # one size for the batch: checked whatever the methods
    window, pool_kernel = per_request(window, n_req), per_request(pool_kernel, n_req)
    need = 0
    for r in range(n_req):
        m, L, B = int(method[r]), int(seq_lens[r]), int(budget[r])
        if m == METHOD_NONE:
            continue
        if m not in (METHOD_SNAPKV, METHOD_KNORM, METHOD_STREAMING):
            return "EINVAL"
        if B < 1 or B > L:
            return "EINVAL"
        if m == METHOD_SNAPKV and (window[r] < 1 or L < window[r] or B < window[r]):
            return "EINVAL"
        if m == METHOD_SNAPKV and (pool_kernel[r] < 1 or pool_kernel[r] % 2 == 0):
            return "EINVAL"
        if blocks_for(L, block_size) > block_tables.shape[1]:
            return "EINVAL"
        need += blocks_for(B, block_size)
    if need > stack.num_free() and not in_place:
        return "ENOMEM"
    return None


def compress_batch(kv_pool, stack, block_tables, seq_lens, q_window, window,
                   method, budget, pool_kernel=7, scale=None, kept_override=None, n_sink=4,
                   in_place=False, lse_window=None):
    """The whole stage for one batch, in place.

    kv_pool      float16 [n_layers][n_blocks][2][n_heads][block_size][d]
    stack        FreeStack
    block_tables int32 [n_req][max_blocks], row r valid for ceil(L_r/bs) entries
    seq_lens     int array [n_req], L_r on entry, B_r on exit
    q_window     float16 [n_req][n_layers][n_heads][window][d] (may be None if
                 no request uses SnapKV); with per-request windows, a list of
                 n_req arrays [n_layers][n_heads][window_r][d] (None where the
                 request does not use SnapKV)
    window, pool_kernel  one int for the batch, or int arrays [n_req]
    method, budget  int arrays [n_req]
    n_sink       attention sinks kept by METHOD_STREAMING requests
    lse_window   optional [n_req][n_layers][n_heads][window]: the log-sum-exp of
                 every window row, supplied by the caller (SnapKV requests)
    in_place     compact inside the request's own blocks: the kept rows move to
                 slots 0..B-1 of its first ceil(B/bs) blocks (in ascending
                 order, which never overwrites a row still to be read because
                 kept[t] >= t), no block is allocated and the remaining blocks
                 are released
    kept_override   optional list (per request) of int arrays
                 [n_layers][n_heads][B_r]: use these kept indices instead of
                 the oracle's own selection (used to check the copy step on
                 a kept list produced elsewhere)

    Returns (status, scores, kept): status None / 'EINVAL' / 'ENOMEM' (then
    nothing was modified); scores[r] fp64 [n_layers][n_heads][L_r] and
    kept[r] int32 [n_layers][n_heads][B_r] (None for untouched requests).
    """
    n_layers, _, _, n_heads, bs, d = kv_pool.shape
    n_req = len(seq_lens)
    status = validate_batch(stack, block_tables, seq_lens, window, method,
                            budget, pool_kernel, bs, in_place)
    if status is not None:
        return status, None, None
    if scale is None or scale <= 0:
        scale = 1.0 / np.sqrt(d)
    pool_kernel = per_request(pool_kernel, n_req)

    # 1. score and select, every unit independently
    scores = [None] * n_req
    kept = [None] * n_req
    for r in range(n_req):
        m = int(method[r])
        if m == METHOD_NONE:
            continue
        L, B = int(seq_lens[r]), int(budget[r])
        scores[r] = np.empty((n_layers, n_heads, L), dtype=np.float64)
        kept[r] = np.empty((n_layers, n_heads, B), dtype=np.int32)
        for l in range(n_layers):
            for h in range(n_heads):
                qw = q_window[r][l, h] if m == METHOD_SNAPKV else None
                lse = (lse_window[r][l, h] if m == METHOD_SNAPKV and lse_window is not None
                       else None)
                s = unit_scores(kv_pool, l, block_tables[r], h, L, m, qw, scale,
                                pool_kernel[r], B, n_sink, lse)
                scores[r][l, h] = s
                if kept_override is not None:
                    kept[r][l, h] = kept_override[r][l, h]
                else:
                    kept[r][l, h] = select_topk(s, B)

    # 2. pop the new blocks of all compressed requests, in batch order
    old_rows = [None] * n_req
    new_rows = [None] * n_req
    for r in range(n_req):
        if int(method[r]) == METHOD_NONE:
            continue
        old_rows[r] = block_tables[r, :blocks_for(int(seq_lens[r]), bs)].copy()
        if in_place:
            new_rows[r] = old_rows[r][:blocks_for(int(budget[r]), bs)].copy()
        else:
            new_rows[r] = stack.alloc(blocks_for(int(budget[r]), bs))

    # 3. copy kept rows old -> new
    for r in range(n_req):
        if new_rows[r] is None:
            continue
        for l in range(n_layers):
            for h in range(n_heads):
                copy_rows(kv_pool, l, h, old_rows[r], new_rows[r], kept[r][l, h])

    # 4. reclaim the pre-compression blocks, rewrite tables and lengths
    for r in range(n_req):
        if new_rows[r] is None:
            continue
        stack.free(old_rows[r][new_rows[r].shape[0]:] if in_place else old_rows[r])
        block_tables[r, :] = -1
        block_tables[r, :new_rows[r].shape[0]] = new_rows[r]
        seq_lens[r] = int(budget[r])
    return None, scores, kept
