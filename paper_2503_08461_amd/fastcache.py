"""ctypes binding over libfastcache.so (the C ABI of include/fastcache.h).

Argument marshalling only: torch tensors supply device pointers, numpy arrays
supply host arrays, and every step of the stage runs in the library's HIP
kernels.  There is no fallback: if the library has not been built, or no GPU
is present, the calls raise.
"""

import ctypes
import os

import numpy as np

FC_OK, FC_EINVAL, FC_ENOMEM, FC_EDEVICE = 0, -1, -2, -3
FC_METHOD_NONE, FC_METHOD_SNAPKV, FC_METHOD_KNORM, FC_METHOD_STREAMING = 0, 1, 2, 3
FC_DTYPE_F16 = 0
FC_BLOCK_SIZE = 16
FC_N_KERNELS = 11
FC_SCORE_AUTO, FC_SCORE_TWO_PASS = 0, 1
FC_COMPACT_FRESH, FC_COMPACT_IN_PLACE = 0, 1
FC_ACT_GELU_ERF, FC_ACT_GELU_TANH = 0, 1

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libfastcache.so")

EXPORTS = [
    "fc_pool_create", "fc_pool_destroy", "fc_pool_alloc", "fc_pool_free",
    "fc_pool_num_free", "fc_pool_export_state", "fc_pool_import_state",
    "fc_pool_import_state_dev",
    "fc_compress_batch", "fc_compress_batch_noalloc", "fc_compress_batch_var", "fc_compress_batch_lse", "fc_window_lse",
    "fc_append_batch", "fc_decode_attention",
    "fc_decode_attention_kept",
    "fc_mlp_set_weights", "fc_compress_batch_mlp", "fc_set_compaction_mode", "fc_set_streaming_sinks", "fc_set_score_mode", "fc_set_score_pruning", "fc_set_debug_checks", "fc_set_profiling", "fc_get_kernel_times",
    "fc_kernel_name", "fc_last_error",
    "fc_sched_create", "fc_sched_destroy", "fc_sched_submit", "fc_sched_pending",
    "fc_sched_batch_target", "fc_sched_ready", "fc_sched_form_batch", "fc_sched_adjust",
]

_lib = None


class MlpWeights(ctypes.Structure):
    """struct fc_mlp_weights"""
    _fields_ = [("k", ctypes.c_int), ("hidden", ctypes.c_int), ("activation", ctypes.c_int),
                ("w1", ctypes.c_void_p * 2), ("b1", ctypes.c_void_p * 2),
                ("w2", ctypes.c_void_p * 2), ("b2", ctypes.c_void_p * 2)]


class FastCacheError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("libfastcache error %d: %s" % (code, text))
        self.code = code


def _hip_runtimes_loaded():
    paths = set()
    with open("/proc/self/maps") as f:
        for line in f:
            if "libamdhip64" in line:
                paths.add(line.split()[-1])
    return sorted(paths)


def load_library():
    """Loads libfastcache.so once.  torch is imported first so that the HIP
    runtime torch ships is the one the library binds to (same soname)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            "%s is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'`"
            % LIB_PATH)
    import torch  # noqa: F401  (loads libamdhip64 before the library asks for it)
    lib = ctypes.CDLL(LIB_PATH)
    runtimes = _hip_runtimes_loaded()
    if len(runtimes) > 1:
        raise RuntimeError("two HIP runtimes in one process: %s" % runtimes)
    vp, i32p, i = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32), ctypes.c_int
    lib.fc_pool_create.argtypes = [ctypes.POINTER(vp), vp, ctypes.c_size_t, i, i, i, i, i, i]
    lib.fc_pool_destroy.argtypes = [vp]
    lib.fc_pool_alloc.argtypes = [vp, i, vp, vp]
    lib.fc_pool_free.argtypes = [vp, vp, i, vp]
    lib.fc_pool_num_free.argtypes = [vp]
    lib.fc_pool_export_state.argtypes = [vp, i32p, ctypes.POINTER(i)]
    lib.fc_pool_import_state.argtypes = [vp, i32p, i]
    lib.fc_pool_import_state_dev.argtypes = [vp, vp, i, vp]
    lib.fc_compress_batch.argtypes = [vp, vp, i, i32p, vp, i, i32p, i32p, i, i,
                                      ctypes.c_float, vp, vp, vp]
    lib.fc_compress_batch_noalloc.argtypes = lib.fc_compress_batch.argtypes
    lib.fc_compress_batch_var.argtypes = [vp, vp, i, i32p, vp, i32p, i32p, i32p, i32p, i,
                                          ctypes.c_float, vp, vp, vp]
    lib.fc_compress_batch_lse.argtypes = [vp, vp, i, i32p, vp, vp, i, i32p, i32p, i, i,
                                          ctypes.c_float, vp, vp, vp]
    lib.fc_window_lse.argtypes = [vp, vp, i, i32p, vp, i, i32p, i, ctypes.c_float, vp, vp]
    lib.fc_append_batch.argtypes = [vp, vp, i, i32p, vp, i32p, i, vp]
    lib.fc_decode_attention.argtypes = [vp, vp, i, i32p, vp, vp, i, ctypes.c_float, vp]
    lib.fc_decode_attention_kept.argtypes = [vp, vp, i, i32p, i32p, vp, vp, vp, i, ctypes.c_float,
                                             vp]
    lib.fc_mlp_set_weights.argtypes = [vp, ctypes.POINTER(MlpWeights), vp]
    lib.fc_compress_batch_mlp.argtypes = [vp, vp, i, i32p, i32p, i32p, i32p, i, vp]
    lib.fc_set_score_mode.argtypes = [vp, i]
    lib.fc_set_score_pruning.argtypes = [vp, i]
    lib.fc_set_debug_checks.argtypes = [vp, i]
    lib.fc_set_streaming_sinks.argtypes = [vp, i]
    lib.fc_set_compaction_mode.argtypes = [vp, i]
    lib.fc_set_profiling.argtypes = [vp, i]
    lib.fc_get_kernel_times.argtypes = [vp, ctypes.POINTER(ctypes.c_float)]
    i64 = ctypes.c_int64
    lib.fc_sched_create.argtypes = [ctypes.POINTER(vp), i, i, i64]
    lib.fc_sched_destroy.argtypes = [vp]
    lib.fc_sched_destroy.restype = None
    lib.fc_sched_submit.argtypes = [vp, i64, i64, i, i]
    lib.fc_sched_pending.argtypes = [vp]
    lib.fc_sched_batch_target.argtypes = [vp]
    lib.fc_sched_ready.argtypes = [vp, i64]
    lib.fc_sched_form_batch.argtypes = [vp, i64, i, ctypes.POINTER(i64), i]
    lib.fc_sched_adjust.argtypes = [vp, i64]
    lib.fc_kernel_name.argtypes = [i]
    lib.fc_kernel_name.restype = ctypes.c_char_p
    lib.fc_last_error.restype = ctypes.c_char_p
    for name in EXPORTS:
        if name not in ("fc_kernel_name", "fc_last_error", "fc_sched_destroy"):
            getattr(lib, name).restype = i
    _lib = lib
    return lib


def _check(rc):
    if rc < 0:
        raise FastCacheError(rc, _lib.fc_last_error().decode())
    return rc


def _dev_ptr(t, dtype=None):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError("expected dtype %s, got %s" % (dtype, t.dtype))
    return ctypes.c_void_p(t.data_ptr())


def _stream_ptr(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _host_i32(a):
    if not (isinstance(a, np.ndarray) and a.dtype == np.int32 and a.flags.c_contiguous):
        raise ValueError("expected a contiguous int32 numpy array")
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


class PoolHandle:
    """Opaque fc_pool* plus the geometry it was created with (for marshalling)."""

    def __init__(self, ptr, kv, n_blocks, n_layers, n_heads, head_dim):
        self.ptr = ptr
        self.kv = kv  # keeps the caller's tensor alive
        self.n_blocks, self.n_layers, self.n_heads, self.head_dim = \
            n_blocks, n_layers, n_heads, head_dim


def fc_pool_create(kv, n_blocks, n_layers, n_heads, head_dim, block_size=FC_BLOCK_SIZE):
    """kv: torch fp16 device tensor holding kv[layer][block][2][head][16][head_dim]."""
    import torch
    lib = load_library()
    out = ctypes.c_void_p()
    _check(lib.fc_pool_create(ctypes.byref(out), _dev_ptr(kv, torch.float16),
                              kv.numel() * kv.element_size(), n_blocks, block_size,
                              n_layers, n_heads, head_dim, FC_DTYPE_F16))
    return PoolHandle(out, kv, n_blocks, n_layers, n_heads, head_dim)


def fc_pool_destroy(pool):
    lib = load_library()
    if pool.ptr:
        _check(lib.fc_pool_destroy(pool.ptr))
        pool.ptr = None


def fc_pool_alloc(pool, n_blocks, out_ids=None, stream=None):
    """Pops n_blocks ids into out_ids (int32 device tensor; created if None)."""
    import torch
    lib = load_library()
    if out_ids is None:
        out_ids = torch.empty(max(n_blocks, 0), dtype=torch.int32, device=pool.kv.device)
    if out_ids.numel() < n_blocks:
        raise ValueError("out_ids too small")
    _check(lib.fc_pool_alloc(pool.ptr, n_blocks, _dev_ptr(out_ids, torch.int32),
                             _stream_ptr(stream)))
    return out_ids


def fc_pool_free(pool, ids, stream=None):
    import torch
    lib = load_library()
    _check(lib.fc_pool_free(pool.ptr, _dev_ptr(ids, torch.int32), ids.numel(),
                            _stream_ptr(stream)))


def fc_pool_num_free(pool):
    return _check(load_library().fc_pool_num_free(pool.ptr))


def fc_pool_export_state(pool):
    """Returns (stack int32[n_blocks] numpy, top)."""
    lib = load_library()
    stack = np.empty(pool.n_blocks, dtype=np.int32)
    top = ctypes.c_int()
    _check(lib.fc_pool_export_state(pool.ptr, _host_i32(stack), ctypes.byref(top)))
    return stack, top.value


def fc_pool_import_state(pool, stack, top):
    lib = load_library()
    if stack.shape[0] != pool.n_blocks:
        raise ValueError("stack must have n_blocks entries")
    _check(lib.fc_pool_import_state(pool.ptr, _host_i32(stack), int(top)))


def fc_pool_import_state_dev(pool, dev_stack, top, stream=None):
    """dev_stack: int32 device tensor [n_blocks]; asynchronous on the stream."""
    import torch
    lib = load_library()
    if dev_stack.numel() != pool.n_blocks:
        raise ValueError("stack must have n_blocks entries")
    _check(lib.fc_pool_import_state_dev(pool.ptr, _dev_ptr(dev_stack, torch.int32), int(top),
                                        _stream_ptr(stream)))


def fc_compress_batch_noalloc(pool, block_tables, seq_lens, q_window, window, method, budget,
                              pool_kernel=7, scale=0.0, scores_out=None, kept_out=None,
                              stream=None):
    """fc_compress_batch through the entry point that allocates nothing."""
    return fc_compress_batch(pool, block_tables, seq_lens, q_window, window, method, budget,
                             pool_kernel, scale, scores_out, kept_out, stream,
                             _entry="fc_compress_batch_noalloc")


def fc_compress_batch(pool, block_tables, seq_lens, q_window, window, method, budget,
                      pool_kernel=7, scale=0.0, scores_out=None, kept_out=None, stream=None,
                      _entry="fc_compress_batch"):
    """block_tables: int32 device tensor [n_req][max_blocks] (in/out);
    seq_lens, method, budget: int32 numpy arrays [n_req] (seq_lens in/out);
    q_window: fp16 device tensor [n_req][n_layers][n_heads][window][head_dim] or None;
    scores_out / kept_out: optional fp32 / int32 device tensors (packed)."""
    import torch
    lib = load_library()
    n_req = int(seq_lens.shape[0])
    if block_tables.dim() != 2 or block_tables.shape[0] != n_req:
        raise ValueError("block_tables must be [n_req][max_blocks]")
    if method.shape[0] != n_req or budget.shape[0] != n_req:
        raise ValueError("method / budget must have n_req entries")
    if q_window is not None:
        want = (n_req, pool.n_layers, pool.n_heads, window, pool.head_dim)
        if tuple(q_window.shape) != want:
            raise ValueError("q_window must have shape %s" % (want,))
    comp = method != FC_METHOD_NONE
    if scores_out is not None:
        need = int((seq_lens[comp].astype(np.int64)).sum()) * pool.n_layers * pool.n_heads
        if scores_out.numel() < need:
            raise ValueError("scores_out too small")
    if kept_out is not None:
        need = int((budget[comp].astype(np.int64)).sum()) * pool.n_layers * pool.n_heads
        if kept_out.numel() < need:
            raise ValueError("kept_out too small")
    _check(getattr(lib, _entry)(
        pool.ptr, _dev_ptr(block_tables, torch.int32), int(block_tables.shape[1]),
        _host_i32(seq_lens), _dev_ptr(q_window, torch.float16), int(window),
        _host_i32(method), _host_i32(budget), n_req, int(pool_kernel), float(scale),
        _dev_ptr(scores_out, torch.float32), _dev_ptr(kept_out, torch.int32),
        _stream_ptr(stream)))


def fc_compress_batch_lse(pool, block_tables, seq_lens, q_window, lse_window, window, method,
                          budget, pool_kernel=7, scale=0.0, scores_out=None, kept_out=None,
                          stream=None):
    """As fc_compress_batch, with lse_window: fp32 device tensor
    [n_req][n_layers][n_heads][window], the log-sum-exp of every window row."""
    import torch
    lib = load_library()
    n_req = int(seq_lens.shape[0])
    if block_tables.dim() != 2 or block_tables.shape[0] != n_req:
        raise ValueError("block_tables must be [n_req][max_blocks]")
    if method.shape[0] != n_req or budget.shape[0] != n_req:
        raise ValueError("method / budget must have n_req entries")
    if q_window is not None:
        want = (n_req, pool.n_layers, pool.n_heads, window, pool.head_dim)
        if tuple(q_window.shape) != want:
            raise ValueError("q_window must have shape %s" % (want,))
    if lse_window is not None and tuple(lse_window.shape) != (n_req, pool.n_layers, pool.n_heads,
                                                              window):
        raise ValueError("lse_window must be [n_req][n_layers][n_heads][window]")
    comp = method != FC_METHOD_NONE
    if scores_out is not None:
        need = int((seq_lens[comp].astype(np.int64)).sum()) * pool.n_layers * pool.n_heads
        if scores_out.numel() < need:
            raise ValueError("scores_out too small")
    if kept_out is not None:
        need = int((budget[comp].astype(np.int64)).sum()) * pool.n_layers * pool.n_heads
        if kept_out.numel() < need:
            raise ValueError("kept_out too small")
    _check(lib.fc_compress_batch_lse(
        pool.ptr, _dev_ptr(block_tables, torch.int32), int(block_tables.shape[1]),
        _host_i32(seq_lens), _dev_ptr(q_window, torch.float16),
        _dev_ptr(lse_window, torch.float32), int(window), _host_i32(method), _host_i32(budget),
        n_req, int(pool_kernel), float(scale), _dev_ptr(scores_out, torch.float32),
        _dev_ptr(kept_out, torch.int32), _stream_ptr(stream)))


def fc_window_lse(pool, block_tables, seq_lens, q_window, window, method, lse_out, scale=0.0,
                  stream=None):
    """lse_out: fp32 device tensor [n_req][n_layers][n_heads][window], rows of the
    SnapKV requests (all requests if method is None) are written."""
    import torch
    lib = load_library()
    n_req = int(seq_lens.shape[0])
    if block_tables.dim() != 2 or block_tables.shape[0] != n_req:
        raise ValueError("block_tables must be [n_req][max_blocks]")
    if method is not None and method.shape[0] != n_req:
        raise ValueError("method must have n_req entries")
    want = (n_req, pool.n_layers, pool.n_heads, window, pool.head_dim)
    if q_window is not None and tuple(q_window.shape) != want:
        raise ValueError("q_window must have shape %s" % (want,))
    if lse_out is not None and tuple(lse_out.shape) != want[:4]:
        raise ValueError("lse_out must be [n_req][n_layers][n_heads][window]")
    _check(lib.fc_window_lse(
        pool.ptr, _dev_ptr(block_tables, torch.int32), int(block_tables.shape[1]),
        _host_i32(seq_lens), _dev_ptr(q_window, torch.float16), int(window),
        _host_i32(method) if method is not None else None, n_req, float(scale),
        _dev_ptr(lse_out, torch.float32), _stream_ptr(stream)))


def fc_compress_batch_var(pool, block_tables, seq_lens, q_window, window, method, budget,
                          pool_kernel, scale=0.0, scores_out=None, kept_out=None, stream=None):
    """As fc_compress_batch with window and pool_kernel as int32 numpy arrays
    [n_req]; q_window: flat fp16 device tensor, the SnapKV requests' queries
    [n_layers][n_heads][window_r][head_dim] one after the other, or None."""
    import torch
    lib = load_library()
    n_req = int(seq_lens.shape[0])
    if block_tables.dim() != 2 or block_tables.shape[0] != n_req:
        raise ValueError("block_tables must be [n_req][max_blocks]")
    for a in (window, method, budget, pool_kernel):
        if a.shape[0] != n_req:
            raise ValueError("window / method / budget / pool_kernel must have n_req entries")
    snap = method == FC_METHOD_SNAPKV
    need_q = int(window[snap].astype(np.int64).clip(min=0).sum()) * pool.n_layers * \
        pool.n_heads * pool.head_dim
    if need_q > 0 and (q_window is None or q_window.numel() < need_q):
        raise ValueError("q_window holds fewer than %d elements" % need_q)
    comp = method != FC_METHOD_NONE
    if scores_out is not None:
        need = int((seq_lens[comp].astype(np.int64)).sum()) * pool.n_layers * pool.n_heads
        if scores_out.numel() < need:
            raise ValueError("scores_out too small")
    if kept_out is not None:
        need = int((budget[comp].astype(np.int64)).sum()) * pool.n_layers * pool.n_heads
        if kept_out.numel() < need:
            raise ValueError("kept_out too small")
    _check(lib.fc_compress_batch_var(
        pool.ptr, _dev_ptr(block_tables, torch.int32), int(block_tables.shape[1]),
        _host_i32(seq_lens), _dev_ptr(q_window, torch.float16), _host_i32(window),
        _host_i32(method), _host_i32(budget), _host_i32(pool_kernel), n_req, float(scale),
        _dev_ptr(scores_out, torch.float32), _dev_ptr(kept_out, torch.int32),
        _stream_ptr(stream)))


def fc_append_batch(pool, block_tables, seq_lens, new_kv, enable=None, stream=None):
    """new_kv: fp16 device tensor [n_req][n_layers][2][n_heads][head_dim];
    seq_lens (in/out), enable: int32 numpy arrays [n_req]."""
    import torch
    lib = load_library()
    n_req = int(seq_lens.shape[0])
    if block_tables.dim() != 2 or block_tables.shape[0] != n_req:
        raise ValueError("block_tables must be [n_req][max_blocks]")
    want = (n_req, pool.n_layers, 2, pool.n_heads, pool.head_dim)
    if tuple(new_kv.shape) != want:
        raise ValueError("new_kv must have shape %s" % (want,))
    _check(lib.fc_append_batch(
        pool.ptr, _dev_ptr(block_tables, torch.int32), int(block_tables.shape[1]),
        _host_i32(seq_lens), _dev_ptr(new_kv, torch.float16),
        _host_i32(enable) if enable is not None else None, n_req, _stream_ptr(stream)))


def fc_decode_attention(pool, block_tables, seq_lens, q, out=None, scale=0.0, stream=None):
    """q: fp16 device tensor [n_req][n_layers][n_heads][head_dim]; returns out,
    fp32 device tensor of the same shape (created if None)."""
    import torch
    lib = load_library()
    n_req = int(seq_lens.shape[0])
    if block_tables.dim() != 2 or block_tables.shape[0] != n_req:
        raise ValueError("block_tables must be [n_req][max_blocks]")
    want = (n_req, pool.n_layers, pool.n_heads, pool.head_dim)
    if tuple(q.shape) != want:
        raise ValueError("q must have shape %s" % (want,))
    if out is None:
        out = torch.empty(want, dtype=torch.float32, device=q.device)
    elif tuple(out.shape) != want:
        raise ValueError("out must have shape %s" % (want,))
    _check(lib.fc_decode_attention(
        pool.ptr, _dev_ptr(block_tables, torch.int32), int(block_tables.shape[1]),
        _host_i32(seq_lens), _dev_ptr(q, torch.float16), _dev_ptr(out, torch.float32), n_req,
        float(scale), _stream_ptr(stream)))
    return out


def fc_decode_attention_kept(pool, block_tables, seq_lens, budget, kept, q, out=None, scale=0.0,
                             stream=None):
    """Attention over the kept tokens of an uncompacted cache; kept: int32
    device tensor packed [r][layer][head][budget_r] (fc_compress_batch's kept_out)."""
    import torch
    lib = load_library()
    n_req = int(seq_lens.shape[0])
    if block_tables.dim() != 2 or block_tables.shape[0] != n_req or budget.shape[0] != n_req:
        raise ValueError("block_tables must be [n_req][max_blocks], budget [n_req]")
    want = (n_req, pool.n_layers, pool.n_heads, pool.head_dim)
    if tuple(q.shape) != want:
        raise ValueError("q must have shape %s" % (want,))
    need = int(budget.astype(np.int64).sum()) * pool.n_layers * pool.n_heads
    if kept.numel() < need:
        raise ValueError("kept holds fewer than %d entries" % need)
    if out is None:
        out = torch.empty(want, dtype=torch.float32, device=q.device)
    _check(lib.fc_decode_attention_kept(
        pool.ptr, _dev_ptr(block_tables, torch.int32), int(block_tables.shape[1]),
        _host_i32(seq_lens), _host_i32(budget), _dev_ptr(kept, torch.int32),
        _dev_ptr(q, torch.float16), _dev_ptr(out, torch.float32), n_req, float(scale),
        _stream_ptr(stream)))
    return out


def fc_mlp_set_weights(pool, k, w1, b1, w2, b2, activation=FC_ACT_GELU_ERF, stream=None):
    """w1, b1, w2, b2: pairs (text, image) of device tensors: w1 fp16
    [hidden][k*head_dim], b1 fp32 [hidden], w2 fp16 [head_dim][hidden], b2 fp32 [head_dim];
    activation: FC_ACT_GELU_ERF or FC_ACT_GELU_TANH."""
    import torch
    lib = load_library()
    hidden = int(w1[0].shape[0])
    for m in range(2):
        if tuple(w1[m].shape) != (hidden, k * pool.head_dim) or \
                tuple(w2[m].shape) != (pool.head_dim, hidden) or \
                tuple(b1[m].shape) != (hidden,) or tuple(b2[m].shape) != (pool.head_dim,):
            raise ValueError("weight shapes do not match k, hidden and head_dim")
    w = MlpWeights()
    w.k, w.hidden, w.activation = int(k), hidden, int(activation)
    for m in range(2):
        w.w1[m] = _dev_ptr(w1[m], torch.float16).value
        w.b1[m] = _dev_ptr(b1[m], torch.float32).value
        w.w2[m] = _dev_ptr(w2[m], torch.float16).value
        w.b2[m] = _dev_ptr(b2[m], torch.float32).value
    _check(lib.fc_mlp_set_weights(pool.ptr, ctypes.byref(w), _stream_ptr(stream)))


def fc_compress_batch_mlp(pool, block_tables, seq_lens, img_begin, img_end, enable=None,
                          stream=None):
    """seq_lens (in/out), img_begin, img_end, enable: int32 numpy arrays [n_req]."""
    import torch
    lib = load_library()
    n_req = int(seq_lens.shape[0])
    if block_tables.dim() != 2 or block_tables.shape[0] != n_req:
        raise ValueError("block_tables must be [n_req][max_blocks]")
    _check(lib.fc_compress_batch_mlp(
        pool.ptr, _dev_ptr(block_tables, torch.int32), int(block_tables.shape[1]),
        _host_i32(seq_lens), _host_i32(img_begin), _host_i32(img_end),
        _host_i32(enable) if enable is not None else None, n_req, _stream_ptr(stream)))


def fc_set_compaction_mode(pool, mode):
    _check(load_library().fc_set_compaction_mode(pool.ptr, int(mode)))


def fc_set_streaming_sinks(pool, n_sink):
    _check(load_library().fc_set_streaming_sinks(pool.ptr, int(n_sink)))


def fc_set_score_mode(pool, mode):
    _check(load_library().fc_set_score_mode(pool.ptr, int(mode)))


def fc_set_debug_checks(pool, enable):
    _check(load_library().fc_set_debug_checks(pool.ptr, int(bool(enable))))


def fc_set_score_pruning(pool, enable):
    _check(load_library().fc_set_score_pruning(pool.ptr, 1 if enable else 0))


def fc_set_profiling(pool, enable):
    _check(load_library().fc_set_profiling(pool.ptr, 1 if enable else 0))


def fc_get_kernel_times(pool):
    """{kernel name: mean milliseconds} over the profiled fc_compress_batch calls
    since profiling was switched on (at most the last 32)."""
    lib = load_library()
    ms = (ctypes.c_float * FC_N_KERNELS)()
    _check(lib.fc_get_kernel_times(pool.ptr, ms))
    return {lib.fc_kernel_name(k).decode(): float(ms[k]) for k in range(FC_N_KERNELS)}


class Scheduler:
    """fc_sched_*: the host-side scheduler of the compress queue (same names
    as the C ABI; times in integer microseconds)."""

    def __init__(self, b_min, b_max, max_wait_us):
        lib = load_library()
        self._lib = lib
        out = ctypes.c_void_p()
        rc = lib.fc_sched_create(ctypes.byref(out), int(b_min), int(b_max), int(max_wait_us))
        if rc < 0:
            raise FastCacheError(rc, "fc_sched_create: invalid bounds")
        self.ptr = out
        self.b_max = int(b_max)

    def submit(self, req_id, arrival_us, seq_len, budget):
        return self._lib.fc_sched_submit(self.ptr, int(req_id), int(arrival_us), int(seq_len),
                                         int(budget)) == FC_OK

    def pending(self):
        return self._lib.fc_sched_pending(self.ptr)

    def batch_target(self):
        return self._lib.fc_sched_batch_target(self.ptr)

    def ready(self, now_us):
        return self._lib.fc_sched_ready(self.ptr, int(now_us)) == 1

    def form_batch(self, now_us, free_blocks):
        ids = (ctypes.c_int64 * self.b_max)()
        n = self._lib.fc_sched_form_batch(self.ptr, int(now_us), int(free_blocks), ids,
                                          self.b_max)
        if n < 0:
            raise FastCacheError(n, "fc_sched_form_batch")
        return [int(ids[i]) for i in range(n)]

    def adjust(self, service_us):
        return self._lib.fc_sched_adjust(self.ptr, int(service_us))

    def close(self):
        if self.ptr:
            self._lib.fc_sched_destroy(self.ptr)
            self.ptr = None

