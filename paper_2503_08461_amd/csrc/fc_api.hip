// Host side of libfastcache: the C ABI declared in include/fastcache.h.
// Validates a batch with what the host scheduler knows (lengths, methods,
// budgets, free-block count), builds the per-request descriptors and issues
// the stage's kernels on the caller's stream.  No device->host transfer and
// no host wait happens inside fc_compress_batch once scratch is sized.

#include "../../include/fastcache.h"
#include "fc_internal.h"
#include "fc_plan.h"

#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <numeric>
#include <vector>

using namespace fc;

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

#define FC_HIP(call)                                                            \
  do {                                                                          \
    hipError_t e_ = (call);                                                     \
    if (e_ != hipSuccess)                                                       \
      return fail(FC_EDEVICE, "%s failed: %s", #call, hipGetErrorString(e_));   \
  } while (0)

// The calls of a launch sequence change the pool on the device step by step;
// if one of them fails after the first has been queued, the device state and
// the host mirrors no longer agree.  The pool is then marked and every later
// call on it is refused.
#define FC_HIP_STAGE(pool, call)                                                    \
  do {                                                                              \
    hipError_t e_ = (call);                                                         \
    if (e_ != hipSuccess) {                                                         \
      (pool)->poisoned = true;                                                      \
      return fail(FC_EDEVICE, "%s failed: %s; the pool is now unusable", #call,     \
                  hipGetErrorString(e_));                                           \
    }                                                                               \
  } while (0)

#define FC_CHECK_POOL(pool)                                                         \
  do {                                                                              \
    if (!(pool)) return fail(FC_EINVAL, "pool is NULL");                            \
    if ((pool)->poisoned)                                                           \
      return fail(FC_EDEVICE, "a device error in an earlier call left this pool in an " \
                              "undefined state; destroy it");                       \
  } while (0)

const char* const kKernelNames[K_COUNT] = {"plan_alloc", "snapkv_score", "knorm_score",
                                           "select",     "gather",       "reclaim",
                                           "fused_unit", "mlp_compress", "append",
                                           "decode_attention", "window_lse"};

// the planning module restates the public constants; they must agree
static_assert(PLAN_OK == FC_OK && PLAN_EINVAL == FC_EINVAL && PLAN_ENOMEM == FC_ENOMEM, "codes");
static_assert(PLAN_METHOD_SNAPKV == FC_METHOD_SNAPKV && PLAN_METHOD_KNORM == FC_METHOD_KNORM &&
              PLAN_METHOD_STREAMING == FC_METHOD_STREAMING && PLAN_METHOD_NONE == FC_METHOD_NONE,
              "methods");
static_assert(PLAN_SCORE_AUTO == FC_SCORE_AUTO && PLAN_SCORE_TWO_PASS == FC_SCORE_TWO_PASS,
              "score modes");
static_assert(K_COUNT == FC_N_KERNELS, "timing slots");
static_assert(kPlanBlockSize == FC_BLOCK_SIZE && kPlanMaxWindow == FC_MAX_WINDOW &&
              kPlanMaxSeqLen == FC_MAX_SEQ_LEN && kPlanMaxPoolKernel == FC_MAX_POOL_KERNEL &&
              kPlanFusedMaxLen == kFusedMaxLen && kPlanClasses == FC_MAX_WINDOW / 16 + 1,
              "limits");

// ---- scratch of the allocation-free entry point --------------------------------
// One file-scope device array per GPU, carved into the kept lists, the saved
// and new block ids and the descriptors.  Its name is only a host-side handle:
// the device address comes from hipGetSymbolAddress, once per device.
constexpr size_t kNoAllocKeptInts = (size_t)15 << 20;  // 60 MiB of kept indices
constexpr size_t kNoAllocIdInts = (size_t)256 << 10;   // 1 MiB of block ids
constexpr size_t kNoAllocMetaBytes = (size_t)16 << 10;
constexpr size_t kNoAllocKeptOff = 0;
constexpr size_t kNoAllocIdsOff = kNoAllocKeptOff + kNoAllocKeptInts * sizeof(int32_t);
constexpr size_t kNoAllocMetaOff = kNoAllocIdsOff + kNoAllocIdInts * sizeof(int32_t);
constexpr size_t kNoAllocBytes = kNoAllocMetaOff + kNoAllocMetaBytes;
static_assert(kNoAllocBytes == FC_NOALLOC_SCRATCH_BYTES, "the header states the size");
constexpr int kMaxDevices = 64;
unsigned char* g_scratch_ptr[kMaxDevices] = {};

size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

constexpr int kProfRing = 32;

}  // namespace

static __device__ __align__(256) unsigned char scratch[kNoAllocBytes];

namespace {

// Device address of `scratch` on the current device (looked up once per device).
int fixed_scratch_of_current_device(unsigned char** out) {
  int dev = 0;
  FC_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(FC_EDEVICE, "device index %d out of range", dev);
  if (!g_scratch_ptr[dev]) {
    unsigned char* ptr = nullptr;
    FC_HIP(hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch)));
    if (!ptr) return fail(FC_EDEVICE, "hipGetSymbolAddress returned a null address");
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return FC_OK;
}

}  // namespace

struct fc_pool;
namespace {
int release_verdict(fc_pool* p, hipStream_t stream, const char* what);
}

struct fc_pool {
  _Float16* kv = nullptr;
  size_t kv_bytes = 0;
  int n_blocks = 0, n_layers = 0, n_heads = 0, head_dim = 0;
  int32_t* stack = nullptr;  // device
  int top = 0;               // host mirror, exact
  bool poisoned = false;     // a launch failed in the middle of a stage: device and host disagree
  unsigned char* fixed_scratch = nullptr;  // this device's copy of the file-scope scratch array
  // ownership checks (debug mode): one int per block, 0 free, 1 handed out, 2 being released
  bool debug_checks = false;
  int32_t* owner = nullptr;
  int32_t* check_word = nullptr;  // device: what the last release check found

  // scratch, grown on demand
  float* raw_scores = nullptr;
  size_t raw_cap = 0;  // floats
  int32_t* kept = nullptr;
  size_t kept_cap = 0;  // ints
  int32_t* ids = nullptr;
  size_t ids_cap = 0;  // ints (old ids then new ids)
  char* dev_meta = nullptr;
  char* host_meta = nullptr;  // pinned
  size_t meta_cap = 0;
  hipEvent_t meta_event = nullptr;
  bool meta_pending = false;

  int32_t* error_flag = nullptr;  // device, one int, zero unless a kernel found something wrong
  int score_mode = FC_SCORE_AUTO;
  bool score_pruning = true;       // the fused kernel prunes the second pass of SnapKV units
  int n_sink = 4;
  int compact_mode = FC_COMPACT_FRESH;
  // chunk-MLP compressor weights in operand order (library-owned)
  int mlp_k = 0, mlp_hidden = 0, mlp_activation = 0;
  _Float16* mlp_w1p[2] = {nullptr, nullptr};
  _Float16* mlp_w2p[2] = {nullptr, nullptr};
  float* mlp_b1[2] = {nullptr, nullptr};
  float* mlp_b2[2] = {nullptr, nullptr};

  bool profiling = false;
  // event ring: the last kProfRing profiled calls, [call][kernel][start, stop]
  hipEvent_t ev[kProfRing][K_COUNT][2] = {};
  bool timed[kProfRing][K_COUNT] = {};
  int prof_calls = 0;  // profiled calls since profiling was last switched on
};

namespace {

template <typename T>
int grow(T** buf, size_t* cap, size_t need) {
  if (need <= *cap) return FC_OK;
  // the old buffer may still be in use by queued work
  FC_HIP(hipDeviceSynchronize());
  if (*buf) FC_HIP(hipFree(*buf));
  *buf = nullptr;
  *cap = 0;
  const size_t n = round_up(need + need / 8, 4096);
  FC_HIP(hipMalloc(reinterpret_cast<void**>(buf), n * sizeof(T)));
  *cap = n;
  return FC_OK;
}


int grow_meta(fc_pool* p, size_t need) {
  if (need <= p->meta_cap) return FC_OK;
  FC_HIP(hipDeviceSynchronize());
  if (p->dev_meta) FC_HIP(hipFree(p->dev_meta));
  if (p->host_meta) FC_HIP(hipHostFree(p->host_meta));
  p->dev_meta = nullptr;
  p->host_meta = nullptr;
  p->meta_cap = 0;
  p->meta_pending = false;
  const size_t n = round_up(need * 2, 4096);
  FC_HIP(hipMalloc(reinterpret_cast<void**>(&p->dev_meta), n));
  FC_HIP(hipHostMalloc(reinterpret_cast<void**>(&p->host_meta), n, hipHostMallocDefault));
  p->meta_cap = n;
  return FC_OK;
}

}  // namespace

extern "C" {

const char* fc_last_error(void) { return g_err; }

const char* fc_kernel_name(int i) { return (i >= 0 && i < K_COUNT) ? kKernelNames[i] : ""; }

int fc_pool_create(fc_pool** out, void* kv_base, size_t kv_bytes, int n_blocks, int block_size,
                   int n_layers, int n_heads, int head_dim, int dtype) {
  if (!out) return fail(FC_EINVAL, "out is NULL");
  *out = nullptr;
  if (!kv_base || (reinterpret_cast<uintptr_t>(kv_base) & 255))
    return fail(FC_EINVAL, "kv_base must be a 256-byte aligned device pointer");
  if (block_size != FC_BLOCK_SIZE) return fail(FC_EINVAL, "block_size must be 16");
  if (dtype != FC_DTYPE_F16) return fail(FC_EINVAL, "dtype must be FC_DTYPE_F16");
  if (head_dim != 64 && head_dim != 128) return fail(FC_EINVAL, "head_dim must be 64 or 128");
  if (n_blocks < 1 || n_layers < 1 || n_heads < 1) return fail(FC_EINVAL, "bad pool geometry");
  const size_t need = (size_t)n_layers * n_blocks * 2 * n_heads * FC_BLOCK_SIZE * head_dim * 2;
  if (kv_bytes < need)
    return fail(FC_EINVAL, "kv_bytes %zu is smaller than the pool geometry needs (%zu)", kv_bytes,
                need);
  FC_HIP(kernels_one_time_setup());
  FC_HIP(mlp_one_time_setup());
  // this device's copy of the allocation-free entry point's scratch array
  unsigned char* fixed = nullptr;
  if (int rc = fixed_scratch_of_current_device(&fixed)) return rc;
  fc_pool* p = new fc_pool();
  p->fixed_scratch = fixed;
  p->kv = static_cast<_Float16*>(kv_base);
  p->kv_bytes = kv_bytes;
  p->n_blocks = n_blocks;
  p->n_layers = n_layers;
  p->n_heads = n_heads;
  p->head_dim = head_dim;
  p->top = n_blocks;
  hipError_t e = hipMalloc(reinterpret_cast<void**>(&p->stack), (size_t)n_blocks * sizeof(int32_t));
  if (e == hipSuccess) e = launch_stack_init(p->stack, n_blocks, nullptr);
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&p->error_flag), sizeof(int32_t));
  if (e == hipSuccess) e = launch_zero_ints(p->error_flag, 1, nullptr);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&p->meta_event, hipEventDisableTiming);
  for (int c = 0; c < kProfRing && e == hipSuccess; ++c)
    for (int k = 0; k < K_COUNT && e == hipSuccess; ++k)
      for (int j = 0; j < 2 && e == hipSuccess; ++j) e = hipEventCreate(&p->ev[c][k][j]);
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) {
    fc_pool_destroy(p);
    return fail(FC_EDEVICE, "pool creation failed: %s", hipGetErrorString(e));
  }
  *out = p;
  return FC_OK;
}

int fc_pool_destroy(fc_pool* p) {
  if (!p) return FC_OK;
  (void)hipDeviceSynchronize();
  if (p->stack) (void)hipFree(p->stack);
  if (p->owner) (void)hipFree(p->owner);
  if (p->check_word) (void)hipFree(p->check_word);
  if (p->raw_scores) (void)hipFree(p->raw_scores);
  if (p->kept) (void)hipFree(p->kept);
  if (p->ids) (void)hipFree(p->ids);
  if (p->error_flag) (void)hipFree(p->error_flag);
  for (int m = 0; m < 2; ++m) {
    if (p->mlp_w1p[m]) (void)hipFree(p->mlp_w1p[m]);  // w2p lies in the same allocation
    if (p->mlp_b1[m]) (void)hipFree(p->mlp_b1[m]);
    if (p->mlp_b2[m]) (void)hipFree(p->mlp_b2[m]);
  }
  if (p->dev_meta) (void)hipFree(p->dev_meta);
  if (p->host_meta) (void)hipHostFree(p->host_meta);
  if (p->meta_event) (void)hipEventDestroy(p->meta_event);
  for (int c = 0; c < kProfRing; ++c)
    for (int k = 0; k < K_COUNT; ++k)
      for (int j = 0; j < 2; ++j)
        if (p->ev[c][k][j]) (void)hipEventDestroy(p->ev[c][k][j]);
  delete p;
  return FC_OK;
}

int fc_pool_alloc(fc_pool* p, int n, int32_t* dev_out_ids, void* stream) {
  FC_CHECK_POOL(p);
  if (n < 0) return fail(FC_EINVAL, "n_blocks < 0");
  if (n == 0) return FC_OK;
  if (!dev_out_ids) return fail(FC_EINVAL, "dev_out_ids is NULL");
  if (n > p->top) return fail(FC_ENOMEM, "asked for %d blocks, %d free", n, p->top);
  FC_HIP(launch_pool_pop(p->stack, p->top, n, dev_out_ids, p->debug_checks ? p->owner : nullptr,
                         p->n_blocks, p->error_flag, static_cast<hipStream_t>(stream)));
  p->top -= n;
  return FC_OK;
}

int fc_pool_free(fc_pool* p, const int32_t* dev_ids, int n, void* stream) {
  FC_CHECK_POOL(p);
  if (n < 0) return fail(FC_EINVAL, "n_blocks < 0");
  if (n == 0) return FC_OK;
  if (!dev_ids) return fail(FC_EINVAL, "dev_ids is NULL");
  if (p->top + n > p->n_blocks)
    return fail(FC_EINVAL, "freeing %d blocks with %d already free exceeds the pool (%d)", n,
                p->top, p->n_blocks);
  if (p->debug_checks) {
    // every id in range, handed out, and named once: checked before anything is pushed
    hipStream_t st = static_cast<hipStream_t>(stream);
    FC_HIP(launch_zero_ints(p->check_word, 1, st));
    FC_HIP(launch_owner_check_ids(dev_ids, n, p->n_blocks, p->owner, p->check_word, false, st));
    if (int rc = release_verdict(p, st, "fc_pool_free")) {
      (void)launch_owner_check_ids(dev_ids, n, p->n_blocks, p->owner, p->check_word, true, st);
      return rc;
    }
  }
  FC_HIP(launch_pool_push(p->stack, p->top, n, dev_ids, p->debug_checks ? p->owner : nullptr,
                         p->n_blocks, static_cast<hipStream_t>(stream)));
  p->top += n;
  return FC_OK;
}

int fc_pool_num_free(const fc_pool* p) { return p ? p->top : FC_EINVAL; }

int fc_pool_export_state(fc_pool* p, int32_t* host_stack, int* top) {
  if (!p || !host_stack || !top) return fail(FC_EINVAL, "NULL argument");
  FC_HIP(hipDeviceSynchronize());
  int32_t flag = 0;
  FC_HIP(hipMemcpy(&flag, p->error_flag, sizeof(flag), hipMemcpyDeviceToHost));
  if (flag) {
    // reported once: the flag starts over, so that a later export says what happened since
    FC_HIP(launch_zero_ints(p->error_flag, 1, nullptr));
    FC_HIP(hipDeviceSynchronize());
    return fail(FC_EDEVICE, "ownership checks: a block that was popped off the free stack was "
                            "not free (the free list is corrupt)");
  }
  FC_HIP(hipMemcpy(host_stack, p->stack, (size_t)p->n_blocks * sizeof(int32_t),
                   hipMemcpyDeviceToHost));
  *top = p->top;
  return FC_OK;
}

int fc_pool_import_state(fc_pool* p, const int32_t* host_stack, int top) {
  if (!p || !host_stack) return fail(FC_EINVAL, "NULL argument");
  if (top < 0 || top > p->n_blocks) return fail(FC_EINVAL, "top out of range");
  FC_HIP(hipDeviceSynchronize());
  FC_HIP(hipMemcpy(p->stack, host_stack, (size_t)p->n_blocks * sizeof(int32_t),
                   hipMemcpyHostToDevice));
  p->top = top;
  if (p->debug_checks) {  // what is not on the new stack counts as handed out
    FC_HIP(launch_owner_init(p->owner, p->stack, top, p->n_blocks, nullptr));
    FC_HIP(hipDeviceSynchronize());
  }
  return FC_OK;
}

int fc_set_compaction_mode(fc_pool* p, int mode) {
  if (!p) return fail(FC_EINVAL, "pool is NULL");
  if (mode != FC_COMPACT_FRESH && mode != FC_COMPACT_IN_PLACE)
    return fail(FC_EINVAL, "unknown compaction mode %d", mode);
  p->compact_mode = mode;
  return FC_OK;
}

int fc_set_streaming_sinks(fc_pool* p, int n_sink) {
  if (!p) return fail(FC_EINVAL, "pool is NULL");
  if (n_sink < 0) return fail(FC_EINVAL, "n_sink < 0");
  p->n_sink = n_sink;
  return FC_OK;
}

int fc_set_score_mode(fc_pool* p, int mode) {
  if (!p) return fail(FC_EINVAL, "pool is NULL");
  if (mode != FC_SCORE_AUTO && mode != FC_SCORE_TWO_PASS)
    return fail(FC_EINVAL, "unknown score mode %d", mode);
  p->score_mode = mode;
  return FC_OK;
}

int fc_set_debug_checks(fc_pool* p, int enable) {
  FC_CHECK_POOL(p);
  if (!enable) {
    p->debug_checks = false;
    return FC_OK;
  }
  FC_HIP(hipDeviceSynchronize());  // the free stack must be what the host mirror says
  if (!p->owner) FC_HIP(hipMalloc(reinterpret_cast<void**>(&p->owner), (size_t)p->n_blocks * sizeof(int32_t)));
  if (!p->check_word) FC_HIP(hipMalloc(reinterpret_cast<void**>(&p->check_word), sizeof(int32_t)));
  FC_HIP(launch_owner_init(p->owner, p->stack, p->top, p->n_blocks, nullptr));
  FC_HIP(hipDeviceSynchronize());
  p->debug_checks = true;
  return FC_OK;
}

int fc_set_score_pruning(fc_pool* p, int enable) {
  if (!p) return fail(FC_EINVAL, "pool is NULL");
  p->score_pruning = enable != 0;
  return FC_OK;
}

int fc_set_profiling(fc_pool* p, int enable) {
  if (!p) return fail(FC_EINVAL, "pool is NULL");
  p->profiling = enable != 0;
  p->prof_calls = 0;
  return FC_OK;
}

int fc_get_kernel_times(fc_pool* p, float* host_ms) {
  if (!p || !host_ms) return fail(FC_EINVAL, "NULL argument");
  const int n = std::min(p->prof_calls, kProfRing);
  for (int k = 0; k < K_COUNT; ++k) {
    double sum = 0.0;
    int cnt = 0;
    for (int c = 0; c < n; ++c) {
      if (!p->timed[c][k]) continue;
      float ms = 0.f;
      FC_HIP(hipEventSynchronize(p->ev[c][k][1]));
      FC_HIP(hipEventElapsedTime(&ms, p->ev[c][k][0], p->ev[c][k][1]));
      sum += ms;
      ++cnt;
    }
    host_ms[k] = cnt ? (float)(sum / cnt) : 0.f;
  }
  return FC_OK;
}

int fc_pool_import_state_dev(fc_pool* p, const int32_t* dev_stack, int top, void* stream) {
  if (!p || !dev_stack) return fail(FC_EINVAL, "NULL argument");
  if (top < 0 || top > p->n_blocks) return fail(FC_EINVAL, "top out of range");
  FC_HIP(launch_pool_push(p->stack, 0, p->n_blocks, dev_stack, nullptr, p->n_blocks,
                         static_cast<hipStream_t>(stream)));
  p->top = top;
  if (p->debug_checks)  // what is not on the new stack counts as handed out
    FC_HIP(launch_owner_init(p->owner, p->stack, top, p->n_blocks, static_cast<hipStream_t>(stream)));
  return FC_OK;
}

}  // extern "C"

namespace {

PoolView pool_view(fc_pool* p) {
  PoolView v;
  v.n_layers = p->n_layers;
  v.n_heads = p->n_heads;
  v.head_dim = p->head_dim;
  v.n_free = p->top;
  v.score_mode = p->score_mode;
  v.in_place = p->compact_mode == FC_COMPACT_IN_PLACE;
  return v;
}

// Ownership checks: waits for the check kernel on `stream` and reads its word.
int release_verdict(fc_pool* p, hipStream_t stream, const char* what) {
  int32_t word = 0;
  FC_HIP(hipStreamSynchronize(stream));
  FC_HIP(hipMemcpy(&word, p->check_word, sizeof(word), hipMemcpyDeviceToHost));
  if (word == 0) return FC_OK;
  return fail(FC_EINVAL, "%s: %s%s%s", what,
              (word & 1) ? "a block id lies outside the pool; " : "",
              (word & 2) ? "a block id is not handed out (double free, foreign id) or is named "
                           "twice; " : "",
              "nothing was changed");
}

// Descriptors and work lists to the device.  With the library's own scratch
// they go through the pinned staging buffer and one asynchronous copy; the
// allocation-free path sends them as kernel arguments, a few KB per launch.
int upload_meta(fc_pool* p, const char* image, size_t bytes, char* dev_dst, bool no_alloc,
                hipStream_t stream) {
  if (no_alloc) {
    for (size_t off = 0; off < bytes; off += sizeof(MetaChunk)) {
      MetaChunk c;
      const size_t n = std::min(sizeof(MetaChunk), bytes - off);
      memcpy(c.bytes, image + off, n);
      FC_HIP(launch_meta_upload(c, dev_dst + off, (int)n, stream));
    }
    return FC_OK;
  }
  if (p->meta_pending) {
    // the previous call's descriptor upload must have left the staging buffer
    FC_HIP(hipEventSynchronize(p->meta_event));
    p->meta_pending = false;
  }
  memcpy(p->host_meta, image, bytes);
  FC_HIP(hipMemcpyAsync(dev_dst, p->host_meta, bytes, hipMemcpyHostToDevice, stream));
  FC_HIP(hipEventRecord(p->meta_event, stream));
  p->meta_pending = true;
  return FC_OK;
}

// All entry points of the pruning stage.  host_window / host_pool_kernel are
// NULL for the calls that take one size for the whole batch.  no_alloc: every
// scratch buffer lies in the file-scope device array and nothing is allocated.
int compress_batch_impl(fc_pool* p, int32_t* dev_block_tables, int max_blocks_per_req,
                        int32_t* host_seq_lens, const void* dev_q_window,
                        const float* dev_lse_window, bool need_lse, const int32_t* host_window,
                        int window, const int32_t* host_method, const int32_t* host_budget,
                        int n_req, const int32_t* host_pool_kernel, int pool_kernel, float scale,
                        float* dev_scores_out, int32_t* dev_kept_out, void* stream_,
                        bool no_alloc) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  FC_CHECK_POOL(p);
  if (n_req > 0 && !dev_block_tables) return fail(FC_EINVAL, "NULL argument");

  // ---- plan with host-known quantities; nothing is touched on error -----------
  CompressArgs a;
  a.n_req = n_req;
  a.max_blocks = max_blocks_per_req;
  a.seq_lens = host_seq_lens;
  a.method = host_method;
  a.budget = host_budget;
  a.window_per_req = host_window;
  a.pool_kernel_per_req = host_pool_kernel;
  a.window = window;
  a.pool_kernel = pool_kernel;
  a.need_lse = need_lse;
  a.q_ok = dev_q_window && (reinterpret_cast<uintptr_t>(dev_q_window) & 15) == 0;
  a.lse_ok = dev_lse_window && (reinterpret_cast<uintptr_t>(dev_lse_window) & 3) == 0;
  const PoolView pv = pool_view(p);
  CompressPlan plan;
  if (plan_compress(pv, a, &plan) != PLAN_OK) return fail(plan.code, "%s", plan.message);
  const int n_comp = (int)plan.descs.size();
  if (n_comp == 0) return FC_OK;

  // ---- scratch: kept lists, saved ids, un-pooled scores, descriptors -----------
  const size_t desc_bytes = round_up((size_t)n_comp * sizeof(ReqDesc), 16);
  const size_t order_bytes = round_up((size_t)n_comp * sizeof(int32_t), 16);
  const size_t meta_bytes = desc_bytes + N_LISTS * order_bytes;
  const size_t n_ids = (size_t)plan.total_old + plan.total_new;
  int32_t* kept_buf = dev_kept_out;
  int32_t* ids_buf = nullptr;
  char* dev_meta = nullptr;
  int rc;
  const bool pruned_call = p->score_pruning && !dev_scores_out && !need_lse;
  if (no_alloc) {
    if (!p->fixed_scratch) return fail(FC_EDEVICE, "the fixed scratch array was not set up");
    if (n_comp > FC_NOALLOC_MAX_REQUESTS)
      return fail(FC_EINVAL, "%d requests exceed the %d of the allocation-free call", n_comp,
                  FC_NOALLOC_MAX_REQUESTS);
    if (plan.raw_floats > 0)
      return fail(FC_EINVAL, "the allocation-free call takes heads of at most %d tokens with "
                             "the default scheduling", kFusedMaxLen);
    if (!dev_kept_out && plan.kept_entries > kNoAllocKeptInts)
      return fail(FC_EINVAL, "%zu kept entries exceed the %zu of the fixed scratch (pass "
                             "dev_kept_out)", plan.kept_entries, kNoAllocKeptInts);
    if (n_ids > kNoAllocIdInts)
      return fail(FC_EINVAL, "%zu block ids exceed the %zu of the fixed scratch", n_ids,
                  kNoAllocIdInts);
    if (meta_bytes > kNoAllocMetaBytes) return fail(FC_EINVAL, "descriptors exceed the fixed scratch");
    if (!kept_buf) kept_buf = reinterpret_cast<int32_t*>(p->fixed_scratch + kNoAllocKeptOff);
    ids_buf = reinterpret_cast<int32_t*>(p->fixed_scratch + kNoAllocIdsOff);
    dev_meta = reinterpret_cast<char*>(p->fixed_scratch + kNoAllocMetaOff);
  } else {
    // (growth waits for the device and frees: it happens before anything is queued)
    if (!dev_kept_out && (rc = grow(&p->kept, &p->kept_cap, plan.kept_entries)) != FC_OK) return rc;
    if ((rc = grow(&p->ids, &p->ids_cap, n_ids)) != FC_OK) return rc;
    if ((rc = grow(&p->raw_scores, &p->raw_cap, plan.raw_floats)) != FC_OK) return rc;
    if ((rc = grow_meta(p, meta_bytes)) != FC_OK) return rc;
    if (!kept_buf) kept_buf = p->kept;
    ids_buf = p->ids;
    dev_meta = p->dev_meta;
  }
  std::vector<char> image(meta_bytes, 0);
  memcpy(image.data(), plan.descs.data(), (size_t)n_comp * sizeof(ReqDesc));
  size_t list_off[N_LISTS];
  int n_list[N_LISTS];
  for (int i = 0; i < N_LISTS; ++i) {
    list_off[i] = desc_bytes + (size_t)i * order_bytes;
    n_list[i] = (int)plan.lists[i].size();
    if (n_list[i] > 0)
      memcpy(image.data() + list_off[i], plan.lists[i].data(), (size_t)n_list[i] * sizeof(int32_t));
  }
  if ((rc = upload_meta(p, image.data(), meta_bytes, dev_meta, no_alloc, stream)) != FC_OK) return rc;

  BatchParams bp = {};
  bp.kv = p->kv;
  bp.n_blocks = p->n_blocks;
  bp.n_layers = p->n_layers;
  bp.n_heads = p->n_heads;
  bp.head_dim = p->head_dim;
  bp.stack = p->stack;
  bp.top_before = p->top;
  bp.total_new = plan.total_new;
  bp.total_old = plan.total_old;
  bp.descs = reinterpret_cast<const ReqDesc*>(dev_meta);
  auto dev_list = [&](int i) { return reinterpret_cast<const int32_t*>(dev_meta + list_off[i]); };
  bp.order_all = dev_list(LIST_ALL);
  bp.order_knorm = dev_list(LIST_KNORM);
  bp.n_comp = n_comp;  // plan_alloc / reclaim walk every descriptor
  bp.n_knorm = n_list[LIST_KNORM];
  bp.n_unfused = n_list[LIST_ALL];
  // per launch: order_snap / n_snap, order_fused / n_fused, window (of the class)
  bp.block_tables = dev_block_tables;
  bp.max_blocks = max_blocks_per_req;
  bp.old_ids = ids_buf;
  bp.new_ids = ids_buf + plan.total_old;
  bp.q_window = static_cast<const _Float16*>(dev_q_window);
  bp.lse_window = need_lse ? dev_lse_window : nullptr;
  bp.window = plan.window_hi;
  bp.n_sink = p->n_sink;
  bp.in_place = pv.in_place ? 1 : 0;
  const float sc = (scale > 0.f) ? scale : 1.0f / sqrtf((float)p->head_dim);
  bp.scale_log2e = sc * 1.44269504088896340736f;
  bp.raw_scores = p->raw_scores;
  bp.scores_out = dev_scores_out;
  bp.kept = kept_buf;
  bp.error_flag = p->error_flag;
  bp.owner = p->debug_checks ? p->owner : nullptr;
  bp.bounded = pruned_call ? 1 : 0;

  if (p->debug_checks) {
    // the table rows that the stage will release: every id in range, handed out, named once
    FC_HIP(launch_zero_ints(p->check_word, 1, stream));
    FC_HIP(launch_owner_check_tables(bp, p->check_word, false, stream));
    if (int vr = release_verdict(p, stream, "block tables of the compressed requests")) {
      (void)launch_owner_check_tables(bp, p->check_word, true, stream);
      return vr;
    }
  }

  // ---- the stage ------------------------------------------------------------
  int ns = 0, n_fused = 0;
  for (int c = 0; c < kPlanClasses; ++c) {
    ns += n_list[LIST_SNAP + c];
    n_fused += n_list[LIST_FUSED + c];
  }
  const int ring = p->prof_calls % kProfRing;
  if (p->profiling) {
    for (int k = 0; k < K_COUNT; ++k) p->timed[ring][k] = false;
    ++p->prof_calls;
  }
  auto run = [&](int slot, bool active, auto&& launch) -> hipError_t {
    if (!active) return hipSuccess;
    hipError_t e = hipSuccess;
    if (p->profiling) e = hipEventRecord(p->ev[ring][slot][0], stream);
    if (e == hipSuccess) e = launch();
    if (e == hipSuccess && p->profiling) {
      e = hipEventRecord(p->ev[ring][slot][1], stream);
      p->timed[ring][slot] = true;
    }
    return e;
  };
  FC_HIP_STAGE(p, run(K_PLAN_ALLOC, true, [&] { return launch_plan_alloc(bp, stream); }));
  FC_HIP_STAGE(p, run(K_SNAPKV_SCORE, ns > 0, [&] {
    hipError_t e = hipSuccess;
    for (int c = 1; c < kPlanClasses && e == hipSuccess; ++c) {
      if (n_list[LIST_SNAP + c] == 0) continue;
      BatchParams bc = bp;
      bc.order_snap = dev_list(LIST_SNAP + c);
      bc.n_snap = n_list[LIST_SNAP + c];
      bc.window = 16 * c;
      e = launch_snapkv_score(bc, stream);
    }
    return e;
  }));
  FC_HIP_STAGE(p, run(K_KNORM_SCORE, bp.n_knorm > 0, [&] { return launch_knorm_score(bp, stream); }));
  FC_HIP_STAGE(p, run(K_SELECT, bp.n_unfused > 0,
                      [&] { return launch_select(bp, plan.max_len[LIST_ALL], stream); }));
  FC_HIP_STAGE(p, run(K_GATHER, bp.n_unfused > 0, [&] { return launch_gather(bp, stream); }));
  FC_HIP_STAGE(p, run(K_FUSED, n_fused > 0, [&] {
    hipError_t e = hipSuccess;
    for (int c = 0; c < kPlanClasses && e == hipSuccess; ++c) {
      if (n_list[LIST_FUSED + c] == 0) continue;
      BatchParams bc = bp;
      bc.order_fused = dev_list(LIST_FUSED + c);
      bc.n_fused = n_list[LIST_FUSED + c];
      bc.window = 16 * c;
      e = launch_fused(bc, c > 0, plan.max_len[LIST_FUSED + c], stream);
    }
    return e;
  }));
  FC_HIP_STAGE(p, run(K_RECLAIM, true, [&] { return launch_reclaim(bp, stream); }));

  // ---- host mirrors ------------------------------------------------------------
  p->top = plan.top_after;
  for (const ReqDesc& d : plan.descs) host_seq_lens[d.table_row] = d.budget;
  return FC_OK;
}

}  // namespace

extern "C" {

int fc_compress_batch(fc_pool* p, int32_t* dev_block_tables, int max_blocks_per_req,
                      int32_t* host_seq_lens, const void* dev_q_window, int window,
                      const int32_t* host_method, const int32_t* host_budget, int n_req,
                      int pool_kernel, float scale, float* dev_scores_out, int32_t* dev_kept_out,
                      void* stream) {
  return compress_batch_impl(p, dev_block_tables, max_blocks_per_req, host_seq_lens, dev_q_window,
                             nullptr, false, nullptr, window, host_method, host_budget, n_req,
                             nullptr, pool_kernel, scale, dev_scores_out, dev_kept_out, stream,
                             false);
}

int fc_compress_batch_noalloc(fc_pool* p, int32_t* dev_block_tables, int max_blocks_per_req,
                              int32_t* host_seq_lens, const void* dev_q_window, int window,
                              const int32_t* host_method, const int32_t* host_budget, int n_req,
                              int pool_kernel, float scale, float* dev_scores_out,
                              int32_t* dev_kept_out, void* stream) {
  return compress_batch_impl(p, dev_block_tables, max_blocks_per_req, host_seq_lens, dev_q_window,
                             nullptr, false, nullptr, window, host_method, host_budget, n_req,
                             nullptr, pool_kernel, scale, dev_scores_out, dev_kept_out, stream,
                             true);
}

int fc_compress_batch_lse(fc_pool* p, int32_t* dev_block_tables, int max_blocks_per_req,
                          int32_t* host_seq_lens, const void* dev_q_window,
                          const float* dev_lse_window, int window, const int32_t* host_method,
                          const int32_t* host_budget, int n_req, int pool_kernel, float scale,
                          float* dev_scores_out, int32_t* dev_kept_out, void* stream) {
  return compress_batch_impl(p, dev_block_tables, max_blocks_per_req, host_seq_lens, dev_q_window,
                             dev_lse_window, true, nullptr, window, host_method, host_budget,
                             n_req, nullptr, pool_kernel, scale, dev_scores_out, dev_kept_out,
                             stream, false);
}

int fc_compress_batch_var(fc_pool* p, int32_t* dev_block_tables, int max_blocks_per_req,
                          int32_t* host_seq_lens, const void* dev_q_window,
                          const int32_t* host_window, const int32_t* host_method,
                          const int32_t* host_budget, const int32_t* host_pool_kernel, int n_req,
                          float scale, float* dev_scores_out, int32_t* dev_kept_out,
                          void* stream) {
  if (n_req > 0 && (!host_window || !host_pool_kernel)) return fail(FC_EINVAL, "NULL argument");
  return compress_batch_impl(p, dev_block_tables, max_blocks_per_req, host_seq_lens, dev_q_window,
                             nullptr, false, host_window, 0, host_method, host_budget, n_req,
                             host_pool_kernel, 0, scale, dev_scores_out, dev_kept_out, stream,
                             false);
}

int fc_window_lse(fc_pool* p, const int32_t* dev_block_tables, int max_blocks_per_req,
                  const int32_t* host_seq_lens, const void* dev_q_window, int window,
                  const int32_t* host_method, int n_req, float scale, float* dev_lse_out,
                  void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  FC_CHECK_POOL(p);
  if (n_req < 0) return fail(FC_EINVAL, "n_req < 0");
  if (n_req == 0) return FC_OK;
  if (!dev_block_tables || !host_seq_lens || !dev_q_window || !dev_lse_out)
    return fail(FC_EINVAL, "NULL argument");
  if (reinterpret_cast<uintptr_t>(dev_q_window) & 15)
    return fail(FC_EINVAL, "dev_q_window must be 16-byte aligned");
  if (reinterpret_cast<uintptr_t>(dev_lse_out) & 3)
    return fail(FC_EINVAL, "dev_lse_out must be 4-byte aligned");
  LsePlan plan;
  if (plan_window_lse(pool_view(p), n_req, max_blocks_per_req, host_seq_lens, host_method,
                      window, &plan) != PLAN_OK)
    return fail(plan.code, "%s", plan.message);
  if (plan.descs.empty()) return FC_OK;
  const int n = (int)plan.descs.size();
  const size_t desc_bytes = round_up((size_t)n * sizeof(ReqDesc), 16);
  const size_t meta_bytes = desc_bytes + round_up((size_t)n * sizeof(int32_t), 16);
  int rc;
  if ((rc = grow_meta(p, meta_bytes)) != FC_OK) return rc;
  std::vector<char> image(meta_bytes, 0);
  memcpy(image.data(), plan.descs.data(), (size_t)n * sizeof(ReqDesc));
  int32_t* order = reinterpret_cast<int32_t*>(image.data() + desc_bytes);
  for (int i = 0; i < n; ++i) order[i] = i;
  if ((rc = upload_meta(p, image.data(), meta_bytes, p->dev_meta, false, stream)) != FC_OK) return rc;

  BatchParams bp = {};
  bp.kv = p->kv;
  bp.n_blocks = p->n_blocks;
  bp.n_layers = p->n_layers;
  bp.n_heads = p->n_heads;
  bp.head_dim = p->head_dim;
  bp.descs = reinterpret_cast<const ReqDesc*>(p->dev_meta);
  bp.order_snap = reinterpret_cast<const int32_t*>(p->dev_meta + desc_bytes);
  bp.n_snap = n;
  bp.block_tables = const_cast<int32_t*>(dev_block_tables);  // read only on this path
  bp.max_blocks = max_blocks_per_req;
  bp.q_window = static_cast<const _Float16*>(dev_q_window);
  bp.lse_out = dev_lse_out;
  bp.window = window;
  const float sc = (scale > 0.f) ? scale : 1.0f / sqrtf((float)p->head_dim);
  bp.scale_log2e = sc * 1.44269504088896340736f;
  const int ring = p->prof_calls % kProfRing;
  if (p->profiling) {
    for (int k = 0; k < K_COUNT; ++k) p->timed[ring][k] = false;
    ++p->prof_calls;
    FC_HIP(hipEventRecord(p->ev[ring][K_WINDOW_LSE][0], stream));
  }
  FC_HIP(launch_snapkv_score(bp, stream));
  if (p->profiling) {
    FC_HIP(hipEventRecord(p->ev[ring][K_WINDOW_LSE][1], stream));
    p->timed[ring][K_WINDOW_LSE] = true;
  }
  return FC_OK;
}

int fc_mlp_set_weights(fc_pool* p, const fc_mlp_weights* w, void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if (!p || !w) return fail(FC_EINVAL, "NULL argument");
  if (w->k < 1 || w->k > 8) return fail(FC_EINVAL, "k must be in 1..8");
  if (w->hidden != 128 && w->hidden != 256) return fail(FC_EINVAL, "hidden must be 128 or 256");
  if (w->activation != FC_ACT_GELU_ERF && w->activation != FC_ACT_GELU_TANH)
    return fail(FC_EINVAL, "unknown activation %d", w->activation);
  for (int m = 0; m < 2; ++m)
    if (!w->w1[m] || !w->b1[m] || !w->w2[m] || !w->b2[m])
      return fail(FC_EINVAL, "NULL weight pointer");
  FC_HIP(hipDeviceSynchronize());  // earlier calls may still read the old copies
  const size_t n1 = mlp_w1p_elems(p->head_dim, w->hidden, w->k);
  const size_t n2 = mlp_w2p_elems(p->head_dim, w->hidden);
  for (int m = 0; m < 2; ++m) {
    if (p->mlp_w1p[m]) FC_HIP(hipFree(p->mlp_w1p[m]));  // w2p lies in the same allocation
    if (p->mlp_b1[m]) FC_HIP(hipFree(p->mlp_b1[m]));
    if (p->mlp_b2[m]) FC_HIP(hipFree(p->mlp_b2[m]));
    p->mlp_w1p[m] = p->mlp_w2p[m] = nullptr;
    p->mlp_b1[m] = p->mlp_b2[m] = nullptr;
  }
  p->mlp_k = p->mlp_hidden = 0;
  for (int m = 0; m < 2; ++m) {
    // one allocation: the kernel streams W1 and then W2 through the same ring
    FC_HIP(hipMalloc(reinterpret_cast<void**>(&p->mlp_w1p[m]), (n1 + n2) * sizeof(_Float16)));
    p->mlp_w2p[m] = p->mlp_w1p[m] + n1;
    FC_HIP(hipMalloc(reinterpret_cast<void**>(&p->mlp_b1[m]), (size_t)w->hidden * sizeof(float)));
    FC_HIP(hipMalloc(reinterpret_cast<void**>(&p->mlp_b2[m]), (size_t)p->head_dim * sizeof(float)));
    FC_HIP(launch_mlp_permute_weights(static_cast<const _Float16*>(w->w1[m]),
                                      static_cast<const _Float16*>(w->w2[m]), p->mlp_w1p[m],
                                      p->mlp_w2p[m], p->head_dim, w->hidden, w->k, stream));
    FC_HIP(hipMemcpyAsync(p->mlp_b1[m], w->b1[m], (size_t)w->hidden * sizeof(float),
                          hipMemcpyDeviceToDevice, stream));
    FC_HIP(hipMemcpyAsync(p->mlp_b2[m], w->b2[m], (size_t)p->head_dim * sizeof(float),
                          hipMemcpyDeviceToDevice, stream));
  }
  p->mlp_k = w->k;
  p->mlp_hidden = w->hidden;
  p->mlp_activation = w->activation;
  return FC_OK;
}

int fc_compress_batch_mlp(fc_pool* p, int32_t* dev_block_tables, int max_blocks_per_req,
                          int32_t* host_seq_lens, const int32_t* host_img_begin,
                          const int32_t* host_img_end, const int32_t* host_enable, int n_req,
                          void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  FC_CHECK_POOL(p);
  if (p->mlp_k == 0) return fail(FC_EINVAL, "fc_mlp_set_weights has not been called");
  if (n_req > 0 && !dev_block_tables) return fail(FC_EINVAL, "NULL argument");
  MlpPlan plan;
  if (plan_mlp(pool_view(p), n_req, max_blocks_per_req, host_seq_lens, host_img_begin,
               host_img_end, host_enable, p->mlp_k, mlp_rows_per_tile(p->mlp_hidden),
               &plan) != PLAN_OK)
    return fail(plan.code, "%s", plan.message);
  const int n_comp = (int)plan.descs.size();
  if (n_comp == 0) return FC_OK;

  int rc;
  if ((rc = grow(&p->ids, &p->ids_cap, (size_t)plan.total_old + plan.total_new)) != FC_OK) return rc;
  const size_t desc_bytes = round_up((size_t)n_comp * sizeof(ReqDesc), 16);
  const size_t job_bytes = round_up(plan.jobs.size() * sizeof(MlpJob), 16);
  if ((rc = grow_meta(p, desc_bytes + job_bytes)) != FC_OK) return rc;
  std::vector<char> image(desc_bytes + job_bytes, 0);
  memcpy(image.data(), plan.descs.data(), (size_t)n_comp * sizeof(ReqDesc));
  memcpy(image.data() + desc_bytes, plan.jobs.data(), plan.jobs.size() * sizeof(MlpJob));
  if ((rc = upload_meta(p, image.data(), image.size(), p->dev_meta, false, stream)) != FC_OK)
    return rc;

  BatchParams bp = {};
  bp.kv = p->kv;
  bp.n_blocks = p->n_blocks;
  bp.n_layers = p->n_layers;
  bp.n_heads = p->n_heads;
  bp.head_dim = p->head_dim;
  bp.stack = p->stack;
  bp.top_before = p->top;
  bp.total_new = plan.total_new;
  bp.total_old = plan.total_old;
  bp.descs = reinterpret_cast<const ReqDesc*>(p->dev_meta);
  bp.n_comp = n_comp;
  bp.block_tables = dev_block_tables;
  bp.max_blocks = max_blocks_per_req;
  bp.old_ids = p->ids;
  bp.new_ids = p->ids + plan.total_old;
  bp.error_flag = p->error_flag;
  bp.owner = p->debug_checks ? p->owner : nullptr;
  MlpParams mp = {};
  mp.jobs = reinterpret_cast<const MlpJob*>(p->dev_meta + desc_bytes);
  mp.n_jobs = (int)plan.jobs.size();
  mp.n_tiles = (int)plan.n_tiles;
  {
    int dev = 0, cus = 0;
    FC_HIP(hipGetDevice(&dev));
    FC_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    mp.max_grid = std::max(cus, 1) * mlp_workgroups_per_cu();
  }
  mp.k = p->mlp_k;
  mp.hidden = p->mlp_hidden;
  mp.activation = p->mlp_activation;
  for (int m = 0; m < 2; ++m) {
    mp.w1p[m] = p->mlp_w1p[m];
    mp.w2p[m] = p->mlp_w2p[m];
    mp.b1[m] = p->mlp_b1[m];
    mp.b2[m] = p->mlp_b2[m];
  }

  if (p->debug_checks) {
    FC_HIP(launch_zero_ints(p->check_word, 1, stream));
    FC_HIP(launch_owner_check_tables(bp, p->check_word, false, stream));
    if (int vr = release_verdict(p, stream, "block tables of the compressed requests")) {
      (void)launch_owner_check_tables(bp, p->check_word, true, stream);
      return vr;
    }
  }
  const int ring = p->prof_calls % kProfRing;
  if (p->profiling) {
    for (int kk = 0; kk < K_COUNT; ++kk) p->timed[ring][kk] = false;
    ++p->prof_calls;
  }
  auto run = [&](int slot, auto&& launch) -> hipError_t {
    hipError_t e = hipSuccess;
    if (p->profiling) e = hipEventRecord(p->ev[ring][slot][0], stream);
    if (e == hipSuccess) e = launch();
    if (e == hipSuccess && p->profiling) {
      e = hipEventRecord(p->ev[ring][slot][1], stream);
      p->timed[ring][slot] = true;
    }
    return e;
  };
  FC_HIP_STAGE(p, run(K_PLAN_ALLOC, [&] { return launch_plan_alloc(bp, stream); }));
  FC_HIP_STAGE(p, run(K_MLP, [&] { return launch_mlp_compress(bp, mp, stream); }));
  FC_HIP_STAGE(p, run(K_RECLAIM, [&] { return launch_reclaim(bp, stream); }));

  p->top = plan.top_after;
  for (const ReqDesc& d : plan.descs) host_seq_lens[d.table_row] = d.budget;
  return FC_OK;
}

}  // extern "C"

namespace {

// One profiled launch outside fc_compress_batch (same event ring).
template <typename F>
hipError_t run_profiled(fc_pool* p, int slot, hipStream_t stream, F&& launch) {
  const int ring = p->prof_calls % kProfRing;
  if (p->profiling) {
    for (int k = 0; k < K_COUNT; ++k) p->timed[ring][k] = false;
    ++p->prof_calls;
  }
  hipError_t e = hipSuccess;
  if (p->profiling) e = hipEventRecord(p->ev[ring][slot][0], stream);
  if (e == hipSuccess) e = launch();
  if (e == hipSuccess && p->profiling) {
    e = hipEventRecord(p->ev[ring][slot][1], stream);
    p->timed[ring][slot] = true;
  }
  return e;
}

// descriptors of a decode step to the device through the pinned staging buffer
int upload_decode_reqs(fc_pool* p, const std::vector<DecodeReq>& reqs, hipStream_t stream) {
  const size_t bytes = round_up(reqs.size() * sizeof(DecodeReq), 16);
  int rc;
  if ((rc = grow_meta(p, bytes)) != FC_OK) return rc;
  std::vector<char> image(bytes, 0);
  memcpy(image.data(), reqs.data(), reqs.size() * sizeof(DecodeReq));
  return upload_meta(p, image.data(), bytes, p->dev_meta, false, stream);
}

DecodeParams decode_params(fc_pool* p) {
  DecodeParams dp = {};
  dp.kv = p->kv;
  dp.n_blocks = p->n_blocks;
  dp.n_layers = p->n_layers;
  dp.n_heads = p->n_heads;
  dp.head_dim = p->head_dim;
  dp.stack = p->stack;
  dp.top_before = p->top;
  dp.reqs = reinterpret_cast<const DecodeReq*>(p->dev_meta);
  dp.owner = p->debug_checks ? p->owner : nullptr;
  dp.error_flag = p->error_flag;
  return dp;
}

int decode_attention_impl(fc_pool* p, const int32_t* dev_block_tables, int max_blocks_per_req,
                          const int32_t* host_seq_lens, const int32_t* host_budget,
                          const int32_t* dev_kept, const void* dev_q, float* dev_out, int n_req,
                          float scale, void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  FC_CHECK_POOL(p);
  if (n_req < 0) return fail(FC_EINVAL, "n_req < 0");
  if (n_req == 0) return FC_OK;
  if (!dev_block_tables || !host_seq_lens || !dev_q || !dev_out)
    return fail(FC_EINVAL, "NULL argument");
  if (reinterpret_cast<uintptr_t>(dev_q) & 15) return fail(FC_EINVAL, "dev_q must be 16-byte aligned");
  DecodePlan plan;
  if (plan_decode_attention(pool_view(p), n_req, max_blocks_per_req, host_seq_lens,
                            dev_kept ? host_budget : nullptr, &plan) != PLAN_OK)
    return fail(plan.code, "%s", plan.message);
  int rc;
  if ((rc = upload_decode_reqs(p, plan.reqs, stream)) != FC_OK) return rc;
  DecodeParams dp = decode_params(p);
  dp.block_tables = const_cast<int32_t*>(dev_block_tables);
  dp.max_blocks = max_blocks_per_req;
  dp.n_req = n_req;
  dp.q = static_cast<const _Float16*>(dev_q);
  dp.out = dev_out;
  dp.kept = dev_kept;
  const float sc = (scale > 0.f) ? scale : 1.0f / sqrtf((float)p->head_dim);
  dp.scale_log2e = sc * 1.44269504088896340736f;
  FC_HIP(run_profiled(p, K_DECODE_ATTENTION, stream,
                      [&] { return launch_decode_attention(dp, stream); }));
  return FC_OK;
}

}  // namespace

extern "C" {

int fc_append_batch(fc_pool* p, int32_t* dev_block_tables, int max_blocks_per_req,
                    int32_t* host_seq_lens, const void* dev_new_kv, const int32_t* host_enable,
                    int n_req, void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  FC_CHECK_POOL(p);
  if (n_req < 0) return fail(FC_EINVAL, "n_req < 0");
  if (n_req == 0) return FC_OK;
  if (!dev_block_tables || !host_seq_lens || !dev_new_kv) return fail(FC_EINVAL, "NULL argument");
  if (reinterpret_cast<uintptr_t>(dev_new_kv) & 15)
    return fail(FC_EINVAL, "dev_new_kv must be 16-byte aligned");
  DecodePlan plan;
  if (plan_append(pool_view(p), n_req, max_blocks_per_req, host_seq_lens, host_enable,
                  &plan) != PLAN_OK)
    return fail(plan.code, "%s", plan.message);
  if (plan.reqs.empty()) return FC_OK;
  int rc;
  if ((rc = upload_decode_reqs(p, plan.reqs, stream)) != FC_OK) return rc;
  DecodeParams dp = decode_params(p);
  dp.block_tables = dev_block_tables;
  dp.max_blocks = max_blocks_per_req;
  dp.n_req = (int)plan.reqs.size();
  dp.new_kv = static_cast<const _Float16*>(dev_new_kv);
  FC_HIP_STAGE(p, run_profiled(p, K_APPEND, stream, [&] { return launch_append(dp, stream); }));
  p->top -= plan.n_pop;
  for (const DecodeReq& q : plan.reqs) host_seq_lens[q.table_row] = q.seq_len + 1;
  return FC_OK;
}

int fc_decode_attention(fc_pool* p, const int32_t* dev_block_tables, int max_blocks_per_req,
                        const int32_t* host_seq_lens, const void* dev_q, float* dev_out, int n_req,
                        float scale, void* stream) {
  return decode_attention_impl(p, dev_block_tables, max_blocks_per_req, host_seq_lens, nullptr,
                               nullptr, dev_q, dev_out, n_req, scale, stream);
}

int fc_decode_attention_kept(fc_pool* p, const int32_t* dev_block_tables, int max_blocks_per_req,
                             const int32_t* host_seq_lens, const int32_t* host_budget,
                             const int32_t* dev_kept, const void* dev_q, float* dev_out, int n_req,
                             float scale, void* stream) {
  if (n_req > 0 && (!host_budget || !dev_kept)) return fail(FC_EINVAL, "NULL argument");
  return decode_attention_impl(p, dev_block_tables, max_blocks_per_req, host_seq_lens, host_budget,
                               dev_kept, dev_q, dev_out, n_req, scale, stream);
}

}  // extern "C"
