// Host-side planning of libfastcache's batched calls (see fc_plan.h).
//
// The batch compression step of FastCache's serving loop (Algorithm 1) is
// issued once for the whole batch; what the host scheduler knows about the
// batch (lengths, methods, budgets, free blocks: "Memory-Aware Scheduling"
// paragraph) is enough to validate it, to detect that the pool cannot take
// it, and to lay out every request's share of the stage's buffers before any
// device work is queued.

#include "fc_plan.h"

#include <stdarg.h>
#include <stdio.h>

#include <algorithm>
#include <numeric>

namespace fc {

namespace {

int blocks_for(int tokens) { return (tokens + kPlanBlockSize - 1) / kPlanBlockSize; }

template <typename Plan>
int fail(Plan* plan, int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(plan->message, sizeof(plan->message), fmt, ap);
  va_end(ap);
  plan->code = code;
  return code;
}

}  // namespace

int plan_compress(const PoolView& pool, const CompressArgs& a, CompressPlan* plan) {
  *plan = CompressPlan();
  plan->top_after = pool.n_free;
  if (a.n_req < 0) return fail(plan, PLAN_EINVAL, "n_req < 0");
  if (a.n_req == 0) return PLAN_OK;
  if (!a.seq_lens || !a.method || !a.budget) return fail(plan, PLAN_EINVAL, "NULL argument");
  if (a.max_blocks < 1) return fail(plan, PLAN_EINVAL, "max_blocks_per_req < 1");
  const bool per_request = a.window_per_req != nullptr;
  if (per_request && !a.pool_kernel_per_req) return fail(plan, PLAN_EINVAL, "NULL argument");
  if (!per_request &&
      (a.pool_kernel < 1 || a.pool_kernel > kPlanMaxPoolKernel || (a.pool_kernel & 1) == 0))
    return fail(plan, PLAN_EINVAL, "pool_kernel must be odd and in 1..%d", kPlanMaxPoolKernel);

  // ---- validate; lay out every request's share of the buffers ---------------
  const size_t n_lh = (size_t)pool.n_layers * pool.n_heads;
  std::vector<ReqDesc>& descs = plan->descs;
  descs.reserve(a.n_req);
  long long total_new = 0, total_old = 0, total_released = 0;
  size_t score_off = 0, kept_off = 0, q_off = 0;
  for (int r = 0; r < a.n_req; ++r) {
    const int m = a.method[r];
    // queries are packed: with per-request windows only SnapKV requests have any
    const size_t q_here = q_off;
    if (per_request) {
      if (m == PLAN_METHOD_SNAPKV)
        q_off += n_lh * (size_t)std::max(a.window_per_req[r], 0) * pool.head_dim;
    } else {
      q_off += n_lh * (size_t)std::max(a.window, 0) * pool.head_dim;
    }
    if (m == PLAN_METHOD_NONE) continue;
    const int L = a.seq_lens[r], B = a.budget[r];
    const int win = per_request ? a.window_per_req[r] : a.window;
    const int pk = per_request ? a.pool_kernel_per_req[r] : a.pool_kernel;
    if (m != PLAN_METHOD_SNAPKV && m != PLAN_METHOD_KNORM && m != PLAN_METHOD_STREAMING)
      return fail(plan, PLAN_EINVAL, "request %d: unknown method %d", r, m);
    if (L < 1 || L > kPlanMaxSeqLen)
      return fail(plan, PLAN_EINVAL, "request %d: length %d outside 1..%d", r, L, kPlanMaxSeqLen);
    if (B < 1 || B > L)
      return fail(plan, PLAN_EINVAL, "request %d: budget %d outside 1..%d", r, B, L);
    if (m == PLAN_METHOD_SNAPKV) {
      if (win < 1 || win > kPlanMaxWindow)
        return fail(plan, PLAN_EINVAL, "request %d: window %d outside 1..%d", r, win,
                    kPlanMaxWindow);
      if (pk < 1 || pk > kPlanMaxPoolKernel || (pk & 1) == 0)
        return fail(plan, PLAN_EINVAL, "request %d: pool_kernel must be odd and in 1..%d", r,
                    kPlanMaxPoolKernel);
      if (L < win || B < win)
        return fail(plan, PLAN_EINVAL, "request %d: SnapKV needs length and budget >= window", r);
      if (!a.q_ok)
        return fail(plan, PLAN_EINVAL, "dev_q_window must be a 16-byte aligned device pointer");
      if (a.need_lse && !a.lse_ok)
        return fail(plan, PLAN_EINVAL, "dev_lse_window must be a 4-byte aligned device pointer");
      plan->window_hi = std::max(plan->window_hi, win);
    }
    ReqDesc d = {};
    d.window = m == PLAN_METHOD_SNAPKV ? win : 0;
    d.pool_kernel = m == PLAN_METHOD_SNAPKV ? pk : 1;
    d.seq_len = L;
    d.budget = B;
    d.method = m;
    d.table_row = r;
    d.n_old = blocks_for(L);
    d.n_new = blocks_for(B);
    if (d.n_old > a.max_blocks)
      return fail(plan, PLAN_EINVAL, "request %d: %d blocks exceed max_blocks_per_req %d", r,
                  d.n_old, a.max_blocks);
    d.old_off = (int32_t)total_old;
    d.new_off = (int32_t)(pool.in_place ? total_released : total_new);
    d.score_off = (int64_t)score_off;
    d.raw_off = 0;
    d.kept_off = (int64_t)kept_off;
    d.q_off = (int64_t)q_here;
    total_old += d.n_old;
    total_new += pool.in_place ? 0 : d.n_new;
    total_released += d.n_old - d.n_new;
    score_off += n_lh * (size_t)L;
    kept_off += n_lh * (size_t)B;
    descs.push_back(d);
  }
  const int n_comp = (int)descs.size();
  if (n_comp == 0) return PLAN_OK;
  if (total_old > 0x7fffffffLL || total_new > 0x7fffffffLL)
    return fail(plan, PLAN_EINVAL, "batch too large");
  if (total_new > pool.n_free)
    return fail(plan, PLAN_ENOMEM, "batch needs %lld new blocks, %d free", total_new, pool.n_free);
  plan->total_new = (int)total_new;
  plan->total_old = (int)total_old;
  plan->total_released = (int)total_released;
  plan->kept_entries = kept_off;
  plan->score_entries = score_off;
  plan->top_after = pool.in_place ? pool.n_free + (int)total_released
                                  : pool.n_free - (int)total_new + (int)total_old;

  // ---- work lists ------------------------------------------------------------------
  // Descriptor indices, heaviest first so that the tail of each launch is made
  // of light units.  Heads short enough for the fused kernel (score -> select ->
  // gather in one workgroup) are listed per window class (class c: SnapKV with
  // ceil(window/16) == c, the number of 16-row query tiles the kernel is
  // compiled for; class 0: no queries at all); the rest go through the
  // separate kernels: SnapKV per class, key-norm, and one list of all of them
  // for select and gather.
  std::vector<int> sorted(n_comp);
  std::iota(sorted.begin(), sorted.end(), 0);
  // bytes a unit moves (K once or twice, kept K/V read and written)
  auto weight = [&](int i) {
    const ReqDesc& d = descs[i];
    const int passes = d.method == PLAN_METHOD_SNAPKV ? (a.need_lse ? 1 : 2)
                                                      : d.method == PLAN_METHOD_KNORM ? 1 : 0;
    return (int64_t)d.seq_len * passes + (int64_t)d.budget * 4;
  };
  std::stable_sort(sorted.begin(), sorted.end(),
                   [&](int x, int y) { return weight(x) > weight(y); });
  const bool allow_fused = pool.score_mode == PLAN_SCORE_AUTO;
  auto fused = [&](int i) {
    const ReqDesc& d = descs[i];
    // (streaming: no score, no LDS, so the fused kernel whatever the length)
    return d.method == PLAN_METHOD_STREAMING ||
           (allow_fused && d.seq_len <= kPlanFusedMaxLen);
  };
  // Units without queries (key-norm, streaming) ride in the launch of the
  // SnapKV class that has the most fused units, if there is one: one launch
  // fills the chip better than two that each end in a tail.
  int home_class = 0;
  {
    int count[kPlanClasses] = {};
    for (int i = 0; i < n_comp; ++i)
      if (descs[i].method == PLAN_METHOD_SNAPKV && fused(i)) ++count[(descs[i].window + 15) / 16];
    for (int c = 1; c < kPlanClasses; ++c)
      if (count[c] > count[home_class]) home_class = c;
  }
  size_t raw_need = 0;
  for (int di : sorted) {
    ReqDesc& d = descs[di];
    const bool snap = d.method == PLAN_METHOD_SNAPKV;
    const int cls = snap ? (d.window + 15) / 16 : 0;
    int li;
    if (fused(di)) {
      li = LIST_FUSED + (snap ? cls : home_class);
    } else {
      // scores of these units travel through the library's scratch
      d.raw_off = (int64_t)raw_need;
      raw_need += n_lh * (size_t)d.seq_len;
      li = snap ? LIST_SNAP + cls : LIST_KNORM;
      plan->lists[LIST_ALL].push_back(di);
      plan->max_len[LIST_ALL] = std::max(plan->max_len[LIST_ALL], d.seq_len);
    }
    plan->lists[li].push_back(di);
    // (sizes the score buffer in LDS, which streaming units do not use)
    if (d.method != PLAN_METHOD_STREAMING) plan->max_len[li] = std::max(plan->max_len[li], d.seq_len);
  }
  plan->raw_floats = raw_need;
  return PLAN_OK;
}

int plan_window_lse(const PoolView& pool, int n_req, int max_blocks, const int32_t* seq_lens,
                    const int32_t* method, int window, LsePlan* plan) {
  *plan = LsePlan();
  if (n_req < 0) return fail(plan, PLAN_EINVAL, "n_req < 0");
  if (n_req == 0) return PLAN_OK;
  if (!seq_lens) return fail(plan, PLAN_EINVAL, "NULL argument");
  if (max_blocks < 1) return fail(plan, PLAN_EINVAL, "max_blocks_per_req < 1");
  if (window < 1 || window > kPlanMaxWindow)
    return fail(plan, PLAN_EINVAL, "window %d outside 1..%d", window, kPlanMaxWindow);
  const size_t n_lh = (size_t)pool.n_layers * pool.n_heads;
  for (int r = 0; r < n_req; ++r) {
    if (method && method[r] != PLAN_METHOD_SNAPKV) continue;
    const int L = seq_lens[r];
    if (L < window || L > kPlanMaxSeqLen)
      return fail(plan, PLAN_EINVAL, "request %d: length %d outside %d..%d", r, L, window,
                  kPlanMaxSeqLen);
    ReqDesc d = {};
    d.window = window;
    d.pool_kernel = 1;
    d.seq_len = L;
    d.budget = L;
    d.method = PLAN_METHOD_SNAPKV;
    d.table_row = r;
    d.n_old = blocks_for(L);
    if (d.n_old > max_blocks)
      return fail(plan, PLAN_EINVAL, "request %d: %d blocks exceed max_blocks_per_req %d", r,
                  d.n_old, max_blocks);
    d.q_off = (int64_t)((size_t)r * n_lh * window * pool.head_dim);
    plan->descs.push_back(d);
  }
  // longest first, so that the tail of the launch is made of short units
  std::stable_sort(plan->descs.begin(), plan->descs.end(),
                   [](const ReqDesc& x, const ReqDesc& y) { return x.seq_len > y.seq_len; });
  return PLAN_OK;
}

int plan_mlp(const PoolView& pool, int n_req, int max_blocks, const int32_t* seq_lens,
             const int32_t* img_begin, const int32_t* img_end, const int32_t* enable, int k,
             int tile_rows, MlpPlan* plan) {
  *plan = MlpPlan();
  plan->top_after = pool.n_free;
  if (n_req < 0) return fail(plan, PLAN_EINVAL, "n_req < 0");
  if (n_req == 0) return PLAN_OK;
  if (!seq_lens || !img_begin || !img_end) return fail(plan, PLAN_EINVAL, "NULL argument");
  if (max_blocks < 1) return fail(plan, PLAN_EINVAL, "max_blocks_per_req < 1");
  if (k < 1 || tile_rows < 1) return fail(plan, PLAN_EINVAL, "bad chunk size or tile size");
  const long long n_units = (long long)pool.n_layers * pool.n_heads * 2;
  long long total_new = 0, total_old = 0;
  for (int r = 0; r < n_req; ++r) {
    if (enable && !enable[r]) continue;
    const int L = seq_lens[r], ib = img_begin[r], ie = img_end[r];
    if (L < 1 || L > kPlanMaxSeqLen)
      return fail(plan, PLAN_EINVAL, "request %d: length %d outside 1..%d", r, L, kPlanMaxSeqLen);
    if (ib < 0 || ib > ie || ie > L)
      return fail(plan, PLAN_EINVAL, "request %d: image span [%d, %d) outside [0, %d]", r, ib, ie,
                  L);
    ReqDesc d = {};
    d.seq_len = L;
    d.img_begin = ib;
    d.img_end = ie;
    d.chunks_text0 = (ib + k - 1) / k;
    d.chunks_image = (ie - ib + k - 1) / k;
    d.chunks_text1 = (L - ie + k - 1) / k;
    d.budget = d.chunks_text0 + d.chunks_image + d.chunks_text1;
    d.method = PLAN_METHOD_NONE;
    d.table_row = r;
    d.n_old = blocks_for(L);
    d.n_new = blocks_for(d.budget);
    if (d.n_old > max_blocks)
      return fail(plan, PLAN_EINVAL, "request %d: %d blocks exceed max_blocks_per_req %d", r,
                  d.n_old, max_blocks);
    d.old_off = (int32_t)total_old;
    d.new_off = (int32_t)total_new;
    total_old += d.n_old;
    total_new += d.n_new;
    const int di = (int)plan->descs.size();
    const int per_modality[2] = {d.chunks_text0 + d.chunks_text1, d.chunks_image};
    for (int m = 0; m < 2; ++m) {
      if (per_modality[m] == 0) continue;
      MlpJob j;
      j.desc = di;
      j.modality = m;
      j.chunks = per_modality[m];
      j.tile_start = (int)plan->n_tiles;
      plan->n_tiles += (n_units * per_modality[m] + tile_rows - 1) / tile_rows;
      if (plan->n_tiles > 0x7fffffffLL)
        return fail(plan, PLAN_EINVAL, "batch too large for one launch");
      plan->jobs.push_back(j);
    }
    plan->descs.push_back(d);
  }
  if (plan->descs.empty()) return PLAN_OK;
  if (total_old > 0x7fffffffLL) return fail(plan, PLAN_EINVAL, "batch too large");
  if (total_new > pool.n_free)
    return fail(plan, PLAN_ENOMEM, "batch needs %lld new blocks, %d free", total_new, pool.n_free);
  plan->total_new = (int)total_new;
  plan->total_old = (int)total_old;
  plan->top_after = pool.n_free - (int)total_new + (int)total_old;
  return PLAN_OK;
}

int plan_append(const PoolView& pool, int n_req, int max_blocks, const int32_t* seq_lens,
                const int32_t* enable, DecodePlan* plan) {
  *plan = DecodePlan();
  if (n_req < 0) return fail(plan, PLAN_EINVAL, "n_req < 0");
  if (n_req == 0) return PLAN_OK;
  if (!seq_lens) return fail(plan, PLAN_EINVAL, "NULL argument");
  if (max_blocks < 1) return fail(plan, PLAN_EINVAL, "max_blocks_per_req < 1");
  for (int r = 0; r < n_req; ++r) {
    if (enable && !enable[r]) continue;
    const int L = seq_lens[r];
    if (L < 0 || L >= kPlanMaxSeqLen)
      return fail(plan, PLAN_EINVAL, "request %d: length %d outside 0..%d", r, L,
                  kPlanMaxSeqLen - 1);
    if (L / kPlanBlockSize >= max_blocks)
      return fail(plan, PLAN_EINVAL, "request %d: its table row is full", r);
    DecodeReq q = {r, L, (L % kPlanBlockSize == 0) ? plan->n_pop++ : -1, 0, 0};
    plan->reqs.push_back(q);
  }
  if (plan->n_pop > pool.n_free)
    return fail(plan, PLAN_ENOMEM, "append needs %d new blocks, %d free", plan->n_pop,
                pool.n_free);
  return PLAN_OK;
}

int plan_decode_attention(const PoolView& pool, int n_req, int max_blocks, const int32_t* seq_lens,
                          const int32_t* budget, DecodePlan* plan) {
  *plan = DecodePlan();
  if (n_req < 0) return fail(plan, PLAN_EINVAL, "n_req < 0");
  if (n_req == 0) return PLAN_OK;
  if (!seq_lens) return fail(plan, PLAN_EINVAL, "NULL argument");
  if (max_blocks < 1) return fail(plan, PLAN_EINVAL, "max_blocks_per_req < 1");
  const size_t n_lh = (size_t)pool.n_layers * pool.n_heads;
  plan->reqs.resize(n_req);
  for (int r = 0; r < n_req; ++r) {
    const int L = seq_lens[r];
    if (L < 0 || L > kPlanMaxSeqLen)
      return fail(plan, PLAN_EINVAL, "request %d: length %d outside 0..%d", r, L, kPlanMaxSeqLen);
    if (blocks_for(L) > max_blocks)
      return fail(plan, PLAN_EINVAL, "request %d: %d tokens exceed max_blocks_per_req", r, L);
    DecodeReq q = {r, L, -1, 0, 0};
    if (budget) {
      const int B = budget[r];
      if (B < 0 || B > L)
        return fail(plan, PLAN_EINVAL, "request %d: budget %d outside 0..%d", r, B, L);
      q.pop_index = B;
      q.kept_off = (int64_t)plan->kept_entries;
      plan->kept_entries += n_lh * (size_t)B;
    }
    plan->reqs[r] = q;
  }
  // longest first, so that the tail of the launch is made of short units
  std::stable_sort(plan->reqs.begin(), plan->reqs.end(),
                   [&](const DecodeReq& x, const DecodeReq& y) {
                     return budget ? x.pop_index > y.pop_index : x.seq_len > y.seq_len;
                   });
  return PLAN_OK;
}

}  // namespace fc
