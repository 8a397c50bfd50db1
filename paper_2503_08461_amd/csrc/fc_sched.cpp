// Host-side scheduler of the compress queue (Algorithm 1: requests are
// accumulated; when at least B_min are pending or the wait time is exceeded,
// FormBatch(Q, B_max) builds a batch; "Memory-Aware Scheduling": all pending
// requests are examined and the largest batch that fits the free memory is
// built; AdjustBatch adapts the batch size to runtime conditions).  No device
// code: the caller passes the pool's free block count (fc_pool_num_free) and
// hands the returned batch to fc_compress_batch.  All times are integer
// microseconds so that decisions are reproducible bit for bit.

#include "../../include/fastcache.h"

#include <algorithm>
#include <cstdint>
#include <vector>

namespace {

struct Pending {
  int64_t arrival_us;
  int64_t id;
  int32_t seq_len;
  int32_t budget;
  int32_t need() const { return (budget + FC_BLOCK_SIZE - 1) / FC_BLOCK_SIZE; }
};

// floor(a / 4) for either sign
int64_t floor_div4(int64_t a) { return a >= 0 ? a / 4 : -((-a + 3) / 4); }

// running average: the first sample sets it, then avg += floor((x - avg) / 4)
int64_t running_avg(int64_t avg, int64_t x) { return avg == 0 ? x : avg + floor_div4(x - avg); }

}  // namespace

struct fc_sched {
  int b_min, b_max, b_target;
  int64_t max_wait_us;
  int64_t gap_avg = 0, svc_avg = 0;  // 0: no sample yet
  bool any_arrival = false;
  int64_t last_arrival = 0;
  std::vector<Pending> pending;  // arrival order
};

extern "C" {

int fc_sched_create(fc_sched** out, int b_min, int b_max, int64_t max_wait_us) {
  if (!out || b_min < 1 || b_max < b_min || max_wait_us < 0) return FC_EINVAL;
  fc_sched* s = new (std::nothrow) fc_sched;
  if (!s) return FC_ENOMEM;
  s->b_min = s->b_target = b_min;
  s->b_max = b_max;
  s->max_wait_us = max_wait_us;
  *out = s;
  return FC_OK;
}

void fc_sched_destroy(fc_sched* s) { delete s; }

int fc_sched_submit(fc_sched* s, int64_t req_id, int64_t arrival_us, int seq_len, int budget) {
  if (!s) return FC_EINVAL;
  if (s->any_arrival && arrival_us < s->last_arrival) return FC_EINVAL;
  if (budget < 1 || budget > seq_len) return FC_EINVAL;
  for (const Pending& p : s->pending)
    if (p.id == req_id) return FC_EINVAL;
  if (s->any_arrival) s->gap_avg = running_avg(s->gap_avg, arrival_us - s->last_arrival);
  s->any_arrival = true;
  s->last_arrival = arrival_us;
  s->pending.push_back({arrival_us, req_id, seq_len, budget});
  return FC_OK;
}

int fc_sched_pending(const fc_sched* s) { return s ? (int)s->pending.size() : FC_EINVAL; }

int fc_sched_batch_target(const fc_sched* s) { return s ? s->b_target : FC_EINVAL; }

int fc_sched_ready(const fc_sched* s, int64_t now_us) {
  if (!s) return FC_EINVAL;
  if (s->pending.empty()) return 0;
  return (int)s->pending.size() >= s->b_target ||
         now_us - s->pending.front().arrival_us >= s->max_wait_us;
}

int fc_sched_form_batch(fc_sched* s, int64_t now_us, int free_blocks, int64_t* out_ids,
                        int capacity) {
  if (!s || (!out_ids && capacity > 0) || capacity < 0) return FC_EINVAL;
  if (fc_sched_ready(s, now_us) != 1) return 0;
  const int limit = std::min(s->b_max, capacity);
  const size_t n = s->pending.size();
  std::vector<char> take(n, 0);
  std::vector<int> rest;
  int count = 0;
  int64_t used = 0;
  // requests whose wait time is exceeded: arrival order, skipped if they do not fit
  for (size_t i = 0; i < n; ++i) {
    const Pending& p = s->pending[i];
    if (now_us - p.arrival_us < s->max_wait_us) {
      rest.push_back((int)i);
      continue;
    }
    if (count < limit && used + p.need() <= free_blocks) {
      take[i] = 1;
      ++count;
      used += p.need();
    }
  }
  // the others, smallest need first: the largest number of requests that fits
  std::stable_sort(rest.begin(), rest.end(), [&](int a, int b) {
    const Pending &x = s->pending[a], &y = s->pending[b];
    if (x.need() != y.need()) return x.need() < y.need();
    if (x.arrival_us != y.arrival_us) return x.arrival_us < y.arrival_us;
    return x.id < y.id;
  });
  for (int i : rest) {
    const Pending& p = s->pending[i];
    if (count >= limit || used + p.need() > free_blocks) break;
    take[i] = 1;
    ++count;
    used += p.need();
  }
  // the batch in arrival order; the rest stays queued
  int k = 0;
  std::vector<Pending> left;
  left.reserve(n - count);
  for (size_t i = 0; i < n; ++i) {
    if (take[i])
      out_ids[k++] = s->pending[i].id;
    else
      left.push_back(s->pending[i]);
  }
  s->pending.swap(left);
  return count;
}

int fc_sched_adjust(fc_sched* s, int64_t service_us) {
  if (!s || service_us < 0) return FC_EINVAL;
  s->svc_avg = running_avg(s->svc_avg, service_us);
  if (s->gap_avg > 0 && s->svc_avg > 0) {
    const int64_t want = (s->svc_avg + s->gap_avg - 1) / s->gap_avg;
    s->b_target = (int)std::min<int64_t>(std::max<int64_t>(want, s->b_min), s->b_max);
  } else {
    s->b_target = s->b_min;
  }
  return s->b_target;
}

}  // extern "C"
