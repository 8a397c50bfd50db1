// Host-side planning of libfastcache's batched calls: validation with what the
// host scheduler knows (lengths, methods, budgets, free-block count), prefix
// sums of block counts, request descriptors and work lists.  Plain C++ with no
// HIP in it: fc_api.hip turns a plan into launches, and the CPU tests build
// this file with the host sanitizers and drive it on its own.
#pragma once

#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "fc_types.h"

namespace fc {

// Result codes and limits, numerically those of include/fastcache.h (the
// translation unit that includes both checks it).
enum { PLAN_OK = 0, PLAN_EINVAL = -1, PLAN_ENOMEM = -2 };
enum { PLAN_METHOD_NONE = 0, PLAN_METHOD_SNAPKV = 1, PLAN_METHOD_KNORM = 2, PLAN_METHOD_STREAMING = 3 };
enum { PLAN_SCORE_AUTO = 0, PLAN_SCORE_TWO_PASS = 1 };
static constexpr int kPlanBlockSize = 16;
static constexpr int kPlanMaxWindow = 64;
static constexpr int kPlanMaxSeqLen = 32768;
static constexpr int kPlanMaxPoolKernel = 63;
static constexpr int kPlanFusedMaxLen = 8192;   // longest head the fused kernel takes
static constexpr int kPlanClasses = 5;          // query-tile counts 0..4 (0: no queries)

// What the pool contributes to a plan.
struct PoolView {
  int n_layers = 0, n_heads = 0, head_dim = 0;
  int n_free = 0;                       // free blocks on entry
  int score_mode = PLAN_SCORE_AUTO;
  bool in_place = false;
};

// The caller's arguments of fc_compress_batch / _var / _lse, pointers reduced
// to what validation needs.
struct CompressArgs {
  int n_req = 0, max_blocks = 0;
  const int32_t* seq_lens = nullptr;    // [n_req]
  const int32_t* method = nullptr;      // [n_req]
  const int32_t* budget = nullptr;      // [n_req]
  const int32_t* window_per_req = nullptr;       // [n_req] or NULL: `window` for all
  const int32_t* pool_kernel_per_req = nullptr;  // [n_req] or NULL: `pool_kernel` for all
  int window = 0, pool_kernel = 0;
  bool need_lse = false;
  bool q_ok = false;                    // dev_q_window non-NULL and 16-byte aligned
  bool lse_ok = false;                  // dev_lse_window non-NULL and 4-byte aligned
};

// Work lists of a compress call (descriptor indices, heaviest first).
enum {
  LIST_FUSED = 0,                  // + class: units of the fused kernel, per query-tile count
  LIST_SNAP = kPlanClasses,        // + class: separate two-pass score kernel
  LIST_KNORM = 2 * kPlanClasses,   // separate key-norm score kernel
  LIST_ALL,                        // select and gather of the separate path
  N_LISTS
};

struct CompressPlan {
  int code = PLAN_OK;
  char message[256] = "";
  std::vector<ReqDesc> descs;                 // compressed requests, batch order
  std::vector<int32_t> lists[N_LISTS];
  int max_len[N_LISTS] = {};
  int total_new = 0, total_old = 0, total_released = 0;
  int window_hi = 0;                          // largest window of a SnapKV request
  size_t kept_entries = 0;                    // ints of the kept buffer
  size_t score_entries = 0;                   // floats of a packed scores_out
  size_t raw_floats = 0;                      // floats of un-pooled score scratch
  int top_after = 0;                          // free blocks after the call
};

// Fills `plan`; returns plan->code.  On an error nothing else in the plan is
// meaningful.  A batch with nothing to compress gives PLAN_OK and no descs.
int plan_compress(const PoolView& pool, const CompressArgs& args, CompressPlan* plan);

// fc_window_lse: one descriptor per SnapKV request (all if method is NULL),
// longest first, queries packed as [n_req][...][window].
struct LsePlan {
  int code = PLAN_OK;
  char message[256] = "";
  std::vector<ReqDesc> descs;
};
int plan_window_lse(const PoolView& pool, int n_req, int max_blocks, const int32_t* seq_lens,
                    const int32_t* method, int window, LsePlan* plan);

// fc_compress_batch_mlp.
struct MlpPlan {
  int code = PLAN_OK;
  char message[256] = "";
  std::vector<ReqDesc> descs;
  std::vector<MlpJob> jobs;
  int total_new = 0, total_old = 0;
  long long n_tiles = 0;
  int top_after = 0;
};
int plan_mlp(const PoolView& pool, int n_req, int max_blocks, const int32_t* seq_lens,
             const int32_t* img_begin, const int32_t* img_end, const int32_t* enable, int k,
             int tile_rows, MlpPlan* plan);

// fc_append_batch and the decode attentions.
struct DecodePlan {
  int code = PLAN_OK;
  char message[256] = "";
  std::vector<DecodeReq> reqs;
  int n_pop = 0;
  size_t kept_entries = 0;
};
int plan_append(const PoolView& pool, int n_req, int max_blocks, const int32_t* seq_lens,
                const int32_t* enable, DecodePlan* plan);
int plan_decode_attention(const PoolView& pool, int n_req, int max_blocks, const int32_t* seq_lens,
                          const int32_t* budget /* NULL: whole cache */, DecodePlan* plan);

}  // namespace fc
