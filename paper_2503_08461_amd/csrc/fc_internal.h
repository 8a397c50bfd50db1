// Internal declarations shared by the host API and the kernel launchers of
// libfastcache.  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fc_types.h"

namespace fc {

struct MlpParams {
  const MlpJob* jobs;
  int32_t n_jobs, n_tiles;
  int32_t max_grid;    // workgroups to launch at most (as many as are resident)
  int32_t k, hidden;
  int32_t activation;  // FC_ACT_*
  // weights in operand order, index 0 text / 1 image; w2p[m] starts where w1p[m] ends
  const _Float16* w1p[2];
  const _Float16* w2p[2];
  const float* b1[2];
  const float* b2[2];
};

struct DecodeParams {
  _Float16* kv;
  int32_t n_blocks, n_layers, n_heads, head_dim;
  const int32_t* stack;  // free stack (append: new blocks are stack[top_before - 1 - pop_index])
  int32_t top_before;
  int32_t* block_tables;
  int32_t max_blocks;
  const DecodeReq* reqs;
  int32_t n_req;
  const _Float16* new_kv;  // append: [row][layer][2][head][d]
  const _Float16* q;       // attention: [row][layer][head][d]
  float* out;              // attention: [row][layer][head][d]
  const int32_t* kept;     // attention over kept lists of an uncompacted cache, else NULL
  float scale_log2e;
  int32_t* owner;          // ownership checks (debug mode), else NULL
  int32_t* error_flag;
};

// Everything a kernel of the stage needs.  Passed by value.
struct BatchParams {
  // pool geometry
  _Float16* kv;        // kv[layer][block][2][head][16][d]
  int32_t n_blocks, n_layers, n_heads, head_dim;
  // free stack
  int32_t* stack;
  int32_t top_before;  // top on entry to the call
  int32_t total_new;   // sum of n_new
  int32_t total_old;   // sum of n_old
  // batch
  const ReqDesc* descs;        // [n_comp] in batch order
  const int32_t* order_all;    // [n_comp] desc indices, longest first
  const int32_t* order_snap;   // [n_snap]
  const int32_t* order_knorm;  // [n_knorm]
  const int32_t* order_fused;  // [n_fused] units handled by the fused kernel (both methods)
  int32_t n_comp, n_snap, n_knorm, n_unfused, n_fused;
  int32_t* block_tables;       // caller's [n_req][max_blocks]
  int32_t max_blocks;
  int32_t* old_ids;            // [total_old] saved pre-compression ids
  int32_t* new_ids;            // [total_new]
  const _Float16* q_window;
  const float* lse_window;     // nullable: natural log-sum-exp of every window row, packed like
                               // q_window without the channel axis; pass 1 is skipped
  float* lse_out;              // nullable: write that quantity (from pass 1) and stop
  int32_t window;              // a bound on the windows of this launch's SnapKV units (picks the
                               // number of 16-row query tiles); the unit's own is in its descriptor
  int32_t n_sink;              // leading tokens kept by streaming requests
  int32_t in_place;            // 1: compact inside the request's own blocks
  float scale_log2e;           // scale * log2(e)
  float* raw_scores;           // un-pooled scores of the units that take the separate kernels
  float* scores_out;           // nullable
  int32_t* kept;               // kept indices, packed
  int32_t* error_flag;         // set if a kernel finds something wrong (an ownership check that fails)
  int32_t bounded;             // 1: the fused kernel prunes the second pass of its SnapKV units
  int32_t* owner;              // ownership checks (debug mode): [n_blocks] 0 free, 1 handed out,
                               // 2 being released; NULL when the checks are off
};

// Descriptor bytes that travel as a kernel argument (allocation-free entry point).
struct MetaChunk {
  char bytes[3584];
};

enum KernelSlot {
  K_PLAN_ALLOC = 0,
  K_SNAPKV_SCORE = 1,
  K_KNORM_SCORE = 2,
  K_SELECT = 3,
  K_GATHER = 4,
  K_RECLAIM = 5,
  K_FUSED = 6,
  K_MLP = 7,
  K_APPEND = 8,
  K_DECODE_ATTENTION = 9,
  K_WINDOW_LSE = 10,
  K_COUNT = 11
};

// Launchers (fc_kernels.hip).  Each returns the hipError_t of the launch.
hipError_t launch_stack_init(int32_t* stack, int n_blocks, hipStream_t s);
// owner / flag: ownership checks (debug mode), NULL when off
hipError_t launch_pool_pop(const int32_t* stack, int top, int n, int32_t* out, int32_t* owner,
                           int n_blocks, int32_t* flag, hipStream_t s);
hipError_t launch_pool_push(int32_t* stack, int top, int n, const int32_t* ids, int32_t* owner,
                            int n_blocks, hipStream_t s);
// owner[b] = 1, then 0 for the blocks on the free stack
hipError_t launch_owner_init(int32_t* owner, const int32_t* stack, int top, int n_blocks,
                             hipStream_t s);
// claim (or, revert: give back) the ids of a release; *word collects what was wrong
hipError_t launch_owner_check_ids(const int32_t* ids, int n, int n_blocks, int32_t* owner,
                                  int32_t* word, bool revert, hipStream_t s);
hipError_t launch_owner_check_tables(const BatchParams& p, int32_t* word, bool revert,
                                     hipStream_t s);
hipError_t launch_plan_alloc(const BatchParams& p, hipStream_t s);
hipError_t launch_snapkv_score(const BatchParams& p, hipStream_t s);
// a fill kernel (not a memset: calls may be captured into a graph)
hipError_t launch_zero_ints(int32_t* p, int n, hipStream_t s);
hipError_t launch_knorm_score(const BatchParams& p, hipStream_t s);
hipError_t launch_select(const BatchParams& p, int max_seq_len, hipStream_t s);
hipError_t launch_gather(const BatchParams& p, hipStream_t s);
// score -> select -> gather of every unit of order_fused in one launch; needs
// max_seq_len <= kFusedMaxLen; any_snap: the list holds a SnapKV request
hipError_t launch_fused(const BatchParams& p, bool any_snap, int max_seq_len, hipStream_t s);
static constexpr int kFusedMaxLen = 8192;
hipError_t launch_reclaim(const BatchParams& p, hipStream_t s);
hipError_t launch_meta_upload(const MetaChunk& c, char* dst, int n_bytes, hipStream_t s);
hipError_t kernels_one_time_setup();
// decode-side pool traffic (fc_decode.hip)
hipError_t launch_append(const DecodeParams& p, hipStream_t s);
hipError_t launch_decode_attention(const DecodeParams& p, hipStream_t s);
// chunk-MLP compressor (fc_mlp.hip)
hipError_t mlp_one_time_setup();
size_t mlp_w1p_elems(int head_dim, int hidden, int k);
size_t mlp_w2p_elems(int head_dim, int hidden);
int mlp_rows_per_tile(int hidden);   // rows (units x chunks) one workgroup takes at a time
int mlp_workgroups_per_cu();
hipError_t launch_mlp_permute_weights(const _Float16* w1, const _Float16* w2, _Float16* w1p,
                                      _Float16* w2p, int head_dim, int hidden, int k,
                                      hipStream_t s);
hipError_t launch_mlp_compress(const BatchParams& p, const MlpParams& mp, hipStream_t s);

}  // namespace fc
