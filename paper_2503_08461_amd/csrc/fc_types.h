// Plain descriptor structs shared by the host-side planning (fc_plan.cpp, which
// is built without HIP so that it can run under host sanitizers), the host API
// and the kernels.  No HIP types here.
#pragma once

#include <stdint.h>

namespace fc {

// One compressed request of a batch (device-visible copy of what the host
// scheduler knows).  Offsets are in elements of the buffer they index.
struct ReqDesc {
  int32_t seq_len;    // L_r on entry
  int32_t budget;     // B_r
  int32_t method;     // FC_METHOD_*
  int32_t table_row;  // row of dev_block_tables
  int32_t n_old;      // ceil(L_r / 16)
  int32_t n_new;      // ceil(B_r / 16)
  int32_t old_off;    // start of this request in the saved old-id list
  int32_t new_off;    // start of this request in the new-id list (fresh blocks) or in
                      // the run of released ids (in-place compaction)
  int64_t score_off;  // start of [layer][head][L_r] in the caller's packed scores_out
  int64_t raw_off;    // same in the library's un-pooled score scratch (separate kernels only)
  int64_t kept_off;   // start of [layer][head][B_r] in the kept buffer
  int64_t q_off;      // start of [layer][head][window][d] in q_window
  // chunk-MLP compressor: the image span and the chunk counts of the three segments
  int32_t img_begin, img_end;
  int32_t chunks_text0, chunks_image, chunks_text1;
  // SnapKV: this request's observation window and max-pool width
  int32_t window, pool_kernel;
};

// One (request, modality) job of the chunk-MLP kernel: rows = units x chunks.
struct MlpJob {
  int32_t desc;        // index into descs
  int32_t modality;    // 0 text, 1 image
  int32_t chunks;      // chunks of this modality in the request
  int32_t tile_start;  // first tile of this job (mlp_rows_per_tile rows each)
};

// One request of a decode step (append / attention).
struct DecodeReq {
  int32_t table_row;  // row of dev_block_tables, of new_kv, q and out
  int32_t seq_len;    // tokens cached before the step
  int32_t pop_index;  // append: which pop of this call gives the request its new block, -1 = none;
                      // attention over a kept list: the request's budget
  int32_t pad_;
  int64_t kept_off;   // attention over a kept list: start of [layer][head][budget] in `kept`
};

}  // namespace fc
