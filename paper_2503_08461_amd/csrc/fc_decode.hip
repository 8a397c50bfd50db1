// Decode-side pool traffic (Algorithm 1, ExecuteDecoding: every step reads the
// compressed cache of each request of the batch and appends the new token's
// K and V): a batched one-token append and the single-query attention of one
// decode step over the paged cache.  Both are HBM-bound: the append moves
// 4*d bytes per (request, layer, head), the attention reads every cached K and
// V row once, 4*d bytes per token of a (layer, head).

#include "fc_device.h"

namespace fc {

// ---------------------------------------------------------------------------
// append: workgroup = (request, layer); the 2 * n_heads new rows of that layer
// go to slot L % 16 of the request's last block.  A request on a block
// boundary takes the block that the host assigned it from the top of the free
// stack (pops in batch order) and the layer-0 workgroup records it in the table.
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kThreads) void append_kernel(DecodeParams p) {
  const int r = blockIdx.x / p.n_layers;
  const int layer = blockIdx.x - r * p.n_layers;
  const DecodeReq rq = p.reqs[r];
  const int L = rq.seq_len;
  int32_t* row = p.block_tables + (size_t)rq.table_row * p.max_blocks;
  int blk;
  if (rq.pop_index >= 0) {
    const int id = p.stack[p.top_before - 1 - rq.pop_index];
    blk = clamp_block(id, p.n_blocks);
    if (layer == 0 && threadIdx.x == 0) {
      row[L >> 4] = blk;
      // ownership checks (debug mode): a popped block must have been free
      if (p.owner && ((unsigned)id >= (unsigned)p.n_blocks || atomicExch(&p.owner[id], 1) != 0))
        atomicOr(p.error_flag, 4 << 8);
    }
  } else {
    blk = clamp_block(row[L >> 4], p.n_blocks);
  }
  constexpr int PPR = D / 8;  // 16-byte pieces of a row
  const size_t blk_stride = (size_t)2 * p.n_heads * 16 * D;
  _Float16* dst = p.kv + ((size_t)layer * p.n_blocks + blk) * blk_stride + (size_t)(L & 15) * D;
  const _Float16* src = p.new_kv + ((size_t)rq.table_row * p.n_layers + layer) * 2 * p.n_heads * D;
  for (int i = threadIdx.x; i < 2 * p.n_heads * PPR; i += kThreads) {
    const int rh = i / PPR, piece = i - rh * PPR;  // rh = kv * n_heads + head
    store_half8(dst + (size_t)rh * 16 * D + piece * 8, load_half8(src + (size_t)rh * D + piece * 8));
  }
}

hipError_t launch_append(const DecodeParams& p, hipStream_t s) {
  if (p.n_req == 0) return hipSuccess;
  const unsigned grid = (unsigned)p.n_req * p.n_layers;
  if (p.head_dim == 128)
    append_kernel<128><<<grid, kThreads, 0, s>>>(p);
  else if (p.head_dim == 64)
    append_kernel<64><<<grid, kThreads, 0, s>>>(p);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// attention of one decode step: workgroup = (request, layer, head), requests
// in the order the host lists them (longest first).  A 16-token block of one
// head is 32*D contiguous bytes for K and for V; a wavefront reads it with
// D/8 neighbouring lanes on one row (fully coalesced 16-byte loads), forms
// q.k by a reduction inside that lane group, and keeps one online-softmax state
// (running max, sum, and this lane's 8 output channels) per lane group.  The
// 4 * (512 / D) states of the workgroup are merged through LDS at the end.
// ---------------------------------------------------------------------------
//
// kIndexed: the counterfactual of a cache that was pruned WITHOUT compaction:
// the unit attends over the budget_r tokens of its kept list, read where they
// lie in the uncompacted cache (every row its own 2*D contiguous bytes).
template <int D, bool kIndexed>
__global__ __launch_bounds__(kThreads) void decode_attention_kernel(DecodeParams p) {
  constexpr int LPR = D / 8;        // lanes per row
  constexpr int RPI = 64 / LPR;     // rows per wavefront load instruction
  constexpr int IPB = 16 / RPI;     // load instructions per 16-token block
  constexpr int NG = kWaves * RPI;  // softmax states per workgroup
  const int n_lh = p.n_layers * p.n_heads;
  const int unit = blockIdx.x;
  const DecodeReq rq = p.reqs[unit / n_lh];
  const int lh = unit - (unit / n_lh) * n_lh;
  const int layer = lh / p.n_heads;
  const int head = lh - layer * p.n_heads;
  const int L = kIndexed ? rq.pop_index : rq.seq_len;  // indexed: pop_index holds the budget
  const int32_t* kept =
      kIndexed ? p.kept + rq.kept_off + (size_t)lh * L : nullptr;  // ascending token indices
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int grp = lane / LPR;    // which row of a load instruction
  const int piece = lane % LPR;  // which 8 channels
  float* out = p.out + ((size_t)rq.table_row * n_lh + lh) * D;

  const _Float16* qp = p.q + ((size_t)rq.table_row * n_lh + lh) * D + piece * 8;
  float qf[8];
  {
    const half8 qh = load_half8(qp);
#pragma unroll
    for (int e = 0; e < 8; ++e) qf[e] = (float)qh[e] * p.scale_log2e;
  }
  const int32_t* row = p.block_tables + (size_t)rq.table_row * p.max_blocks;
  const size_t blk_stride = (size_t)2 * p.n_heads * 16 * D;
  const size_t v_off = (size_t)p.n_heads * 16 * D;
  const _Float16* base = p.kv + (size_t)layer * p.n_blocks * blk_stride + (size_t)head * 16 * D +
                         (kIndexed ? 0 : (size_t)grp * D) + piece * 8;

  float m = -INFINITY, z = 0.f, acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const int nb = (L + 15) >> 4;
  for (int b = wave; b < nb; b += kWaves) {
    half8 k[IPB], v[IPB];
    if (kIndexed) {
      // 16 kept tokens at a time, each fetched from its own block and slot
#pragma unroll
      for (int i = 0; i < IPB; ++i) {
        const int j = b * 16 + i * RPI + grp;
        const int tok = min(max(kept[min(j, L - 1)], 0), rq.seq_len - 1);
        const _Float16* kp = base + (size_t)clamp_block(row[tok >> 4], p.n_blocks) * blk_stride +
                             (size_t)(tok & 15) * D;
        k[i] = load_half8_nt(kp);
        v[i] = load_half8_nt(kp + v_off);
      }
    } else {
      const _Float16* kp = base + (size_t)clamp_block(row[b], p.n_blocks) * blk_stride;
#pragma unroll
      for (int i = 0; i < IPB; ++i) {
        k[i] = load_half8_nt(kp + (size_t)i * RPI * D);
        v[i] = load_half8_nt(kp + v_off + (size_t)i * RPI * D);
      }
    }
#pragma unroll
    for (int i = 0; i < IPB; ++i) {
      float s = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) s += qf[e] * (float)k[i][e];
#pragma unroll
      for (int o = 1; o < LPR; o <<= 1) s += __shfl_xor(s, o);
      const int tok = b * 16 + i * RPI + grp;
      if (tok < L) {  // the whole lane group takes the same branch
        const float mn = fmaxf(m, s);
        const float a = __builtin_amdgcn_exp2f(m - mn);  // 0 for the first token (m = -inf)
        const float w = __builtin_amdgcn_exp2f(s - mn);
        z = z * a + w;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = acc[e] * a + w * (float)v[i][e];
        m = mn;
      }
    }
  }

  // merge the NG states: each has its own max, so rescale to the common one
  __shared__ float sm_m[NG], sm_z[NG];
  __shared__ float sm_acc[NG][D];
  const int g = wave * RPI + grp;
  if (piece == 0) {
    sm_m[g] = m;
    sm_z[g] = z;
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) sm_acc[g][piece * 8 + e] = acc[e];
  __syncthreads();
  if (threadIdx.x < D) {
    float mm = -INFINITY;
    for (int i = 0; i < NG; ++i) mm = fmaxf(mm, sm_m[i]);
    float zz = 0.f, o = 0.f;
    for (int i = 0; i < NG; ++i) {
      const float f = sm_m[i] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(sm_m[i] - mm);
      zz += sm_z[i] * f;
      o += sm_acc[i][threadIdx.x] * f;
    }
    out[threadIdx.x] = L > 0 ? o / zz : 0.f;
  }
}

hipError_t launch_decode_attention(const DecodeParams& p, hipStream_t s) {
  if (p.n_req == 0) return hipSuccess;
  const unsigned grid = (unsigned)p.n_req * p.n_layers * p.n_heads;
  const bool indexed = p.kept != nullptr;
  if (p.head_dim == 128 && !indexed)
    decode_attention_kernel<128, false><<<grid, kThreads, 0, s>>>(p);
  else if (p.head_dim == 128)
    decode_attention_kernel<128, true><<<grid, kThreads, 0, s>>>(p);
  else if (p.head_dim == 64 && !indexed)
    decode_attention_kernel<64, false><<<grid, kThreads, 0, s>>>(p);
  else if (p.head_dim == 64)
    decode_attention_kernel<64, true><<<grid, kThreads, 0, s>>>(p);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace fc
