// HIP kernels of the batched KV-cache compression stage, written for gfx950
// (CDNA4: 64-wide wavefronts, MFMA, 160 KB LDS per CU).
//
// Pool layout (fixed by the public ABI):
//   kv[layer][block][0=K,1=V][head][slot 0..15][d]   fp16
// so one (layer, block, kv, head) chunk is 16*d contiguous halves (4 KiB at
// d = 128) and one token row is d contiguous halves.

#include "fc_device.h"

#include <float.h>

namespace fc {

// ---------------------------------------------------------------------------
// free stack
// ---------------------------------------------------------------------------

__global__ void stack_init_kernel(int32_t* stack, int n_blocks) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_blocks) stack[i] = n_blocks - 1 - i;
}

// ---------------------------------------------------------------------------
// ownership checks (debug mode)
// ---------------------------------------------------------------------------
//
// owner[b]: 0 = block b is on the free stack, 1 = handed out, 2 = named by a
// release that is being checked.  A release (fc_pool_free, or the reclaim of a
// compression) is checked before it is carried out: every id must be in range
// and handed out, and no id may come twice; the check claims each id with a
// compare-and-swap 1 -> 2, so a second occurrence finds 2.  The host reads the
// verdict and either lets the release go ahead (2 -> 0 as the ids are pushed)
// or takes the claims back (2 -> 1) and refuses the call.
enum { kOwnBadRange = 1, kOwnNotOwned = 2, kOwnNotFree = 4 };

__device__ __forceinline__ void owner_claim(int32_t* owner, int id, int n_blocks, int32_t* word) {
  if ((unsigned)id >= (unsigned)n_blocks) {
    atomicOr(word, kOwnBadRange);
  } else if (atomicCAS(&owner[id], 1, 2) != 1) {
    atomicOr(word, kOwnNotOwned);
  }
}

__device__ __forceinline__ void owner_unclaim(int32_t* owner, int id, int n_blocks) {
  if ((unsigned)id < (unsigned)n_blocks) atomicCAS(&owner[id], 2, 1);
}

__global__ void owner_fill_kernel(int32_t* owner, int n_blocks, int value) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_blocks) owner[i] = value;
}

__global__ void owner_mark_free_kernel(int32_t* owner, const int32_t* stack, int top, int n_blocks) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < top && (unsigned)stack[i] < (unsigned)n_blocks) owner[stack[i]] = 0;
}

__global__ void owner_check_ids_kernel(const int32_t* ids, int n, int n_blocks, int32_t* owner,
                                       int32_t* word, int revert) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  if (revert)
    owner_unclaim(owner, ids[i], n_blocks);
  else
    owner_claim(owner, ids[i], n_blocks, word);
}

// the table rows of the requests a compression is about to release
__global__ __launch_bounds__(kThreads) void owner_check_tables_kernel(BatchParams p, int32_t* word,
                                                                    int revert) {
  const ReqDesc rd = p.descs[blockIdx.x];
  const int32_t* row = p.block_tables + (size_t)rd.table_row * p.max_blocks;
  for (int i = threadIdx.x; i < rd.n_old; i += kThreads) {
    if (revert)
      owner_unclaim(p.owner, row[i], p.n_blocks);
    else
      owner_claim(p.owner, row[i], p.n_blocks, word);
  }
}

// a popped id must have been free
__device__ __forceinline__ void owner_take(int32_t* owner, int id, int n_blocks, int32_t* flag) {
  if (!owner) return;
  if ((unsigned)id >= (unsigned)n_blocks || atomicExch(&owner[id], 1) != 0) atomicOr(flag, kOwnNotFree << 8);
}

__global__ void pool_pop_kernel(const int32_t* stack, int top, int n, int32_t* out, int32_t* owner,
                                int n_blocks, int32_t* flag) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) {
    const int id = stack[top - 1 - i];
    out[i] = id;
    owner_take(owner, id, n_blocks, flag);
  }
}

__global__ void pool_push_kernel(int32_t* stack, int top, int n, const int32_t* ids, int32_t* owner,
                                 int n_blocks) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) {
    stack[top + i] = ids[i];
    if (owner && (unsigned)ids[i] < (unsigned)n_blocks) owner[ids[i]] = 0;  // checked before
  }
}

// Writes descriptor bytes that came as a kernel argument to device memory.
__global__ void meta_upload_kernel(MetaChunk c, char* dst, int n_bytes) {
  for (int i = threadIdx.x; i < n_bytes; i += blockDim.x) dst[i] = c.bytes[i];
}

// Pops the new blocks of every compressed request (batch order) and saves the
// pre-compression ids.  One workgroup per request; offsets are exclusive
// prefix sums computed by the host, which knows every count.
__global__ __launch_bounds__(kThreads) void plan_alloc_kernel(BatchParams p) {
  const ReqDesc rd = p.descs[blockIdx.x];
  const int32_t* row = p.block_tables + (size_t)rd.table_row * p.max_blocks;
  for (int i = threadIdx.x; i < rd.n_old; i += kThreads)
    p.old_ids[rd.old_off + i] = row[i];
  if (!p.in_place)
    for (int i = threadIdx.x; i < rd.n_new; i += kThreads) {
      const int id = p.stack[p.top_before - 1 - rd.new_off - i];
      p.new_ids[rd.new_off + i] = id;
      owner_take(p.owner, id, p.n_blocks, p.error_flag);
    }
}

// Zombie reclaim: pushes the pre-compression blocks (batch order, table
// order) above the stack top left by plan_alloc and rewrites the table rows.
__global__ __launch_bounds__(kThreads) void reclaim_kernel(BatchParams p) {
  const ReqDesc rd = p.descs[blockIdx.x];
  int32_t* row = p.block_tables + (size_t)rd.table_row * p.max_blocks;
  if (p.in_place) {
    // the request keeps its first n_new blocks; the rest are released
    for (int i = threadIdx.x; i < rd.n_old - rd.n_new; i += kThreads)
      p.stack[p.top_before + rd.new_off + i] = p.old_ids[rd.old_off + rd.n_new + i];
    for (int i = rd.n_new + threadIdx.x; i < p.max_blocks; i += kThreads) row[i] = -1;
    if (p.owner)  // (ids checked before the stage: in range, claimed)
      for (int i = threadIdx.x; i < rd.n_old; i += kThreads)
        p.owner[p.old_ids[rd.old_off + i]] = i < rd.n_new ? 1 : 0;
    return;
  }
  const int base = p.top_before - p.total_new;
  for (int i = threadIdx.x; i < rd.n_old; i += kThreads) {
    p.stack[base + rd.old_off + i] = p.old_ids[rd.old_off + i];
    if (p.owner) p.owner[p.old_ids[rd.old_off + i]] = 0;  // (checked before the stage)
  }
  for (int i = threadIdx.x; i < p.max_blocks; i += kThreads)
    row[i] = (i < rd.n_new) ? p.new_ids[rd.new_off + i] : -1;
}

// ---------------------------------------------------------------------------
// SnapKV-style observation-window score
// ---------------------------------------------------------------------------
//
// One workgroup per (request, layer, head).  A wavefront takes pool blocks
// (16 tokens) round-robin and feeds them to v_mfma_f32_16x16x32_f16 straight
// from global memory: lane l holds 8 consecutive channels
// [32*ks + 8*(l/16), +8) of token l%16, which is both the A-operand layout
// (rows = tokens) and the B-operand layout (columns = tokens) of that
// instruction, and 4 lanes cover 64 contiguous bytes of a token row.
//
// Pass 1 (A = keys, B = queries): the 16x16 result has the window query on the
// lane (l%16) and 4 tokens in the lane's registers, so every lane keeps an
// online (max, sum-of-exp) pair for its query with no cross-lane traffic.
// Pass 2 (A = queries, B = keys): the result has the token on the lane and 4
// queries in registers, so the sum over window queries is an in-lane add plus
// two cross-lane adds.  Softmax uses exp2 with scale*log2(e) folded in.
//
// The un-pooled column sums of the prefix are written to raw_scores; pooling
// and the forced window are applied by the select kernel.

// Epochs of the bound-keeping first pass: wavefront w takes blocks w, w + kWaves,
// ...; its t-th block belongs to epoch 0 (t = 0), 1 (t = 1), 2 (t = 2, 3) and
// then to 2 + t / 4: the references are renewed before t = 1, 2 and every
// multiple of 4, by all wavefronts together.
static constexpr int kBoundSeg = 4;
static constexpr int kBoundMinLen = 512;  // shorter heads take the two passes
static constexpr int kBoundMaxEpochs = 3 + (kFusedMaxLen / 16 / kWaves + kBoundSeg - 1) / kBoundSeg;
__host__ __device__ constexpr int bound_epoch_of_step(int t) {
  return t < 2 ? t : (t < kBoundSeg ? 2 : 2 + t / kBoundSeg);
}
__host__ __device__ constexpr bool bound_renews_before(int t) {
  return t == 1 || t == 2 || (t >= kBoundSeg && t % kBoundSeg == 0);
}

struct ScoreShared {
  float m[kWaves][4][64];
  float z[kWaves][4][64];
  float fin[64];
};

// Scores one (request, layer, head); store(j, a_j) receives the un-pooled
// column sum of every prefix token j.  All threads of the workgroup call.
// `old_ids` are the request's pre-compression block ids (global or LDS copy).
// The window queries of a (request, layer, head) in MFMA operand layout (rows
// past the window are zero), resident in registers for every pass over K.
template <int D, int NT>
__device__ __forceinline__ void load_window_queries(const BatchParams& p, const ReqDesc& rd, int lh,
                                                    half8 (&qreg)[NT][D / 32]) {
  constexpr int KS = D / 32;
  const int lane = threadIdx.x & 63;
  const int c16 = lane & 15;
  const int q4 = lane >> 4;
  const int W = rd.window;
  const _Float16* qbase = p.q_window + rd.q_off + (size_t)lh * W * D;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int row = nt * 16 + c16;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      half8 z = {0, 0, 0, 0, 0, 0, 0, 0};
      qreg[nt][ks] = (row < W) ? load_half8(qbase + (size_t)row * D + ks * 32 + q4 * 8) : z;
    }
  }
}

template <int D, int NT, typename Store>
__device__ __forceinline__ void snapkv_unit_q(const BatchParams& p, const ReqDesc& rd, int lh,
                                              const int32_t* old_ids, ScoreShared& sh,
                                              half8 (&qreg)[NT][D / 32], Store store) {
  constexpr int KS = D / 32;
  const int layer = lh / p.n_heads;
  const int head = lh - layer * p.n_heads;
  const int L = rd.seq_len;
  const int W = rd.window;  // <= 16 NT; the rows past it are padding
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c16 = lane & 15;
  const int q4 = lane >> 4;

  const size_t blk_stride = (size_t)2 * p.n_heads * 16 * D;
  const _Float16* kbase = p.kv + (size_t)layer * p.n_blocks * blk_stride +
                          (size_t)head * 16 * D + (size_t)c16 * D + q4 * 8;
  const float c = p.scale_log2e;
  const int nb = (L + 15) >> 4;
  const int n_unmasked = (L - W) >> 4;  // blocks that lie wholly before the window

  // last use of a block (second pass)
  auto load_block_nt = [&](int b, half8 (&k)[KS]) {
    const int blk = clamp_block(old_ids[b], p.n_blocks);
    const _Float16* kp = kbase + (size_t)blk * blk_stride;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) k[ks] = load_half8_nt(kp + ks * 32);
  };
  auto load_block = [&](int b, half8 (&k)[KS]) {
    const int blk = clamp_block(old_ids[b], p.n_blocks);
    const _Float16* kp = kbase + (size_t)blk * blk_stride;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) k[ks] = load_half8(kp + ks * 32);
  };

  // log2 of every row's soft-max denominator goes to sh.fin: handed in by the
  // caller (natural log, from its attention kernel), or pass 1 below
  const size_t lse_off = (size_t)(rd.q_off / D) + (size_t)lh * W;
  if (p.lse_window != nullptr) {  // uniform
    if (threadIdx.x < 64)
      sh.fin[threadIdx.x] = (int)threadIdx.x < W
                                ? p.lse_window[lse_off + threadIdx.x] * 1.44269504088896340736f
                                : INFINITY;  // padded rows contribute exp2(-inf) = 0
    __syncthreads();
  } else {
  // ---- pass 1: row maxima and normalisers --------------------------------
  float m[NT], z[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    m[nt] = -3.0e38f;
    z[nt] = 0.f;
  }
  {
    half8 kc[KS], kn[KS];
    int b = wave;
    if (b < nb) load_block(b, kc);
    for (; b < nb; b += kWaves) {
      if (b + kWaves < nb) load_block(b + kWaves, kn);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(kc[ks], qreg[nt][ks], acc, 0, 0, 0);
        float t[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) t[r] = acc[r] * c;
        if (b >= n_unmasked) {
          // query i at position L-W+i sees tokens <= its own position
          const int limit = L - W + nt * 16 + c16;
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int tok = b * 16 + q4 * 4 + r;
            if (tok > limit) t[r] = -INFINITY;
          }
        }
        const float bm = fmaxf(fmaxf(t[0], t[1]), fmaxf(t[2], t[3]));
        const float mn = fmaxf(m[nt], bm);
        float zz = z[nt] * __builtin_amdgcn_exp2f(m[nt] - mn);
#pragma unroll
        for (int r = 0; r < 4; ++r) zz += __builtin_amdgcn_exp2f(t[r] - mn);
        z[nt] = zz;
        m[nt] = mn;
      }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) kc[ks] = kn[ks];
    }
  }

  // combine the 16 partial (max, sum) pairs of every query
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    sh.m[wave][q4][nt * 16 + c16] = m[nt];
    sh.z[wave][q4][nt * 16 + c16] = z[nt];
  }
  __syncthreads();
  if (threadIdx.x < 64) {
    const int row = threadIdx.x;
    float out = INFINITY;  // padded rows contribute exp2(-inf) = 0
    if (row < W) {
      float mm = -3.0e38f;
      for (int w = 0; w < kWaves; ++w)
        for (int q = 0; q < 4; ++q) mm = fmaxf(mm, sh.m[w][q][row]);
      float zz = 0.f;
      for (int w = 0; w < kWaves; ++w)
        for (int q = 0; q < 4; ++q)
          zz += sh.z[w][q][row] * __builtin_amdgcn_exp2f(sh.m[w][q][row] - mm);
      out = mm + log2f(zz);
    }
    sh.fin[row] = out;
  }
  __syncthreads();
  }
  if (p.lse_out != nullptr) {  // uniform: the caller asked for the denominators only
    if ((int)threadIdx.x < W)
      p.lse_out[lse_off + threadIdx.x] = sh.fin[threadIdx.x] * 0.69314718055994530942f;
    return;
  }

  // ---- pass 2: column sums of the soft-maxed rows over the prefix ---------
  const int n_prefix = L - W;
  const int nb2 = (n_prefix + 15) >> 4;
  float mrow[NT][4];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt)
#pragma unroll
    for (int r = 0; r < 4; ++r) mrow[nt][r] = sh.fin[nt * 16 + q4 * 4 + r];

  {
    // from the end of the prefix backwards: the blocks that the first pass read
    // last are the ones most likely to be still in a cache
    half8 kc[KS], kn[KS];
    int b = nb2 - 1 - wave;
    if (b >= 0) load_block_nt(b, kc);
    for (; b >= 0; b -= kWaves) {
      if (b - kWaves >= 0) load_block_nt(b - kWaves, kn);
      float colsum = 0.f;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(qreg[nt][ks], kc[ks], acc, 0, 0, 0);
#pragma unroll
        for (int r = 0; r < 4; ++r)
          colsum += __builtin_amdgcn_exp2f(acc[r] * c - mrow[nt][r]);
      }
      colsum += __shfl_xor(colsum, 16);
      colsum += __shfl_xor(colsum, 32);
      const int tok = b * 16 + c16;
      if (q4 == 0 && tok < n_prefix) store(tok, colsum);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) kc[ks] = kn[ks];
    }
  }
}

template <int D, int NT, typename Store>
__device__ __forceinline__ void snapkv_unit(const BatchParams& p, const ReqDesc& rd, int lh,
                                            const int32_t* old_ids, ScoreShared& sh, Store store) {
  half8 qreg[NT][D / 32];
  load_window_queries<D, NT>(p, rd, lh, qreg);
  snapkv_unit_q<D, NT>(p, rd, lh, old_ids, sh, qreg, store);
}

template <int D, int NT>
__global__ __launch_bounds__(kThreads) void snapkv_score_kernel(BatchParams p) {
  __shared__ ScoreShared sh;
  const int n_lh = p.n_layers * p.n_heads;
  const int slot = blockIdx.x / n_lh;
  const int lh = blockIdx.x - slot * n_lh;
  const ReqDesc rd = p.descs[p.order_snap[slot]];
  float* raw = p.raw_scores + rd.raw_off + (size_t)lh * rd.seq_len;
  // the denominators-only call runs outside a compression: no saved ids, the table row itself
  const int32_t* ids = p.lse_out != nullptr ? p.block_tables + (size_t)rd.table_row * p.max_blocks
                                            : p.old_ids + rd.old_off;
  snapkv_unit<D, NT>(p, rd, lh, ids, sh, [&](int j, float v) { raw[j] = v; });
}

// ---------------------------------------------------------------------------
// key-norm score: raw[j] = -||k_j||_2
// ---------------------------------------------------------------------------
//
// One workgroup per (request, layer, head); a wavefront reads one 16-token
// chunk with fully coalesced 128-bit loads (64 lanes x 16 B = 1 KiB per
// instruction) and reduces the squares over the lanes that share a row.

template <int D, typename Store>
__device__ __forceinline__ void knorm_unit(const BatchParams& p, const ReqDesc& rd, int lh,
                                           const int32_t* old_ids, Store store) {
  constexpr int LPR = D / 8;     // lanes per token row
  constexpr int RPI = 64 / LPR;  // rows per load instruction
  constexpr int NI = 16 / RPI;   // load instructions per block
  const int layer = lh / p.n_heads;
  const int head = lh - layer * p.n_heads;
  const int L = rd.seq_len;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const size_t blk_stride = (size_t)2 * p.n_heads * 16 * D;
  const _Float16* kbase = p.kv + (size_t)layer * p.n_blocks * blk_stride +
                          (size_t)head * 16 * D + lane * 8;
  const int nb = (L + 15) >> 4;
  for (int b = wave; b < nb; b += kWaves) {
    const int blk = clamp_block(old_ids[b], p.n_blocks);
    const _Float16* kp = kbase + (size_t)blk * blk_stride;
    half8 v[NI];
#pragma unroll
    for (int k = 0; k < NI; ++k) v[k] = load_half8(kp + k * 512);
#pragma unroll
    for (int k = 0; k < NI; ++k) {
      float s = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float x = (float)v[k][e];
        s += x * x;
      }
#pragma unroll
      for (int o = 1; o < LPR; o <<= 1) s += __shfl_xor(s, o);
      const int tok = b * 16 + k * RPI + lane / LPR;
      if ((lane % LPR) == 0 && tok < L) store(tok, -sqrtf(s));
    }
  }
}

template <int D>
__global__ __launch_bounds__(kThreads) void knorm_score_kernel(BatchParams p) {
  const int n_lh = p.n_layers * p.n_heads;
  const int slot = blockIdx.x / n_lh;
  const int lh = blockIdx.x - slot * n_lh;
  const ReqDesc rd = p.descs[p.order_knorm[slot]];
  float* raw = p.raw_scores + rd.raw_off + (size_t)lh * rd.seq_len;
  knorm_unit<D>(p, rd, lh, p.old_ids + rd.old_off, [&](int j, float v) { raw[j] = v; });
}

// ---------------------------------------------------------------------------
// per-head top-budget selection
// ---------------------------------------------------------------------------
//
// One workgroup per (request, layer, head).  Only the tokens before the
// observation window compete (window tokens are always kept), so the kernel
// selects the budget-minus-window best of the prefix and appends the window.
//
//   1. the un-pooled scores are staged in LDS, max-pooled from LDS and turned
//      in place into order-preserving 32-bit keys; min and max key are reduced
//      on the way;
//   2. the threshold (the k-th largest key) is found by a bucket select: 2048
//      linear buckets over [min, max] (so the histogram is spread even when
//      every score shares its exponent), then the keys of the one bucket that
//      holds the threshold are compacted to a short candidate list, which is
//      refined with 2048 buckets per pass until a bucket is a single key
//      (at most 3 passes for 32 bits);
//   3. the kept indices are emitted in ascending token order by a ballot /
//      popcount compaction in which keys equal to the threshold are admitted
//      in index order until the budget is met (ties go to the lower index).

__device__ __forceinline__ uint32_t score_key(float s) {
  s += 0.0f;  // -0 and +0 compare equal, give them one key
  const uint32_t u = __float_as_uint(s);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

static constexpr int kBuckets = 2048;
static constexpr int kBucketBits = 11;
static constexpr int kMaxCand = 2048;
static constexpr int kStagePerThread = 32;  // staging path handles up to 32*256 tokens

// Finds, among the `n` keys produced by get(j) that lie in [lo, lo + width)
// (width == 0: all of them do, no check), the bucket (key - lo) >> shift that
// holds the `remaining`-th largest.  Returns the bucket in sel[0] and the rank
// inside it in sel[1].  All threads must call.
template <typename Get>
__device__ __forceinline__ void bucket_pass(int n, uint32_t lo, int shift, uint32_t width,
                                            int remaining, int* hist, int* wsum, int* sel,
                                            Get get) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
#pragma unroll
  for (int i = 0; i < kBuckets / kThreads; ++i) hist[tid + i * kThreads] = 0;
  __syncthreads();
  for (int j = tid; j < n; j += kThreads) {
    const uint32_t k = get(j);
    const uint32_t d = k - lo;
    if (width == 0u || (k >= lo && d < width)) atomicAdd(&hist[d >> shift], 1);
  }
  __syncthreads();
  // thread t owns buckets [8t, 8t+8)
  int own[kBuckets / kThreads];
  int s = 0;
#pragma unroll
  for (int i = 0; i < kBuckets / kThreads; ++i) {
    own[i] = hist[tid * (kBuckets / kThreads) + i];
    s += own[i];
  }
  int v = s;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int t = __shfl_up(v, o);
    if (lane >= o) v += t;
  }
  if (lane == 63) wsum[wave] = v;
  __syncthreads();
  int base = 0, total = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    if (w < wave) base += wsum[w];
    total += wsum[w];
  }
  int above = total - (v + base);  // keys in buckets above this thread's
#pragma unroll
  for (int i = kBuckets / kThreads - 1; i >= 0; --i) {
    if (above < remaining && above + own[i] >= remaining) {
      sel[0] = tid * (kBuckets / kThreads) + i;
      sel[1] = remaining - above;
    }
    above += own[i];
  }
  __syncthreads();
}

struct SelectShared {
  int hist[kBuckets];
  uint32_t cand[kMaxCand];
  int wsum[kWaves];
  uint32_t wmin[kWaves], wmax[kWaves];
  int sel[2];
  int n_cand;
  int cnt[kWaves][2];
};

// Selects the kept tokens of one (request, layer, head) and writes them, in
// ascending order, to the kept list.  `keys` is LDS room for seq_len words.
// kRawInLds: the un-pooled scores already sit in keys[] (as floats, written
// by this workgroup and made visible by a barrier); otherwise they are read
// from raw_scores.  All threads of the workgroup call.
template <bool kRawInLds>
__device__ __forceinline__ void select_unit(const BatchParams& p, const ReqDesc& rd, int lh,
                                            uint32_t* keys, SelectShared& sh) {
  int* hist = sh.hist;
  uint32_t* cand = sh.cand;
  int* wsum = sh.wsum;
  uint32_t* wmin = sh.wmin;
  uint32_t* wmax = sh.wmax;
  int* sel = sh.sel;
  int& n_cand = sh.n_cand;
  int (*cnt)[2] = sh.cnt;
  const int L = rd.seq_len;
  const int B = rd.budget;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const bool snap = rd.method == 1 /* FC_METHOD_SNAPKV */;
  const int n_sel = snap ? L - rd.window : L;  // tokens that compete
  const int k_sel = snap ? B - rd.window : B;  // how many of them are kept
  const float* raw = p.raw_scores + rd.raw_off + (size_t)lh * L;
  float* out = p.scores_out ? p.scores_out + rd.score_off + (size_t)lh * L : nullptr;
  int32_t* kept = p.kept + rd.kept_off + (size_t)lh * B;

  // ---- 1. final scores -> keys, min / max -------------------------------------
  uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
  if (snap && (kRawInLds || n_sel <= kStagePerThread * kThreads)) {
    float* stage = reinterpret_cast<float*>(keys);
    if (!kRawInLds) {
      for (int j = tid; j < n_sel; j += kThreads) stage[j] = raw[j];
      __syncthreads();
    }
    const int h = rd.pool_kernel >> 1;
    float pv[kStagePerThread];
#pragma unroll
    for (int i = 0; i < kStagePerThread; ++i) {
      const int j = tid + i * kThreads;
      float s = 0.f;
      if (j < n_sel) {
        const int lo = max(0, j - h), hi = min(n_sel - 1, j + h);
        s = stage[lo];
        for (int t = lo + 1; t <= hi; ++t) s = fmaxf(s, stage[t]);
      }
      pv[i] = s;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kStagePerThread; ++i) {
      const int j = tid + i * kThreads;
      if (j < n_sel) {
        const uint32_t k = score_key(pv[i]);
        keys[j] = k;
        kmin = min(kmin, k);
        kmax = max(kmax, k);
        if (out) out[j] = pv[i];
      }
    }
  } else if (snap) {
    const int h = rd.pool_kernel >> 1;
    for (int j = tid; j < n_sel; j += kThreads) {
      const int lo = max(0, j - h), hi = min(n_sel - 1, j + h);
      float s = raw[lo];
      for (int t = lo + 1; t <= hi; ++t) s = fmaxf(s, raw[t]);
      const uint32_t k = score_key(s);
      keys[j] = k;
      kmin = min(kmin, k);
      kmax = max(kmax, k);
      if (out) out[j] = s;
    }
  } else {
    for (int j = tid; j < n_sel; j += kThreads) {
      const float s = kRawInLds ? reinterpret_cast<float*>(keys)[j] : raw[j];
      const uint32_t k = score_key(s);
      keys[j] = k;
      kmin = min(kmin, k);
      kmax = max(kmax, k);
      if (out) out[j] = s;
    }
  }
  if (snap) {
    if (out)
      for (int j = n_sel + tid; j < L; j += kThreads) out[j] = INFINITY;
    for (int j = tid; j < rd.window; j += kThreads) kept[k_sel + j] = n_sel + j;  // forced window
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, o));
    kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, o));
  }
  if (lane == 0) {
    wmin[wave] = kmin;
    wmax[wave] = kmax;
  }
  if (tid == 0) n_cand = 0;
  __syncthreads();
  if (k_sel == 0) return;  // only the window is kept (uniform across the workgroup)
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    kmin = min(kmin, wmin[w]);
    kmax = max(kmax, wmax[w]);
  }

  // ---- 2. threshold = k_sel-th largest key ---------------------------------------
  uint32_t thr;
  int need_eq;
  if (kmin == kmax) {
    thr = kmin;
    need_eq = k_sel;
  } else {
    uint32_t lo = kmin;
    const uint32_t range = kmax - kmin;
    int shift = max(0, 32 - __clz(range) - kBucketBits);
    bucket_pass(n_sel, lo, shift, 0u, k_sel, hist, wsum, sel, [&](int j) { return keys[j]; });
    int remaining = sel[1];
    uint32_t bkt = (uint32_t)sel[0];
    if (shift > 0) {
      // candidates: the keys of that one bucket
      for (int j = tid; j < n_sel; j += kThreads) {
        const uint32_t k = keys[j];
        if (((k - lo) >> shift) == bkt) {
          const int pos = atomicAdd(&n_cand, 1);
          if (pos < kMaxCand) cand[pos] = k;
        }
      }
      __syncthreads();
      const int nc = n_cand;
      const bool listed = nc <= kMaxCand;  // else refine over all keys with a range check
      while (shift > 0) {
        lo += bkt << shift;
        const uint32_t width = 1u << shift;  // the chosen bucket spans [lo, lo + width)
        shift = max(0, shift - kBucketBits);
        if (listed)
          bucket_pass(nc, lo, shift, width, remaining, hist, wsum, sel,
                      [&](int j) { return cand[j]; });
        else
          bucket_pass(n_sel, lo, shift, width, remaining, hist, wsum, sel,
                      [&](int j) { return keys[j]; });
        remaining = sel[1];
        bkt = (uint32_t)sel[0];
      }
    }
    thr = lo + bkt;
    need_eq = remaining;
  }

  // ---- 3. ordered compaction; each wavefront owns a contiguous token segment ----
  const int seg = (((n_sel + kWaves - 1) / kWaves) + 63) & ~63;
  const int j0 = wave * seg;
  const int j1 = min(n_sel, j0 + seg);
  int n_gt = 0, n_eq = 0;
  for (int jb = j0; jb < j1; jb += 64) {
    const int j = jb + lane;
    const bool in = j < j1;
    const uint32_t k = in ? keys[j] : 0u;
    n_gt += __popcll(__ballot(in && k > thr));
    n_eq += __popcll(__ballot(in && k == thr));
  }
  if (lane == 0) {
    cnt[wave][0] = n_gt;
    cnt[wave][1] = n_eq;
  }
  __syncthreads();
  int gt_before = 0, eq_before = 0;
  for (int w = 0; w < wave; ++w) {
    gt_before += cnt[w][0];
    eq_before += cnt[w][1];
  }
  int eq_run = eq_before;
  int kept_run = gt_before + min(eq_before, need_eq);
  const uint64_t lt_mask = (1ull << lane) - 1ull;
  for (int jb = j0; jb < j1; jb += 64) {
    const int j = jb + lane;
    const bool in = j < j1;
    const uint32_t k = in ? keys[j] : 0u;
    const bool is_gt = in && k > thr;
    const bool is_eq = in && k == thr;
    const uint64_t eq_ballot = __ballot(is_eq);
    const int eq_rank = eq_run + __popcll(eq_ballot & lt_mask);
    const bool keep = is_gt || (is_eq && eq_rank < need_eq);
    const uint64_t keep_ballot = __ballot(keep);
    if (keep) kept[kept_run + __popcll(keep_ballot & lt_mask)] = j;
    eq_run += __popcll(eq_ballot);
    kept_run += __popcll(keep_ballot);
  }
}

// ---------------------------------------------------------------------------
// SnapKV-style score with a pruned second pass
// ---------------------------------------------------------------------------
//
// The second pass over K only serves the selection, and the selection only
// needs exact column sums near its threshold.  The first pass can bound every
// column sum: it accumulates the soft-max numerators 2^(logit - ref_i) against a
// per-row reference ref_i that is known when the token is read (log2 of the
// row's sum over what the workgroup has read so far, renewed at fixed steps by
// all wavefronts together), so the exact weight of logit (i, j) is that
// numerator times rho_i = 2^(ref_i - lse_i) <= 1, a factor that is only known at
// the end but is the same for every token of an epoch.  With c_j the sum of a
// token's numerators e_ij over the window rows and s_j the root of the sum of
// their squares, for any number m
//     a_j = sum_i e_ij rho_i = m c_j + sum_i e_ij (rho_i - m),
// and because no e_ij is negative, with (x)+ = max(x, 0) and Cauchy-Schwarz,
//     a_j <= m c_j + s_j sqrt(sum_i ((rho_i - m)+)^2),
//     a_j >= m c_j - s_j sqrt(sum_i ((m - rho_i)+)^2).
// A few values of m around the mean of the rho_i are tried for
// each side (the least upper bound over all m is the exact maximum of a_j over
// all non-negative e_ij with these two sums), next to
// c_j min_i rho_i <= a_j <= c_j max_i rho_i.  Both numbers of a token
// share its word of the LDS score array until the pass ends (c_j in the leading
// 20 bits, s_j / c_j <= 1 in the other 12), so the bounds cost no memory traffic.
// After the pass: bounds of the max-pooled scores, a lower and an upper bound of
// the selection threshold from two histograms, and the tokens whose pooled
// interval contains neither are decided without a second look.  For the others
// the tokens of their pooling window that can carry the maximum are re-scored
// exactly, row by row (256 bytes each), and everything else keeps its upper
// bound: the plain selection that follows then returns exactly the set it
// would return from exact scores (a decided-out token stays below the
// threshold, a decided-in one above it, an undecided one carries its exact
// pooled score; ties can only occur among those).
//
// The scores themselves are not produced (callers that ask for them take the
// two-pass path).  A reference can be overtaken by more than the fp32 exponent
// range only by inputs far outside any attention layer; the numerators then
// overflow, the row's log-sum-exp is not finite, and the head falls back to
// the two-pass code.

static constexpr int kBoundCentres = 3;  // values of m tried per side

struct BoundEpoch {  // the factors rho_i of one epoch over the window rows
  float rmax, rmin;               // largest (widened), smallest (narrowed)
  float m_up[kBoundCentres];      // centres for the upper bound ...
  float p_up[kBoundCentres];      // ... and sqrt(sum ((rho_i - m)+)^2) for each (widened)
  float m_dn[kBoundCentres];      // the same for the lower bound, with (m - rho_i)+
  float p_dn[kBoundCentres];
};

struct BoundShared {
  float fin[64];                   // log2 of every row's soft-max denominator
  float pub[2][kWaves][64];        // the wavefronts' row sums at a renewal, absolute log2
  float ref[kBoundMaxEpochs][64];  // the reference of every epoch
  BoundEpoch stat[kBoundMaxEpochs];
};

struct BoundKeep {  // what survives into the selection's LDS
  int bad;          // a row's log-sum-exp is not finite: fall back
};

// A token's two sums during the pass, in one word: the leading 20 bits of the
// sum c of its numerators (truncated: at most 2^-11 below c) and, in 12 bits, a
// number k with sqrt(s2) <= k / 4095 * c, s2 the sum of their squares (the ratio
// is at most 1; where the squares left the fp32 range, or c is too small for
// them to be trusted, k = 4095 says just that).
__device__ __forceinline__ uint32_t pack_sums(float c, float s2) {
  const float r = sqrtf(s2) / c;  // not a number <= 1 when c is 0 or either sum overflowed
  const uint32_t k = (c >= 1.0e-12f && r <= 1.f) ? min(4095u, (uint32_t)(r * 4095.f) + 2u) : 4095u;
  return (__float_as_uint(c) & 0xFFFFF000u) | k;
}

// A token's bounds share one 32-bit word of LDS: the upper bound rounded up to
// its leading 16 bits, the lower bound rounded down to its leading 16 bits
// (both are non-negative floats).  0.8 % of slack against bounds that are tens
// of per cent apart.
__device__ __forceinline__ uint32_t pack_bounds(float lo, float hi) {
  const uint32_t h = (__float_as_uint(hi) + 0xFFFFu) >> 16;
  const uint32_t l = __float_as_uint(lo) >> 16;
  return (h << 16) | l;
}
__device__ __forceinline__ float upper_of(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }
__device__ __forceinline__ float lower_of(uint32_t w) { return __uint_as_float(w << 16); }

__device__ __forceinline__ int bound_epoch_of_token(int j) {
  return bound_epoch_of_step((j >> 4) / kWaves);
}

// First pass with bounds.  On return stage[j] holds the packed bounds of the
// column sum of every prefix token j and bs.fin the rows' log-sum-exps.  All
// threads of the workgroup call; ends with a barrier.
template <int D, int NT>
__device__ __forceinline__ void snapkv_bounds(const BatchParams& p, const ReqDesc& rd, int lh,
                                              const int32_t* old_ids, BoundShared& bs,
                                              BoundKeep& keep, float* stage,
                                              half8 (&qreg)[NT][D / 32]) {
  constexpr int KS = D / 32;
  const int layer = lh / p.n_heads;
  const int head = lh - layer * p.n_heads;
  const int L = rd.seq_len;
  const int W = rd.window;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c16 = lane & 15;
  const int q4 = lane >> 4;
  const size_t blk_stride = (size_t)2 * p.n_heads * 16 * D;
  const _Float16* kbase = p.kv + (size_t)layer * p.n_blocks * blk_stride +
                          (size_t)head * 16 * D + (size_t)c16 * D + q4 * 8;
  const float c = p.scale_log2e;
  const int nb = (L + 15) >> 4;
  const int n_prefix = L - W;
  const int n_unmasked = n_prefix >> 4;
  auto load_block = [&](int b, half8 (&k)[KS]) {
    const int blk = clamp_block(old_ids[b], p.n_blocks);
    const _Float16* kp = kbase + (size_t)blk * blk_stride;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) k[ks] = load_half8(kp + ks * 32);
  };

  float ref[NT], zacc[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    ref[nt] = 0.f;
    zacc[nt] = 0.f;
  }
  // the wavefront's row sums in absolute log2 units -> pub[buf]
  auto publish = [&](int buf) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      float zr = zacc[nt];
      zr += __shfl_xor(zr, 16);
      zr += __shfl_xor(zr, 32);
      if (q4 == 0) bs.pub[buf][wave][nt * 16 + c16] = zr > 0.f ? ref[nt] + log2f(zr) : -INFINITY;
    }
  };
  // log2 of the workgroup's row sum from the published shares; own = this wavefront's share
  auto merged = [&](int buf, int row, float& own) {
    float l[kWaves];
    float mx = -INFINITY;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      l[w] = bs.pub[buf][w][row];
      mx = fmaxf(mx, l[w]);
    }
    own = l[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) own = wave == w ? l[w] : own;
    if (mx == -INFINITY) return 0.f;  // nothing visible yet: any finite reference will do
    float zz = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) zz += __builtin_amdgcn_exp2f(l[w] - mx);
    return mx + log2f(zz);
  };

  const int T = (nb + kWaves - 1) / kWaves;  // steps; every wavefront walks all of them
  int epoch = 0, buf = 0;
  half8 kc[KS], kn[KS];
  if (wave < nb) load_block(wave, kc);
  for (int t = 0; t < T; ++t) {
    const int b = wave + kWaves * t;
    if (b + kWaves < nb) load_block(b + kWaves, kn);
    if (bound_renews_before(t)) {  // uniform over the workgroup
      publish(buf);
      __syncthreads();
      ++epoch;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const int row = nt * 16 + c16;
        float own;
        const float nr = merged(buf, row, own);
        zacc[nt] = (q4 == 0 && own > -INFINITY) ? __builtin_amdgcn_exp2f(own - nr) : 0.f;
        ref[nt] = nr;
        if (wave == 0 && q4 == 0) bs.ref[epoch][row] = nr;
      }
      buf ^= 1;  // the other buffer is written next: its readers passed a barrier since
    }
    if (b < nb) {  // uniform per wavefront
      float cs[4] = {0.f, 0.f, 0.f, 0.f}, ss[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(kc[ks], qreg[nt][ks], acc, 0, 0, 0);
        float tv[4];
        const bool row_ok = nt * 16 + c16 < W;  // padded rows carry no weight
#pragma unroll
        for (int r = 0; r < 4; ++r) tv[r] = row_ok ? acc[r] * c : -INFINITY;
        if (b >= n_unmasked) {
          const int limit = L - W + nt * 16 + c16;
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (b * 16 + q4 * 4 + r > limit) tv[r] = -INFINITY;
        }
        if (t == 0) {
          // no reference yet: the block's own row maximum (these tokens get the
          // trivial bounds, whatever they accumulate here)
          float bm = fmaxf(fmaxf(tv[0], tv[1]), fmaxf(tv[2], tv[3]));
          bm = fmaxf(bm, __shfl_xor(bm, 16));
          bm = fmaxf(bm, __shfl_xor(bm, 32));
          ref[nt] = bm == -INFINITY ? 0.f : bm;
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float e = __builtin_amdgcn_exp2f(tv[r] - ref[nt]);
          zacc[nt] += e;
          cs[r] += e;
          ss[r] = fmaf(e, e, ss[r]);
        }
      }
      // sums over the window rows (the lanes of a row of 16, after the tiles in
      // the lane); lane c16 < 4 of each row keeps those of token 4 q4 + c16
      float mc = 0.f, ms = 0.f;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float vc = row16_sum(cs[r]);
        const float vs = row16_sum(ss[r]);
        mc = c16 == r ? vc : mc;
        ms = c16 == r ? vs : ms;
      }
      const int tok = b * 16 + q4 * 4 + c16;
      if (c16 < 4 && tok < n_prefix) reinterpret_cast<uint32_t*>(stage)[tok] = pack_sums(mc, ms);
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) kc[ks] = kn[ks];
  }
  publish(buf);
  __syncthreads();
  if (threadIdx.x < 64) {
    const int row = threadIdx.x;
    float own;
    const float lse = merged(buf, row, own);
    bs.fin[row] = row < W ? lse : INFINITY;  // padded rows contribute exp2(-inf) = 0
    if (row < W && !(fabsf(lse) < 3.0e38f)) keep.bad = 1;
  }
  __syncthreads();
  // the factors of every epoch, rho_i = 2^(ref_i - lse_i) over the window rows
  // (one per lane): range, and for centres at the mean and half a standard
  // deviation to either side of it the one-sided deviations
  for (int e = 1 + wave; e <= epoch; e += kWaves) {
    const bool ok = lane < W;
    const float rho = ok ? __builtin_amdgcn_exp2f(bs.ref[e][lane] - bs.fin[lane]) : 0.f;
    float lo = ok ? rho : INFINITY, hi = rho, sum = rho;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      lo = fminf(lo, __shfl_xor(lo, o));
      hi = fmaxf(hi, __shfl_xor(hi, o));
      sum += __shfl_xor(sum, o);
    }
    const float mean = sum / (float)W;
    float var = ok ? (rho - mean) * (rho - mean) : 0.f;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) var += __shfl_xor(var, o);
    const float half_sd = 0.5f * sqrtf(var / (float)W);
    float m_up[kBoundCentres], m_dn[kBoundCentres], p_up[kBoundCentres], p_dn[kBoundCentres];
#pragma unroll
    for (int k = 0; k < kBoundCentres; ++k) {
      // (any centre gives a valid bound; none below zero, so that widening the sum widens the bound)
      m_up[k] = fmaxf(mean + (float)(k - 1) * half_sd, 0.f);
      m_dn[k] = fmaxf(mean - (float)(k - 1) * half_sd, 0.f);
      const float du = ok ? fmaxf(rho - m_up[k], 0.f) : 0.f;
      const float dd = ok ? fmaxf(m_dn[k] - rho, 0.f) : 0.f;
      p_up[k] = du * du;
      p_dn[k] = dd * dd;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
#pragma unroll
      for (int k = 0; k < kBoundCentres; ++k) {
        p_up[k] += __shfl_xor(p_up[k], o);
        p_dn[k] += __shfl_xor(p_dn[k], o);
      }
    }
    if (lane == 0) {
      // (margins far above the rounding of the numerators, the sums and the factors)
      BoundEpoch& st = bs.stat[e];
      st.rmax = hi * 1.0002f;
      st.rmin = lo * 0.9998f;
#pragma unroll
      for (int k = 0; k < kBoundCentres; ++k) {
        st.m_up[k] = m_up[k];
        st.m_dn[k] = m_dn[k];
        st.p_up[k] = sqrtf(p_up[k]) * 1.001f + 1.0e-6f * hi;
        st.p_dn[k] = sqrtf(p_dn[k]) * 1.001f + 1.0e-6f * hi;
      }
    }
  }
  __syncthreads();
  // per token: the two sums -> bounds, packed in place
  {
    const float trivial = (float)W;  // every row contributes at most 1
    for (int j = threadIdx.x; j < n_prefix; j += kThreads) {
      const int e = bound_epoch_of_token(j);
      const uint32_t w = reinterpret_cast<const uint32_t*>(stage)[j];
      const float c_lo = __uint_as_float(w & 0xFFFFF000u);
      float lo = 0.f, hi = trivial;
      if (e > 0 && c_lo < 3.0e38f) {  // (a sum that left the fp32 range says nothing)
        const BoundEpoch& st = bs.stat[e];
        const float c_hi = c_lo * 1.00049f + 1.0e-30f;  // what the truncation to 20 bits took, at most
        const float s_hi = (float)(w & 0xFFFu) * (1.f / 4095.f) * c_hi;
        float h = c_hi * st.rmax, l = c_lo * st.rmin;
#pragma unroll
        for (int k = 0; k < kBoundCentres; ++k) {
          h = fminf(h, (st.m_up[k] * c_hi + s_hi * st.p_up[k]) * 1.0002f);
          l = fmaxf(l, (st.m_dn[k] * c_lo - s_hi * st.p_dn[k]) * 0.9998f);
        }
        lo = fmaxf(l, 0.f);
        hi = fminf(h, trivial);
      }
      reinterpret_cast<uint32_t*>(stage)[j] = pack_bounds(lo, hi);
    }
  }
  __syncthreads();
}

// Exact column sums of the tokens named by need[] (one bit per prefix token),
// row by row -> stage[].  mrow: the rows' log-sum-exps as the second product
// leaves the rows in registers.
template <int D, int NT>
__device__ __forceinline__ void snapkv_rescore(const BatchParams& p, const ReqDesc& rd, int lh,
                                               const int32_t* old_ids, const uint32_t* need,
                                               float* stage, half8 (&qreg)[NT][D / 32],
                                               const float (&mrow)[NT][4]) {
  constexpr int KS = D / 32;
  const int layer = lh / p.n_heads;
  const int head = lh - layer * p.n_heads;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c16 = lane & 15;
  const int q4 = lane >> 4;
  const size_t blk_stride = (size_t)2 * p.n_heads * 16 * D;
  const _Float16* base = p.kv + (size_t)layer * p.n_blocks * blk_stride + (size_t)head * 16 * D + q4 * 8;
  const float c = p.scale_log2e;
  const int n_prefix = rd.seq_len - rd.window;
  const int n_words = (n_prefix + 31) >> 5;
  // Tiles of 16 named tokens (a wavefront walks its words of the bit map and
  // fills a tile across them), the rows of the next tile requested before this
  // one is multiplied.
  int w = wave - kWaves;
  uint32_t bits = 0u;
  auto next_tile = [&](int& tok) -> bool {  // uniform over the wavefront
    tok = -1;
    int filled = 0;
    while (filled < 16) {
      while (bits == 0u) {
        w += kWaves;
        if (w >= n_words) return filled > 0;
        bits = __builtin_amdgcn_readfirstlane(need[w]);
      }
#pragma unroll 1
      for (; filled < 16 && bits; ++filled) {
        const int pos = __ffs(bits) - 1;
        bits &= bits - 1;
        tok = c16 == filled ? (w << 5) + pos : tok;
      }
    }
    return true;
  };
  auto load_rows = [&](int tok, half8 (&k)[KS]) {
    // (a lane without a token reads the head's first row and drops the result)
    const int tk = max(tok, 0);
    const int blk = clamp_block(old_ids[tk >> 4], p.n_blocks);
    const _Float16* kp = base + (size_t)blk * blk_stride + (size_t)(tk & 15) * D;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) k[ks] = load_half8_nt(kp + ks * 32);
  };
  half8 kc[KS], kn[KS], kf[KS];
  int tok_c = -1, tok_n = -1, tok_f = -1;
  bool have = next_tile(tok_c);
  if (have) load_rows(tok_c, kc);
  bool have_n = have && next_tile(tok_n);
  if (have_n) load_rows(tok_n, kn);
  while (have) {
    const bool have_f = have_n && next_tile(tok_f);
    if (have_f) load_rows(tok_f, kf);
    float colsum = 0.f;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(qreg[nt][ks], kc[ks], acc, 0, 0, 0);
#pragma unroll
      for (int r = 0; r < 4; ++r) colsum += __builtin_amdgcn_exp2f(acc[r] * c - mrow[nt][r]);
    }
    colsum += __shfl_xor(colsum, 16);
    colsum += __shfl_xor(colsum, 32);
    if (q4 == 0 && tok_c >= 0) stage[tok_c] = colsum;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      kc[ks] = kn[ks];
      kn[ks] = kf[ks];
    }
    tok_c = tok_n;
    tok_n = tok_f;
    have = have_n;
    have_n = have_f;
  }
}

// Between the two: which prefix tokens need their exact column sum.  stage[]
// holds the packed bounds; need[] is set.
__device__ __forceinline__ void bound_classify(const ReqDesc& rd, const float* stage_f,
                                               uint32_t* need, SelectShared& sh) {
  const uint32_t* stage = reinterpret_cast<const uint32_t*>(stage_f);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n_sel = rd.seq_len - rd.window;
  const int k_sel = rd.budget - rd.window;
  const int h = rd.pool_kernel >> 1;
  float vmax = 0.f;
  for (int j = tid; j < n_sel; j += kThreads) vmax = fmaxf(vmax, upper_of(stage[j]));
  for (int j = tid; j < ((n_sel + 31) >> 5); j += kThreads) need[j] = 0u;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) vmax = fmaxf(vmax, __shfl_xor(vmax, o));
  if (lane == 0) sh.wmax[wave] = __float_as_uint(vmax);
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kWaves; ++w) vmax = fmaxf(vmax, __uint_as_float(sh.wmax[w]));
  if (k_sel <= 0 || k_sel >= n_sel) return;  // uniform: window only, or everything is kept
  auto pooled = [&](int j, float& plo, float& phi) {
    const int a = max(0, j - h), b = min(n_sel - 1, j + h);
    plo = 0.f;
    phi = 0.f;
    for (int k = a; k <= b; ++k) {
      const uint32_t w = stage[k];
      phi = fmaxf(phi, upper_of(w));
      plo = fmaxf(plo, lower_of(w));
    }
  };
  // thresholds: the buckets that hold the k_sel-th largest lower and the k_sel-th
  // largest upper bound (two histograms from one evaluation of the pooled bounds)
  int* hist_lo = sh.hist;
  int* hist_hi = reinterpret_cast<int*>(sh.cand);
  static_assert(kMaxCand >= kBuckets, "the candidate list doubles as the second histogram");
  // the bucket of the k_sel-th largest entry of a histogram -> sel[which]
  auto kth_bucket = [&](const int* hist, int which) {
    int own[kBuckets / kThreads];
    int sum = 0;
#pragma unroll
    for (int i = 0; i < kBuckets / kThreads; ++i) {
      own[i] = hist[tid * (kBuckets / kThreads) + i];
      sum += own[i];
    }
    int v = sum;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int t = __shfl_up(v, o);
      if (lane >= o) v += t;
    }
    if (lane == 63) sh.wsum[wave] = v;
    __syncthreads();
    int before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      if (w < wave) before += sh.wsum[w];
      total += sh.wsum[w];
    }
    int above = total - (v + before);  // entries in buckets above this thread's
#pragma unroll
    for (int i = kBuckets / kThreads - 1; i >= 0; --i) {
      if (above < k_sel && above + own[i] >= k_sel) sh.sel[which] = tid * (kBuckets / kThreads) + i;
      above += own[i];
    }
    __syncthreads();
  };
  // buckets of 2^shift keys from kmin upwards; what lies below kmin counts in bucket 0
  auto find_buckets = [&](uint32_t kmin, int shift) {
#pragma unroll
    for (int i = 0; i < kBuckets / kThreads; ++i) {
      hist_lo[tid + i * kThreads] = 0;
      hist_hi[tid + i * kThreads] = 0;
    }
    __syncthreads();
    for (int j = tid; j < n_sel; j += kThreads) {
      float plo, phi;
      pooled(j, plo, phi);
      const uint32_t klo = score_key(plo), khi = score_key(phi);
      // (no key exceeds the largest upper bound; the clamp keeps the index in range whatever the bounds hold)
      atomicAdd(&hist_lo[klo > kmin ? min((klo - kmin) >> shift, (uint32_t)kBuckets - 1u) : 0u], 1);
      atomicAdd(&hist_hi[khi > kmin ? min((khi - kmin) >> shift, (uint32_t)kBuckets - 1u) : 0u], 1);
    }
    __syncthreads();
    kth_bucket(hist_lo, 0);
    kth_bucket(hist_hi, 1);
  };
  // The bounds carry 16 significant bits, the whole range of keys from 0 to the
  // largest upper bound only fits 2048 buckets that are up to 12 % of a value
  // wide.  So first with buckets of 1.6 % (2^17 keys) over the 32 octaves below
  // the largest upper bound; should the k_sel-th largest lower bound lie below
  // all of that, once more over the whole range.
  const uint32_t kzero = score_key(0.f), kmax = score_key(vmax);
  const int coarse = kmax > kzero ? max(0, 32 - __clz(kmax - kzero) - kBucketBits) : 0;
  constexpr int kFine = 17;
  uint32_t kmin = kzero;
  int shift = coarse;
  if (coarse > kFine) {
    kmin = kmax - ((uint32_t)kBuckets << kFine) + 1u;
    shift = kFine;
  }
  find_buckets(kmin, shift);
  if (kmin != kzero && sh.sel[0] == 0) {  // uniform: read after a barrier
    __syncthreads();                      // (everyone has read sel before it is written again)
    kmin = kzero;
    shift = coarse;
    find_buckets(kmin, shift);
  }
  // (bucket 0 also holds what lies below kmin)
  const uint32_t t_lo = sh.sel[0] == 0 ? kzero : kmin + ((uint32_t)sh.sel[0] << shift);  // <= the threshold's key
  const uint32_t t_hi = kmin + (((uint32_t)sh.sel[1] + 1u) << shift) - 1u;                // >= the threshold's key
  for (int j = tid; j < n_sel; j += kThreads) {
    float plo, phi;
    pooled(j, plo, phi);
    if (score_key(phi) >= t_lo && score_key(plo) <= t_hi) {
      const int a = max(0, j - h), b = min(n_sel - 1, j + h);
      for (int k = a; k <= b; ++k)
        if (upper_of(stage[k]) >= plo) atomicOr(&need[k >> 5], 1u << (k & 31));
    }
  }
  __syncthreads();
}

__global__ __launch_bounds__(kThreads) void select_kernel(BatchParams p) {
  extern __shared__ uint32_t keys[];
  __shared__ SelectShared sh;
  const int n_lh = p.n_layers * p.n_heads;
  const int slot = blockIdx.x / n_lh;
  const int lh = blockIdx.x - slot * n_lh;
  const ReqDesc rd = p.descs[p.order_all[slot]];
  select_unit<false>(p, rd, lh, keys, sh);
}

// Streaming requests need no score: the first min(n_sink, budget) tokens and
// the most recent budget - sinks tokens are kept.
__device__ __forceinline__ void streaming_unit(const BatchParams& p, const ReqDesc& rd, int lh) {
  const int L = rd.seq_len;
  const int B = rd.budget;
  const int sinks = min(p.n_sink, B);
  const int first_recent = L - (B - sinks);
  int32_t* kept = p.kept + rd.kept_off + (size_t)lh * B;
  for (int t = threadIdx.x; t < B; t += kThreads)
    kept[t] = (t < sinks) ? t : first_recent + (t - sinks);
  if (p.scores_out) {
    float* out = p.scores_out + rd.score_off + (size_t)lh * L;
    for (int j = threadIdx.x; j < L; j += kThreads)
      out[j] = (j < sinks || j >= first_recent) ? INFINITY : 0.f;
  }
}

// ---------------------------------------------------------------------------
// gather / compact
// ---------------------------------------------------------------------------
//
// One workgroup per (request, layer, head); a wavefront fills one new block
// (16 output slots) at a time for K and V.  D/8 lanes move one row with
// 128-bit accesses, so a wavefront instruction moves 64/(D/8) rows; the
// destination chunk is contiguous.

template <int D>
__device__ __forceinline__ void gather_unit(const BatchParams& p, const ReqDesc& rd, int lh,
                                            const int32_t* old_ids) {
  constexpr int LPR = D / 8;
  constexpr int RPI = 64 / LPR;
  constexpr int NI = 16 / RPI;
  const int layer = lh / p.n_heads;
  const int head = lh - layer * p.n_heads;
  const int B = rd.budget;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // destination blocks: freshly popped ones, or the request's own first blocks
  const int32_t* new_ids = p.in_place ? old_ids : p.new_ids + rd.new_off;
  const int32_t* kept = p.kept + rd.kept_off + (size_t)lh * B;
  const size_t chunk = (size_t)16 * D;               // one (block, kv, head)
  const size_t v_off = (size_t)p.n_heads * chunk;    // K chunk -> V chunk of a block
  const size_t blk_stride = 2 * v_off;
  _Float16* base = p.kv + (size_t)layer * p.n_blocks * blk_stride + (size_t)head * chunk +
                   (lane % LPR) * 8;
  const int row_in_instr = lane / LPR;
  // In place, output t overwrites slot t while kept[t] >= t: a chunk of
  // kWaves*16 outputs only reads slots at or after its own start, so reading
  // the whole chunk, a barrier, then writing it never destroys a row that is
  // still needed (later chunks read strictly later slots).
  for (int c0 = 0; c0 < rd.n_new; c0 += kWaves) {
    const int nbk = c0 + wave;
    half8 kk[NI], vv[NI];
    bool ok[NI];
#pragma unroll
    for (int k = 0; k < NI; ++k) {
      const int row = k * RPI + row_in_instr;
      const int t = nbk * 16 + row;
      ok[k] = nbk < rd.n_new && t < B;
      if (ok[k]) {
        const int idx = min(max(kept[t], 0), rd.seq_len - 1);
        const int sblk = clamp_block(old_ids[idx >> 4], p.n_blocks);
        const _Float16* src = base + (size_t)sblk * blk_stride + (size_t)(idx & 15) * D;
        kk[k] = load_half8_nt(src);
        vv[k] = load_half8_nt(src + v_off);
      }
    }
    if (p.in_place) __syncthreads();  // uniform: c0 and in_place are the same for all threads
    if (nbk < rd.n_new) {
      const int dblk = clamp_block(new_ids[nbk], p.n_blocks);
      _Float16* dst = base + (size_t)dblk * blk_stride;
#pragma unroll
      for (int k = 0; k < NI; ++k) {
        if (ok[k]) {
          const int row = k * RPI + row_in_instr;
          store_half8_nt(dst + (size_t)row * D, kk[k]);
          store_half8_nt(dst + (size_t)row * D + v_off, vv[k]);
        }
      }
    }
  }
}

template <int D>
__global__ __launch_bounds__(kThreads) void gather_kernel(BatchParams p) {
  const int n_lh = p.n_layers * p.n_heads;
  const int slot = blockIdx.x / n_lh;
  const int lh = blockIdx.x - slot * n_lh;
  const ReqDesc rd = p.descs[p.order_all[slot]];
  gather_unit<D>(p, rd, lh, p.old_ids + rd.old_off);
}

// ---------------------------------------------------------------------------
// fused per-unit kernel: score -> select -> gather in one workgroup
// ---------------------------------------------------------------------------
//
// For heads whose scores fit the workgroup's LDS share the three steps run
// back to back in the workgroup that owns the (request, layer, head): the
// column sums (or key norms) go straight into LDS, the selection works on
// them in place and the copy follows.  The scores never travel through HBM,
// the stage is one launch per method, and the LDS/ALU-bound selection of one
// workgroup overlaps the HBM-bound streaming of the others on the same CU.
// One launch serves both methods (the unit's descriptor says which); NT =
// ceil(window / 16), or 0 when the launch holds no SnapKV unit.

template <int D, int NT>
__global__ __launch_bounds__(kThreads) void fused_unit_kernel(BatchParams p) {
  extern __shared__ uint32_t keys[];
  __shared__ union {
    ScoreShared score;
    SelectShared select;
  } sh;
  const int n_lh = p.n_layers * p.n_heads;
  const int slot = blockIdx.x / n_lh;
  const int lh = blockIdx.x - slot * n_lh;
  const ReqDesc rd = p.descs[p.order_fused[slot]];
  float* stage = reinterpret_cast<float*>(keys);
  // the request's block ids, read once per workgroup (every later use is an LDS read)
  __shared__ int32_t sm_ids[kFusedMaxLen / 16];
  const bool ids_in_lds = rd.n_old <= kFusedMaxLen / 16;  // streaming units may be longer
  if (ids_in_lds)
    for (int i = threadIdx.x; i < rd.n_old; i += kThreads)
      sm_ids[i] = clamp_block(p.old_ids[rd.old_off + i], p.n_blocks);
  __syncthreads();
  if (rd.method == 3 /* FC_METHOD_STREAMING */) {  // uniform per workgroup
    streaming_unit(p, rd, lh);
  } else {
    bool snap = false;
    if constexpr (NT > 0) snap = rd.method == 1 /* FC_METHOD_SNAPKV */;
    if (snap) {
      if constexpr (NT > 0)
        snapkv_unit<D, NT>(p, rd, lh, sm_ids, sh.score, [&](int j, float v) { stage[j] = v; });
    } else {
      knorm_unit<D>(p, rd, lh, sm_ids, [&](int j, float v) { stage[j] = v; });
    }
    __syncthreads();
    select_unit<true>(p, rd, lh, keys, sh.select);
  }
  __syncthreads();  // the kept list (global memory, this workgroup's own) is complete
  gather_unit<D>(p, rd, lh, ids_in_lds ? sm_ids : p.old_ids + rd.old_off);
}

// The fused kernel with the pruned second pass for its SnapKV units (see
// snapkv_bounds); key-norm and streaming units that ride in the launch run as in
// fused_unit_kernel.  Dynamic LDS: seq_len words of scores, then one bit per token.
template <int D, int NT>
__global__ __launch_bounds__(kThreads, 3) void fused_bounded_kernel(BatchParams p) {  // 3 wavefronts per SIMD
  extern __shared__ uint32_t keys[];
  __shared__ union {
    ScoreShared score;
    SelectShared select;
    BoundShared bound;
  } sh;
  __shared__ BoundKeep keep;
  const int n_lh = p.n_layers * p.n_heads;
  const int slot = blockIdx.x / n_lh;
  const int lh = blockIdx.x - slot * n_lh;
  const ReqDesc rd = p.descs[p.order_fused[slot]];
  float* stage = reinterpret_cast<float*>(keys);
  uint32_t* need = keys + ((rd.seq_len + 31) & ~31);
  __shared__ int32_t sm_ids[kFusedMaxLen / 16];
  const bool ids_in_lds = rd.n_old <= kFusedMaxLen / 16;  // streaming units may be longer
  if (ids_in_lds)
    for (int i = threadIdx.x; i < rd.n_old; i += kThreads)
      sm_ids[i] = clamp_block(p.old_ids[rd.old_off + i], p.n_blocks);
  if (threadIdx.x == 0) keep.bad = 0;
  __syncthreads();
  if (rd.method == 3 /* FC_METHOD_STREAMING */) {  // uniform per workgroup
    streaming_unit(p, rd, lh);
  } else {
    if (rd.method == 1 /* FC_METHOD_SNAPKV */) {
      constexpr int KS = D / 32;
      const int q4 = (threadIdx.x & 63) >> 4;
      half8 qreg[NT][KS];
      load_window_queries<D, NT>(p, rd, lh, qreg);
      // Short heads gain nothing (the tokens of the first step have no bounds,
      // those of the next few loose ones): they take the two passes.
      const bool prune = rd.seq_len >= kBoundMinLen;  // uniform
      if (prune) snapkv_bounds<D, NT>(p, rd, lh, sm_ids, sh.bound, keep, stage, qreg);
      if (!prune || keep.bad) {  // bad: not representable against a running reference
        snapkv_unit_q<D, NT>(p, rd, lh, sm_ids, sh.score, qreg, [&](int j, float v) { stage[j] = v; });
      } else {
        float mrow[NT][4];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int r = 0; r < 4; ++r) mrow[nt][r] = sh.bound.fin[nt * 16 + q4 * 4 + r];
        __syncthreads();  // the log-sum-exps are in registers: the selection's LDS may take over
        bound_classify(rd, stage, need, sh.select);
        __syncthreads();
        // every token not named keeps its upper bound as its value
        for (int j = threadIdx.x; j < rd.seq_len - rd.window; j += kThreads)
          if (!((need[j >> 5] >> (j & 31)) & 1u)) stage[j] = upper_of(keys[j]);
        snapkv_rescore<D, NT>(p, rd, lh, sm_ids, need, stage, qreg, mrow);
      }
    } else {
      knorm_unit<D>(p, rd, lh, sm_ids, [&](int j, float v) { stage[j] = v; });
    }
    __syncthreads();
    select_unit<true>(p, rd, lh, keys, sh.select);
  }
  __syncthreads();  // the kept list (global memory, this workgroup's own) is complete
  gather_unit<D>(p, rd, lh, ids_in_lds ? sm_ids : p.old_ids + rd.old_off);
}

// a fill kernel for small device arrays (flags, verdict words): calls may be
// captured into a graph, where a memset node is not wanted
__global__ void zero_ints_kernel(int32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------

hipError_t kernels_one_time_setup() {
  // the select kernel may need more than the default 64 KiB of dynamic LDS
  // (the fused kernel never does: kFusedMaxLen * 4 = 32 KiB)
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(select_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, 32768 * 4);
  return e;
}

hipError_t launch_stack_init(int32_t* stack, int n_blocks, hipStream_t s) {
  if (n_blocks <= 0) return hipSuccess;
  stack_init_kernel<<<(n_blocks + 255) / 256, 256, 0, s>>>(stack, n_blocks);
  return hipGetLastError();
}

hipError_t launch_pool_pop(const int32_t* stack, int top, int n, int32_t* out, int32_t* owner,
                           int n_blocks, int32_t* flag, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  pool_pop_kernel<<<(n + 255) / 256, 256, 0, s>>>(stack, top, n, out, owner, n_blocks, flag);
  return hipGetLastError();
}

hipError_t launch_pool_push(int32_t* stack, int top, int n, const int32_t* ids, int32_t* owner,
                            int n_blocks, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  pool_push_kernel<<<(n + 255) / 256, 256, 0, s>>>(stack, top, n, ids, owner, n_blocks);
  return hipGetLastError();
}

hipError_t launch_owner_init(int32_t* owner, const int32_t* stack, int top, int n_blocks,
                             hipStream_t s) {
  owner_fill_kernel<<<(n_blocks + 255) / 256, 256, 0, s>>>(owner, n_blocks, 1);
  if (top > 0) owner_mark_free_kernel<<<(top + 255) / 256, 256, 0, s>>>(owner, stack, top, n_blocks);
  return hipGetLastError();
}

hipError_t launch_owner_check_ids(const int32_t* ids, int n, int n_blocks, int32_t* owner,
                                  int32_t* word, bool revert, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  owner_check_ids_kernel<<<(n + 255) / 256, 256, 0, s>>>(ids, n, n_blocks, owner, word,
                                                         revert ? 1 : 0);
  return hipGetLastError();
}

hipError_t launch_owner_check_tables(const BatchParams& p, int32_t* word, bool revert,
                                     hipStream_t s) {
  if (p.n_comp <= 0) return hipSuccess;
  owner_check_tables_kernel<<<p.n_comp, kThreads, 0, s>>>(p, word, revert ? 1 : 0);
  return hipGetLastError();
}

hipError_t launch_meta_upload(const MetaChunk& c, char* dst, int n_bytes, hipStream_t s) {
  if (n_bytes <= 0) return hipSuccess;
  if (n_bytes > (int)sizeof(MetaChunk)) return hipErrorInvalidValue;
  meta_upload_kernel<<<1, 256, 0, s>>>(c, dst, n_bytes);
  return hipGetLastError();
}

hipError_t launch_plan_alloc(const BatchParams& p, hipStream_t s) {
  plan_alloc_kernel<<<p.n_comp, kThreads, 0, s>>>(p);
  return hipGetLastError();
}

hipError_t launch_reclaim(const BatchParams& p, hipStream_t s) {
  reclaim_kernel<<<p.n_comp, kThreads, 0, s>>>(p);
  return hipGetLastError();
}

template <int D>
static hipError_t launch_snapkv_d(const BatchParams& p, hipStream_t s) {
  const unsigned grid = (unsigned)p.n_snap * p.n_layers * p.n_heads;
  const int nt = (p.window + 15) / 16;
  switch (nt) {
    case 1: snapkv_score_kernel<D, 1><<<grid, kThreads, 0, s>>>(p); break;
    case 2: snapkv_score_kernel<D, 2><<<grid, kThreads, 0, s>>>(p); break;
    case 3: snapkv_score_kernel<D, 3><<<grid, kThreads, 0, s>>>(p); break;
    case 4: snapkv_score_kernel<D, 4><<<grid, kThreads, 0, s>>>(p); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_snapkv_score(const BatchParams& p, hipStream_t s) {
  if (p.n_snap == 0) return hipSuccess;
  if (p.head_dim == 128) return launch_snapkv_d<128>(p, s);
  if (p.head_dim == 64) return launch_snapkv_d<64>(p, s);
  return hipErrorInvalidValue;
}

hipError_t launch_knorm_score(const BatchParams& p, hipStream_t s) {
  if (p.n_knorm == 0) return hipSuccess;
  const unsigned grid = (unsigned)p.n_knorm * p.n_layers * p.n_heads;
  if (p.head_dim == 128)
    knorm_score_kernel<128><<<grid, kThreads, 0, s>>>(p);
  else if (p.head_dim == 64)
    knorm_score_kernel<64><<<grid, kThreads, 0, s>>>(p);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_select(const BatchParams& p, int max_seq_len, hipStream_t s) {
  const unsigned grid = (unsigned)p.n_unfused * p.n_layers * p.n_heads;
  const size_t lds = (size_t)max_seq_len * sizeof(uint32_t);
  select_kernel<<<grid, kThreads, lds, s>>>(p);
  return hipGetLastError();
}

template <int D>
static hipError_t launch_fused_d(const BatchParams& p, bool any_snap, size_t lds, hipStream_t s) {
  const unsigned grid = (unsigned)p.n_fused * p.n_layers * p.n_heads;
  if (any_snap && p.bounded) {
    switch ((p.window + 15) / 16) {
      case 1: fused_bounded_kernel<D, 1><<<grid, kThreads, lds, s>>>(p); break;
      case 2: fused_bounded_kernel<D, 2><<<grid, kThreads, lds, s>>>(p); break;
      case 3: fused_bounded_kernel<D, 3><<<grid, kThreads, lds, s>>>(p); break;
      case 4: fused_bounded_kernel<D, 4><<<grid, kThreads, lds, s>>>(p); break;
      default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
  }
  switch (any_snap ? (p.window + 15) / 16 : 0) {
    case 0: fused_unit_kernel<D, 0><<<grid, kThreads, lds, s>>>(p); break;
    case 1: fused_unit_kernel<D, 1><<<grid, kThreads, lds, s>>>(p); break;
    case 2: fused_unit_kernel<D, 2><<<grid, kThreads, lds, s>>>(p); break;
    case 3: fused_unit_kernel<D, 3><<<grid, kThreads, lds, s>>>(p); break;
    case 4: fused_unit_kernel<D, 4><<<grid, kThreads, lds, s>>>(p); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_fused(const BatchParams& p, bool any_snap, int max_seq_len, hipStream_t s) {
  if (p.n_fused == 0) return hipSuccess;
  // (with the pruned second pass: one bit per token behind the scores)
  const size_t lds = p.bounded && any_snap
                         ? ((size_t)((max_seq_len + 31) & ~31) + (size_t)((max_seq_len + 31) >> 5)) * sizeof(uint32_t)
                         : (size_t)max_seq_len * sizeof(uint32_t);
  if (p.head_dim == 128) return launch_fused_d<128>(p, any_snap, lds, s);
  if (p.head_dim == 64) return launch_fused_d<64>(p, any_snap, lds, s);
  return hipErrorInvalidValue;
}

hipError_t launch_gather(const BatchParams& p, hipStream_t s) {
  const unsigned grid = (unsigned)p.n_unfused * p.n_layers * p.n_heads;
  if (p.head_dim == 128)
    gather_kernel<128><<<grid, kThreads, 0, s>>>(p);
  else if (p.head_dim == 64)
    gather_kernel<64><<<grid, kThreads, 0, s>>>(p);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_zero_ints(int32_t* p, int n, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  zero_ints_kernel<<<(n + 255) / 256, 256, 0, s>>>(p, n);
  return hipGetLastError();
}

}  // namespace fc
