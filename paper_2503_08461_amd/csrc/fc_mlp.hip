// Chunk-MLP compressor kernel for gfx950: every run of k consecutive tokens
// of one modality becomes one row, y = W2 . gelu(W1 . x + b1) + b2 (tanh GELU).
//
// This is the one dense contraction of the library that is MFMA-bound
// (about 390 kflop per 1.3 KB chunk at k = 5, d = 128, hidden = 256), so it is
// laid out around v_mfma_f32_32x32x16_f16 in the TRANSPOSED form
//     H^T [hidden x chunks] = W1 [hidden x k*d] . X^T [k*d x chunks]
//     Y^T [d x chunks]      = W2 [d x hidden]   . H^T
// with chunks on the MFMA column (lane) axis:
//   * the B operand of the first product (lane = chunk, 8 consecutive channels
//     of one token row) is a 16-byte load straight from the scattered pool
//     block, no staging;
//   * the A operand (weights) is pre-permuted once into operand order, so a
//     16-wide K slab of W1 is one contiguous 8 KiB piece that the workgroup
//     double-buffers through LDS, and W2 (64 KiB) stays in LDS;
//   * the 32x32 result tile of the first product already has the chunk on the
//     lane, which is what the B operand of the second product needs; only the
//     order of the contraction index differs, and that is folded into the
//     pre-permutation of W2.  The hidden activations therefore never leave
//     registers.
// A workgroup of 8 wavefronts handles 256 rows (row = (layer, head, K|V) x
// chunk of one request and one modality), 32 per wavefront.

#include "fc_device.h"

#include <math.h>

namespace fc {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));

static constexpr int kMlpThreads = 512;
static constexpr int kMlpRowsPerTile = 256;

// hidden unit that sits at contraction position (slab sl, lane half kh, element e)
// of the second product, given how the first product leaves its result in
// registers (32x32 tile: register 4g + r of lane half kh holds row 8g + 4kh + r)
__host__ __device__ constexpr int mlp_hidden_unit(int sl, int kh, int e) {
  return 32 * (sl / 2) + 16 * (sl % 2) + 8 * (e / 4) + 4 * kh + (e % 4);
}

size_t mlp_w1p_elems(int head_dim, int hidden, int k) { return (size_t)hidden * k * head_dim; }
size_t mlp_w2p_elems(int head_dim, int hidden) { return (size_t)hidden * head_dim; }

// Contraction position (slab s = t*SPT + j, lane half kh, element e) of the
// first product is channel (D/2)*kh + 8*j + e of token t of the chunk: each
// lane half owns one contiguous half row (128 B at D = 128), so a lane's loads
// for one token fall into a single cache line.
// w1p[s][mt][lane][e] = w1[mt*32 + lane%32][t*D + (D/2)*(lane/32) + 8*j + e]
// w2p[sl][ot][lane][e] = w2[ot*32 + lane%32][mlp_hidden_unit(sl, lane/32, e)]
__global__ void mlp_permute_kernel(const _Float16* w1, const _Float16* w2, _Float16* w1p,
                                   _Float16* w2p, int head_dim, int hidden, int k) {
  const int kd = k * head_dim;
  const size_t n1 = (size_t)hidden * kd, n2 = (size_t)hidden * head_dim;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n1) {
    const int e = i & 7, lane = (i >> 3) & 63;
    const size_t rest = i >> 9;
    const int mt1 = hidden / 32;
    const int mt = rest % mt1, s = rest / mt1;
    const int spt = head_dim / 16;
    const int t = s / spt, j = s - t * spt;
    w1p[i] = w1[(size_t)(mt * 32 + (lane & 31)) * kd + t * head_dim + (head_dim / 2) * (lane >> 5) +
                8 * j + e];
  }
  if (i < n2) {
    const int e = i & 7, lane = (i >> 3) & 63;
    const size_t rest = i >> 9;
    const int mt2 = head_dim / 32;
    const int ot = rest % mt2, sl = rest / mt2;
    w2p[i] = w2[(size_t)(ot * 32 + (lane & 31)) * hidden + mlp_hidden_unit(sl, lane >> 5, e)];
  }
}

hipError_t launch_mlp_permute_weights(const _Float16* w1, const _Float16* w2, _Float16* w1p,
                                      _Float16* w2p, int head_dim, int hidden, int k,
                                      hipStream_t s) {
  const size_t n = std::max(mlp_w1p_elems(head_dim, hidden, k), mlp_w2p_elems(head_dim, hidden));
  mlp_permute_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(w1, w2, w1p, w2p, head_dim,
                                                                 hidden, k);
  return hipGetLastError();
}

// tanh form of GELU, v/2 * (1 + tanh(u)) with u = sqrt(2/pi) * (v + 0.044715 v^3),
// written as v / (1 + exp(-2u)): one exp2 and one reciprocal per value (the
// erf form costs about 40 VALU instructions per value, more than the MFMAs)
__device__ __forceinline__ float gelu_tanh(float v) {
  const float u = 0.7978845608028654f * (v + 0.044715f * v * v * v);
  const float e = __builtin_amdgcn_exp2f(-2.8853900817779268f * u);  // exp(-2u)
  return v * __builtin_amdgcn_rcpf(1.0f + e);
}

template <int D, int HID>
__global__ __launch_bounds__(kMlpThreads) void mlp_compress_kernel(BatchParams p, MlpParams mp) {
  constexpr int MT1 = HID / 32;  // 32-row tiles of hidden units
  constexpr int MT2 = D / 32;    // 32-row tiles of output channels
  constexpr int S2 = HID / 16;   // K slabs of the second product
  constexpr int SPT = D / 16;    // K slabs of the first product per token
  extern __shared__ __align__(16) unsigned char smem[];
  half8* sm_w2 = reinterpret_cast<half8*>(smem);                       // [S2][MT2][64]
  half8* sm_w1 = sm_w2 + S2 * MT2 * 64;                                // [2][kMlpThreads]
  float* sm_b1 = reinterpret_cast<float*>(sm_w1 + 2 * kMlpThreads);    // [HID]
  float* sm_b2 = sm_b1 + HID;                                          // [D]

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int col = lane & 31;  // chunk within the wavefront's 32
  const int kh = lane >> 5;   // which 8 of the slab's 16 contraction positions

  // which job does this tile belong to (jobs are sorted by tile_start)
  int lo = 0, hi = mp.n_jobs - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (mp.jobs[mid].tile_start <= (int)blockIdx.x) lo = mid; else hi = mid - 1;
  }
  const MlpJob job = mp.jobs[lo];
  const ReqDesc rd = p.descs[job.desc];
  const int m = job.modality;
  const int n_units = p.n_layers * p.n_heads * 2;
  const long long n_rows = (long long)n_units * job.chunks;
  const long long row = (long long)((int)blockIdx.x - job.tile_start) * kMlpRowsPerTile +
                        wave * 32 + col;
  const bool valid = row < n_rows;
  const int k = mp.k;
  const int S1 = k * SPT;

  // weights of this modality: W2 and the biases stay in LDS for the whole tile
  {
    const half8* w2g = reinterpret_cast<const half8*>(mp.w2p[m]);
    for (int i = tid; i < S2 * MT2 * 64; i += kMlpThreads) sm_w2[i] = w2g[i];
    for (int i = tid; i < HID; i += kMlpThreads) sm_b1[i] = mp.b1[m][i];
    for (int i = tid; i < D; i += kMlpThreads) sm_b2[i] = mp.b2[m][i];
  }
  const half8* w1g = reinterpret_cast<const half8*>(mp.w1p[m]);  // [S1][MT1][64]
  sm_w1[tid] = w1g[tid % (MT1 * 64)];                               // slab 0

  // this lane's chunk
  int unit = 0, o = 0, s0 = 0, n_valid = 0;
  if (valid) {
    unit = (int)(row / job.chunks);
    const int cl = (int)(row - (long long)unit * job.chunks);
    int seg_end;
    if (m == 1) {
      o = rd.chunks_text0 + cl;
      s0 = rd.img_begin + cl * k;
      seg_end = rd.img_end;
    } else if (cl < rd.chunks_text0) {
      o = cl;
      s0 = cl * k;
      seg_end = rd.img_begin;
    } else {
      o = rd.chunks_text0 + rd.chunks_image + (cl - rd.chunks_text0);
      s0 = rd.img_end + (cl - rd.chunks_text0) * k;
      seg_end = rd.seq_len;
    }
    n_valid = min(k, seg_end - s0);
  }
  const int kvsel = unit & 1;
  const int lh = unit >> 1;
  const int layer = lh / p.n_heads;
  const int head = lh - layer * p.n_heads;
  const size_t chunk_el = (size_t)16 * D;
  const size_t v_off = (size_t)p.n_heads * chunk_el;
  const size_t blk_stride = 2 * v_off;
  const _Float16* src_base = p.kv + (size_t)layer * p.n_blocks * blk_stride + kvsel * v_off +
                             (size_t)head * chunk_el + kh * (D / 2);
  const int32_t* old_ids = p.old_ids + rd.old_off;
  // where the chunk's token rows start, looked up once (a lookup inside the
  // pipelined loop would make every iteration wait for all loads in flight)
  long long row_off[8];
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    row_off[t] = -1;
    if (t < n_valid) {
      const int tok = s0 + t;
      const int blk = clamp_block(old_ids[tok >> 4], p.n_blocks);
      row_off[t] = (long long)blk * (long long)blk_stride + (long long)(tok & 15) * D;
    }
  }

  // Every load of the pipelined loop is unconditional (a load under a branch
  // makes the compiler wait for ALL loads in flight at the next use): rows that
  // do not exist read row 0 of the slice and are zeroed by a select, and W1
  // indices past the end wrap to valid ones whose data nobody uses.
  // B operand of slab j of a token: 8 channels [(D/2)kh + 8j, +8) of that token's row
  auto load_x = [&](long long off, int j) -> half8 {
    const half8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
    const half8 x = load_half8(src_base + (off >= 0 ? off : 0) + j * 8);
    return off >= 0 ? x : zero;
  };
  // this thread's 16 bytes of W1 slab s (operand order)
  const int w_tid = tid % (MT1 * 64);
  auto load_w = [&](int s) -> half8 {
    return w1g[(size_t)(s < S1 ? s : 0) * MT1 * 64 + w_tid];
  };

  // ---- first product: H^T tile [HID x 32] per wavefront ---------------------
  // Software pipeline: the B operands of the whole next token are requested in
  // one burst (8 loads of a lane hit one cache line, which is then fetched once)
  // while the current token is multiplied; the W1 pieces of the next kWDepth
  // slabs are in flight in registers; W1 goes through a two-slab LDS ring.
  constexpr int kWDepth = 4;
  floatx16 acc[MT1];
#pragma unroll
  for (int mt = 0; mt < MT1; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[mt][r] = 0.f;
  half8 xq[2][SPT], wq[kWDepth];
#pragma unroll
  for (int j = 0; j < SPT; ++j) xq[0][j] = load_x(row_off[0], j);
#pragma unroll
  for (int j = 0; j < kWDepth; ++j)
    wq[j] = load_w(j == 0 ? kWDepth : j);  // wq[j]: next unwritten slab congruent to j
  __syncthreads();  // W2, biases and slab 0 of W1 are in LDS
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    if (t >= k) break;  // uniform
    const long long next_off = (t + 1 < 8) ? row_off[(t + 1) & 7] : -1;
#pragma unroll
    for (int j = 0; j < SPT; ++j) xq[(t + 1) & 1][j] = load_x(next_off, j);
#pragma unroll
    for (int j = 0; j < SPT; ++j) {
      const int s = t * SPT + j;
      const half8* w1s = sm_w1 + (s & 1) * kMlpThreads;
      const half8 x = xq[t & 1][j];
#pragma unroll
      for (int mt = 0; mt < MT1; ++mt)
        acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(w1s[mt * 64 + lane], x, acc[mt], 0, 0, 0);
      // slab s+1 into the other half of the ring, then refill that register
      const int jn = (s + 1) % kWDepth;
      sm_w1[((s + 1) & 1) * kMlpThreads + tid] = wq[jn];
      wq[jn] = load_w(s + 1 + kWDepth);
      __syncthreads();  // next slab visible; this slab's half may be overwritten next time
    }
  }

  // ---- bias, gelu, fp16: each result tile becomes two B operands of the second
  // product, Y^T tile [D x 32], and is consumed at once (keeps registers down)
  floatx16 acc2[MT2];
#pragma unroll
  for (int ot = 0; ot < MT2; ++ot)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc2[ot][r] = 0.f;
#pragma unroll
  for (int mt = 0; mt < MT1; ++mt) {
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int sl = 2 * mt + half;
      half8 hb;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int u = mlp_hidden_unit(sl, kh, e);  // = 32mt + 16half + 8(e/4) + 4kh + e%4
        hb[e] = (_Float16)gelu_tanh(acc[mt][8 * half + e] + sm_b1[u]);
      }
#pragma unroll
      for (int ot = 0; ot < MT2; ++ot)
        acc2[ot] = __builtin_amdgcn_mfma_f32_32x32x16_f16(sm_w2[(sl * MT2 + ot) * 64 + lane], hb,
                                                          acc2[ot], 0, 0, 0);
    }
  }

  // ---- bias, fp16, store the row into the request's new blocks ---------------
  if (valid) {
    const int nblk = clamp_block(p.new_ids[rd.new_off + (o >> 4)], p.n_blocks);
    _Float16* dst = p.kv + (size_t)layer * p.n_blocks * blk_stride + (size_t)nblk * blk_stride +
                    kvsel * v_off + (size_t)head * chunk_el + (size_t)(o & 15) * D;
#pragma unroll
    for (int ot = 0; ot < MT2; ++ot)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int c0 = 32 * ot + 8 * g + 4 * kh;
        half4 y;
#pragma unroll
        for (int r = 0; r < 4; ++r) y[r] = (_Float16)(acc2[ot][4 * g + r] + sm_b2[c0 + r]);
        *reinterpret_cast<half4*>(dst + c0) = y;
      }
  }
}

template <int D, int HID>
static size_t mlp_lds_bytes() {
  return (size_t)(HID / 16) * (D / 32) * 64 * 16 + (size_t)2 * kMlpThreads * 16 +
         (size_t)(HID + D) * sizeof(float);
}

template <int D, int HID>
static hipError_t mlp_setup_one() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(mlp_compress_kernel<D, HID>),
                             hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)mlp_lds_bytes<D, HID>());
}

hipError_t mlp_one_time_setup() {
  hipError_t e = mlp_setup_one<128, 256>();
  if (e == hipSuccess) e = mlp_setup_one<128, 128>();
  if (e == hipSuccess) e = mlp_setup_one<64, 256>();
  if (e == hipSuccess) e = mlp_setup_one<64, 128>();
  return e;
}

template <int D, int HID>
static hipError_t mlp_launch_one(const BatchParams& p, const MlpParams& mp, hipStream_t s) {
  mlp_compress_kernel<D, HID><<<mp.n_tiles, kMlpThreads, mlp_lds_bytes<D, HID>(), s>>>(p, mp);
  return hipGetLastError();
}

hipError_t launch_mlp_compress(const BatchParams& p, const MlpParams& mp, hipStream_t s) {
  if (mp.n_tiles <= 0) return hipSuccess;
  if (p.head_dim == 128 && mp.hidden == 256) return mlp_launch_one<128, 256>(p, mp, s);
  if (p.head_dim == 128 && mp.hidden == 128) return mlp_launch_one<128, 128>(p, mp, s);
  if (p.head_dim == 64 && mp.hidden == 256) return mlp_launch_one<64, 256>(p, mp, s);
  if (p.head_dim == 64 && mp.hidden == 128) return mlp_launch_one<64, 128>(p, mp, s);
  return hipErrorInvalidValue;
}

}  // namespace fc
