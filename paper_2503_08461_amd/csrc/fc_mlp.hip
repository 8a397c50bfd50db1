// Chunk-MLP compressor kernel for gfx950: every run of k consecutive tokens
// of one modality becomes one row, y = W2 . act(W1 . x + b1) + b2 (GELU, erf or tanh form).
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
//     pulls through a ring in LDS, and W2 (64 KiB) stays in LDS;
//   * the 32x32 result tile of the first product already has the chunk on the
//     lane, which is what the B operand of the second product needs; only the
//     order of the contraction index differs, and that is folded into the
//     pre-permutation of W2.  The hidden activations therefore never leave
//     registers.
// A workgroup handles tiles of 256 rows (row = (layer, head, K|V) x chunk of
// one request and one modality), NT column tiles of 32 rows per wavefront; the kernel
// is persistent (one workgroup per CU walks the tile list) so that W2 is loaded
// into LDS once per modality change rather than once per tile.

#include "fc_device.h"

#include <math.h>

namespace fc {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));

static constexpr int kMlpRowsPerTile = 256;
static constexpr uint32_t kNoRow = 0xffffffffu;  // "no such token" in the table of pool rows
// threads of a workgroup when a wavefront takes NT column tiles of 32 chunks
constexpr int mlp_threads(int nt) { return kMlpRowsPerTile / (32 * nt) * 64; }

int mlp_rows_per_tile(int) { return kMlpRowsPerTile; }
int mlp_workgroups_per_cu() { return 1; }

// hidden unit that sits at contraction position (slab sl, lane half kh, element e)
// of the second product, given how the first product leaves its result in
// registers (32x32 tile: register 4g + r of lane half kh holds row 8g + 4kh + r)
__host__ __device__ constexpr int mlp_hidden_unit(int sl, int kh, int e) {
  return 32 * (sl / 2) + 16 * (sl % 2) + 8 * (e / 4) + 4 * kh + (e % 4);
}

// Output channel (within a 32-channel tile) that sits on row rho of the second
// product's A operand.  The 32x32 result leaves rows 8g + 4kh + r (g = 0..3,
// r = 0..3) in registers 4g + r of lane half kh; with this order a lane's
// registers of g = 2gp and 2gp + 1 are 8 consecutive channels, one 16-byte store.
__host__ __device__ constexpr int mlp_out_channel(int rho) {
  return 16 * (rho / 16) + 8 * ((rho / 4) % 2) + 4 * ((rho / 8) % 2) + rho % 4;
}

size_t mlp_w1p_elems(int head_dim, int hidden, int k) { return (size_t)hidden * k * head_dim; }
size_t mlp_w2p_elems(int head_dim, int hidden) { return (size_t)hidden * head_dim; }

// Contraction position (slab s = t*SPT + j, lane half kh, element e) of the
// first product is channel 16*j + 8*kh + e of token t of the chunk: the two
// lane halves read neighbouring 16-byte pieces of a row.
// w1p[s][mt][lane][e] = w1[mt*32 + lane%32][t*D + 16*j + 8*(lane/32) + e]
// w2p[sl][ot][lane][e] = w2[ot*32 + mlp_out_channel(lane%32)][mlp_hidden_unit(sl, lane/32, e)]
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
    w1p[i] = w1[(size_t)(mt * 32 + (lane & 31)) * kd + t * head_dim + 16 * j + 8 * (lane >> 5) +
                e];
  }
  if (i < n2) {
    const int e = i & 7, lane = (i >> 3) & 63;
    const size_t rest = i >> 9;
    const int mt2 = head_dim / 32;
    const int ot = rest % mt2, sl = rest / mt2;
    w2p[i] = w2[(size_t)(ot * 32 + mlp_out_channel(lane & 31)) * hidden +
                mlp_hidden_unit(sl, lane >> 5, e)];
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
// written as v / (1 + exp(-2u)) = v / (1 + exp2(v * (A + B v^2))) with the
// constants folded (A = -2 log2(e) sqrt(2/pi), B = 0.044715 A): one exp2, one
// reciprocal and five other operations per value
__device__ __forceinline__ float gelu_tanh(float v) {
  const float e = __builtin_amdgcn_exp2f(v * fmaf(v * v, -0.10294324f, -2.3022082f));
  return v * __builtin_amdgcn_rcpf(1.0f + e);
}

// GELU by its definition, v * Phi(v), Phi the standard normal distribution
// function.  Phi(-|v|) = exp2(P(|v|)) with P a polynomial of degree 6: log2 of
// the normal tail is smooth (about -x^2 / 2 ln 2 - log2 x for large x), and a
// fit of P that minimises the largest error of v * Phi(v) over |v| <= 9 leaves
// 1.4e-7 absolute in exact arithmetic, 3e-7 evaluated in fp32 (as accurate as
// the usual five-term rational approximation of erfc, at one transcendental
// instead of two and no division).  Past |v| = 8.5 nothing is left of the tail
// (Phi(-8.5) = 1e-17) and the polynomial is not followed further.
// GELU(v) = v Phi(-|v|) for v < 0, v - v Phi(-|v|) otherwise, i.e. max(v, 0) - |v| Phi(-|v|).
#define FC_GELU_TAIL_P0 -9.999973123e-01f
#define FC_GELU_TAIL_P1 -1.151156811e+00f
#define FC_GELU_TAIL_P2 -4.588952346e-01f
#define FC_GELU_TAIL_P3 -5.326704516e-02f
#define FC_GELU_TAIL_P4 7.999533677e-03f
#define FC_GELU_TAIL_P5 -7.477810617e-04f
#define FC_GELU_TAIL_P6 3.095778387e-05f
#define FC_GELU_TAIL_CLAMP 8.5f
__device__ __forceinline__ float gelu_erf(float v) {
  const float a = fminf(fabsf(v), FC_GELU_TAIL_CLAMP);
  float p = fmaf(a, FC_GELU_TAIL_P6, FC_GELU_TAIL_P5);
  p = fmaf(a, p, FC_GELU_TAIL_P4);
  p = fmaf(a, p, FC_GELU_TAIL_P3);
  p = fmaf(a, p, FC_GELU_TAIL_P2);
  p = fmaf(a, p, FC_GELU_TAIL_P1);
  p = fmaf(a, p, FC_GELU_TAIL_P0);
  // max(v, 0) - |v| Phi(-|v|): v - v Phi(-|v|) for v >= 0, v Phi(-|v|) below
  return fmaf(-fabsf(v), __builtin_amdgcn_exp2f(p), fmaxf(v, 0.f));
}

template <int ACT>
__device__ __forceinline__ float mlp_activation(float v) {
  return ACT == 0 ? gelu_erf(v) : gelu_tanh(v);
}

// what the lanes of a chunk read for the tokens its segment does not have
__device__ __align__(256) _Float16 g_zero_row[128];

template <int D, int HID, int NT, int ACT>
__global__ __launch_bounds__(mlp_threads(NT), 1) void mlp_compress_kernel(BatchParams p,
                                                                      MlpParams mp) {
  constexpr int MT1 = HID / 32;               // 32-row tiles of hidden units
  constexpr int MT2 = D / 32;                 // 32-row tiles of output channels
  constexpr int S2 = HID / 16;                // K slabs of the second product
  constexpr int SPT = D / 16;                 // K slabs of the first product per token
  constexpr int GPT = 4;                      // W1 groups per token
  constexpr int GS = SPT / GPT;               // K slabs per group
  constexpr int GO = GS * MT1;                // A operands (W1 tiles) per group
  constexpr int kMlpThreads = mlp_threads(NT);  // NT column tiles (32 chunks each) per wavefront
  constexpr int PPG = GO * 64 / kMlpThreads;  // 16-byte pieces of a W1 group per thread
  constexpr int AR = 4;                       // A operands in flight from LDS
  constexpr int XR = NT == 1 ? 2 : 1;         // tokens of B operands held in registers
  constexpr int WD = 2;                       // W1 groups in flight in registers (4 measured slower)
  constexpr int RT = 8 + XR;                  // rows of the per-lane token table
  static_assert(GO % AR == 0 && PPG >= 1, "tiling");
  extern __shared__ __align__(16) unsigned char smem[];
  // the W1 ring comes first so that every read of it is one base register
  // plus an immediate offset (the offset field holds less than 64 KB)
  half8* sm_w1 = reinterpret_cast<half8*>(smem);                     // [GPT groups][GO][64]
  half8* sm_w2 = sm_w1 + GPT * GO * 64;                              // [S2][MT2][64]
  float* sm_b1 = reinterpret_cast<float*>(sm_w2 + S2 * MT2 * 64);    // [HID]
  float* sm_b2 = sm_b1 + HID;                                        // [D]
  uint32_t* sm_rows = reinterpret_cast<uint32_t*>(sm_b2 + D);        // [RT][NT][threads]

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int col = lane & 31;  // chunk within a 32-wide column tile
  const int kh = lane >> 5;   // which 8 of the slab's 16 contraction positions
  const int k = mp.k;
  const int n_units = p.n_layers * p.n_heads * 2;
  const size_t chunk_el = (size_t)16 * D;
  const size_t v_off = (size_t)p.n_heads * chunk_el;
  const size_t blk_stride = 2 * v_off;
  const int blk_rows = 2 * p.n_heads * 16;  // blk_stride in rows of D elements

  // Persistent: a workgroup walks tiles blockIdx.x, blockIdx.x + gridDim.x, ...
  // The walk is software-pipelined over tiles, because what a tile needs before
  // its first MFMA (which job it belongs to, where its chunks start, the block
  // ids of its rows, its first pool rows) is a chain of dependent memory
  // accesses of several microseconds: while tile T runs its GELU, second
  // product and store, in which nothing else is loaded, the chain of tile
  // T + gridDim.x is walked, so that its first rows are on their way when it
  // starts.
  struct Lane {            // what a lane knows about its chunk of a tile (per column tile)
    int row;               // row of the job (-1: no chunk)
    int s0, n_valid;       // first token of the chunk, tokens it has (< k at a segment's end)
    uint32_t base_row;     // pool row (units of D elements) of slot 0 of block 0 of its (layer, head, K|V)
  };
  auto find_job = [&](int tile, int& ji) {  // jobs are sorted by tile_start; ji only moves up
    while (ji + 1 < mp.n_jobs && mp.jobs[ji + 1].tile_start <= tile) ++ji;
  };
  auto lane_of = [&](int tile, const MlpJob& job, const ReqDesc& rd, int nt) -> Lane {
    Lane ln;
    const long long n_rows = (long long)n_units * job.chunks;
    const long long row = (long long)(tile - job.tile_start) * kMlpRowsPerTile +
                          wave * (32 * NT) + nt * 32 + col;
    ln.row = row < n_rows ? (int)row : -1;
    int unit = 0;
    ln.s0 = 0;
    ln.n_valid = 0;
    if (row < n_rows) {
      unit = (int)(row / job.chunks);
      const int cl = (int)(row - (long long)unit * job.chunks);
      int seg_end;
      if (job.modality == 1) {
        ln.s0 = rd.img_begin + cl * k;
        seg_end = rd.img_end;
      } else if (cl < rd.chunks_text0) {
        ln.s0 = cl * k;
        seg_end = rd.img_begin;
      } else {
        ln.s0 = rd.img_end + (cl - rd.chunks_text0) * k;
        seg_end = rd.seq_len;
      }
      ln.n_valid = min(k, seg_end - ln.s0);
    }
    const int lh = unit >> 1;
    const int layer = lh / p.n_heads;
    // (the pool has fewer than 2^32 - 1 rows: checked by the launcher)
    ln.base_row = (uint32_t)(layer * p.n_blocks) * (uint32_t)blk_rows +
                  (uint32_t)((unit & 1) * (p.n_heads * 16) + (lh - layer * p.n_heads) * 16);
    return ln;
  };
  // The pool rows of a chunk's tokens (absolute, in units of D elements,
  // kNoRow = no such token) go to a table in LDS, each lane reading back only what it wrote: registers
  // are needed for data in flight, and a lookup inside the pipelined loop would
  // make every iteration wait for all loads in flight.  A chunk has at most 8
  // tokens, so it lies in at most two blocks: bid[0], bid[1].
  auto write_rows = [&](const Lane& ln, const int (&bid)[2], int nt) {
#pragma unroll
    for (int t = 0; t < RT; ++t) {
      const int tok = ln.s0 + t;
      const int blk = (tok >> 4) == (ln.s0 >> 4) ? bid[0] : bid[1];
      sm_rows[(t * NT + nt) * kMlpThreads + tid] =
          t < ln.n_valid ? ln.base_row + (uint32_t)clamp_block(blk, p.n_blocks) * (uint32_t)blk_rows +
                               (uint32_t)(tok & 15)
                         : kNoRow;
    }
  };
  auto row_of = [&](int nt, int t) -> uint32_t {
    return sm_rows[(t * NT + nt) * kMlpThreads + tid];
  };

  // Every load of the pipelined loop is unconditional (a load under a branch
  // makes the compiler wait for ALL loads in flight at the next use): a token
  // that does not exist (past the end of a chunk's segment, or a lane without
  // a chunk) reads a row of zeros instead, and W1 groups past the end wrap to
  // group 0, whose copy nobody uses.
  // B operand of slab j of a token: 8 channels [(D/2)kh + 8j, +8) of its row
  auto load_x = [&](uint32_t ri, int j) -> half8 {
    const _Float16* row = ri != kNoRow ? p.kv + (size_t)ri * D : g_zero_row;
    return load_half8(row + kh * 8 + j * 16);
  };

  int cur_m = -1;
  int ji = 0;
  find_job(blockIdx.x, ji);
  MlpJob job = mp.jobs[ji];
  ReqDesc rd = p.descs[job.desc];
  half8 xq[XR][NT][SPT];
  // the first tile's chain, not overlapped with anything
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const Lane ln = lane_of(blockIdx.x, job, rd, nt);
    const int32_t* ids = p.old_ids + rd.old_off;
    const int last = ln.s0 + max(ln.n_valid, 1) - 1;
    const int bid[2] = {ids[ln.s0 >> 4], ids[last >> 4]};
    write_rows(ln, bid, nt);
  }
#pragma unroll
  for (int u = 0; u < XR; ++u)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const uint32_t ri = row_of(nt, u);
#pragma unroll
      for (int j = 0; j < SPT; ++j) xq[u][nt][j] = load_x(ri, j);
    }

  for (int tile = blockIdx.x; tile < mp.n_tiles; tile += gridDim.x) {
    // the tile after this one (the last tile prefetches itself again: loads in
    // bounds that nobody uses, so that nothing here sits under a branch)
    const int tile_n = tile + (int)gridDim.x < mp.n_tiles ? tile + (int)gridDim.x : tile;
    int ji_n = ji;
    find_job(tile_n, ji_n);
    const MlpJob job_n = mp.jobs[ji_n];
    const ReqDesc rd_n = p.descs[job_n.desc];

    // weights of this modality: W2 and the biases stay in LDS across tiles and
    // are only reloaded when the modality changes
    const int m = job.modality;
    if (m != cur_m) {  // uniform
      __syncthreads();  // the previous tile may still be reading them
      const half8* w2g = reinterpret_cast<const half8*>(mp.w2p[m]);
      for (int i = tid; i < S2 * MT2 * 64; i += kMlpThreads) sm_w2[i] = w2g[i];
      for (int i = tid; i < HID; i += kMlpThreads) sm_b1[i] = mp.b1[m][i];
      for (int i = tid; i < D; i += kMlpThreads) sm_b2[i] = mp.b2[m][i];
      cur_m = m;
    }
    const half8* w1g = reinterpret_cast<const half8*>(mp.w1p[m]);  // [S1][MT1][64]
    // piece i of this thread's share of W1 group g (operand order, contiguous)
    auto load_w = [&](int g, int i) -> half8 {
      return w1g[(size_t)(g < k * GPT ? g : 0) * GO * 64 + i * kMlpThreads + tid];
    };

    // ---- first product: H^T tile [HID x 32 NT] per wavefront -----------------
    // Each W1 operand read from LDS feeds NT MFMAs (one per column tile).
    // Latency is hidden by software pipelining: W1 moves through registers
    // (two groups in flight) into a ring of GPT groups in LDS, one barrier per
    // group; a group is visible one barrier before its turn, so A operands are
    // read AR ahead of their use, across group boundaries.  A scattered pool
    // row takes microseconds to arrive (address translation, HBM) and loads
    // complete in order, so every load waits for the slowest one before it:
    // the B operands of XR tokens are held, and those of a finished group are
    // replaced at once by the same slabs XR tokens on.
    floatx16 acc[MT1][NT];
#pragma unroll
    for (int mt = 0; mt < MT1; ++mt)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0.f;
    half8 wq[WD][PPG], ar[AR];
    // groups 0 and 1 go straight to LDS; wq[i] holds the next unwritten group congruent to i mod WD
#pragma unroll
    for (int g = 0; g < 2; ++g)
#pragma unroll
      for (int i = 0; i < PPG; ++i) sm_w1[g * GO * 64 + i * kMlpThreads + tid] = load_w(g, i);
#pragma unroll
    for (int g = 0; g < WD; ++g)
#pragma unroll
      for (int i = 0; i < PPG; ++i) wq[(2 + g) % WD][i] = load_w(2 + g, i);
    __syncthreads();  // W2, biases and groups 0, 1 of W1 are in LDS
#pragma unroll
    for (int n = 0; n < AR; ++n) ar[n] = sm_w1[n * 64 + lane];
    for (int t0 = 0; t0 < k; t0 += XR) {
#pragma unroll
    for (int u = 0; u < XR; ++u) {
      const int t = t0 + u;
      if (t >= k) break;  // uniform
      uint32_t ri_new[NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) ri_new[nt] = row_of(nt, t + XR);
#pragma unroll
      for (int jj = 0; jj < GPT; ++jj) {
        // group 4t+jj+2 into the ring slot that group 4t+jj-2 left, then refill those registers
        half8* w1n = sm_w1 + ((jj + 2) % GPT) * GO * 64;
#pragma unroll
        for (int i = 0; i < PPG; ++i) {
          w1n[i * kMlpThreads + tid] = wq[(GPT * u + jj + 2) % WD][i];
          wq[(GPT * u + jj + 2) % WD][i] = load_w(GPT * t + jj + 2 + WD, i);
        }
        const half8* w1s = sm_w1 + jj * GO * 64;
        const half8* w1f = sm_w1 + ((jj + 1) % GPT) * GO * 64;  // visible since the last barrier
#pragma unroll
        for (int n = 0; n < GO; ++n) {
          const half8 a = ar[n % AR];
          const int nn = n + AR;
          ar[n % AR] = (nn < GO) ? w1s[nn * 64 + lane] : w1f[(nn - GO) * 64 + lane];
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
            acc[n % MT1][nt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
                a, xq[u][nt][GS * jj + n / MT1], acc[n % MT1][nt], 0, 0, 0);
          // pin the issue order "one LDS read, NT MFMAs": left alone, the
          // scheduler sinks each read to just before its use
          __builtin_amdgcn_sched_barrier(0);
        }
        // this group's B operands are done: fetch the same slabs XR tokens on
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int h = 0; h < GS; ++h)
            xq[u][nt][GS * jj + h] = load_x(ri_new[nt], GS * jj + h);
        __syncthreads();  // the new group is visible; nobody reads this one any more
      }
    }
    }

    // ---- the next tile's chain, first half: where its chunks are, their block ids
    Lane ln_n[NT];
    int bid_n[NT][2];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      ln_n[nt] = lane_of(tile_n, job_n, rd_n, nt);
      const int32_t* ids = p.old_ids + rd_n.old_off;
      const int last = ln_n[nt].s0 + max(ln_n[nt].n_valid, 1) - 1;
      bid_n[nt][0] = ids[ln_n[nt].s0 >> 4];
      bid_n[nt][1] = ids[last >> 4];
    }

    // ---- bias, gelu, fp16: each 32x32 result tile becomes two B operands of
    // the second product and stays in registers.  Half-way through, when half
    // of the accumulators are gone, the next tile's row table is written (this
    // tile's is no longer read, and every lane only ever reads its own entries)
    // and its first XR tokens are requested: they travel while the rest of the
    // GELU, the second product and the store keep the other units busy.
    half8 hb[S2][NT];
    auto gelu_tile = [&](int mt) {
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const int sl = 2 * mt + half;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const int u = mlp_hidden_unit(sl, kh, e);  // = 32mt + 16half + 8(e/4) + 4kh + e%4
            hb[sl][nt][e] = (_Float16)mlp_activation<ACT>(acc[mt][nt][8 * half + e] + sm_b1[u]);
          }
      }
    };
#pragma unroll
    for (int mt = 0; mt < MT1 / 2; ++mt) gelu_tile(mt);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) write_rows(ln_n[nt], bid_n[nt], nt);
#pragma unroll
    for (int u = 0; u < XR; ++u)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const uint32_t ri = row_of(nt, u);
#pragma unroll
        for (int j = 0; j < SPT; ++j) xq[u][nt][j] = load_x(ri, j);
      }
#pragma unroll
    for (int mt = MT1 / 2; mt < MT1; ++mt) gelu_tile(mt);

    // ---- second product, Y^T tile [D x 32 NT]
    floatx16 acc2[MT2][NT];
#pragma unroll
    for (int ot = 0; ot < MT2; ++ot)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc2[ot][nt][r] = 0.f;
#pragma unroll
    for (int sl = 0; sl < S2; ++sl)
#pragma unroll
      for (int ot = 0; ot < MT2; ++ot) {
        const half8 w = sm_w2[(sl * MT2 + ot) * 64 + lane];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          acc2[ot][nt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(w, hb[sl][nt], acc2[ot][nt], 0, 0, 0);
      }

    // ---- bias, fp16, store the rows into the request's new blocks -------------
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      // (this tile's row again: cheaper than a register held across the loops)
      const long long row_ll = (long long)(tile - job.tile_start) * kMlpRowsPerTile +
                               wave * (32 * NT) + nt * 32 + col;
      if (row_ll < (long long)n_units * job.chunks) {
        const int row = (int)row_ll;
        const int unit = row / job.chunks;
        const int cl = row - unit * job.chunks;
        const int o = (m == 1) ? rd.chunks_text0 + cl
                               : (cl < rd.chunks_text0 ? cl : rd.chunks_image + cl);
        const int lh = unit >> 1;
        const int layer = lh / p.n_heads;
        const int nblk = clamp_block(p.new_ids[rd.new_off + (o >> 4)], p.n_blocks);
        _Float16* dst = p.kv + (size_t)layer * p.n_blocks * blk_stride +
                        (size_t)nblk * blk_stride + (unit & 1) * v_off +
                        (size_t)(lh - layer * p.n_heads) * chunk_el + (size_t)(o & 15) * D;
#pragma unroll
        for (int ot = 0; ot < MT2; ++ot)
#pragma unroll
          for (int gp = 0; gp < 2; ++gp) {
            // registers 8gp .. 8gp+7 = rows 16gp + 4kh + {0..3} and 16gp + 8 + 4kh + {0..3}
            // = channels 16gp + 8kh + {0..7} (mlp_out_channel)
            const int c0 = 32 * ot + 16 * gp + 8 * kh;
            half8 y;
#pragma unroll
            for (int r = 0; r < 8; ++r) y[r] = (_Float16)(acc2[ot][nt][8 * gp + r] + sm_b2[c0 + r]);
            store_half8(dst + c0, y);
          }
      }
    }
    job = job_n;
    rd = rd_n;
    ji = ji_n;
  }
}

template <int D, int HID, int NT>
static size_t mlp_lds_bytes() {
  return (size_t)(HID / 16) * (D / 32) * 64 * 16 + (size_t)(D / 16) * (HID / 32) * 64 * 16 +
         (size_t)(HID + D) * sizeof(float) + (size_t)(8 + 2) * NT * mlp_threads(NT) * sizeof(int);
}

// Column tiles per wavefront: with a hidden width of 256 one column tile
// already needs 128 accumulator registers, so a wavefront takes one (eight
// wavefronts, two per SIMD, 256 registers each); with 128 it takes two (four
// wavefronts).  Two tiles at width 256 (four wavefronts with 512 registers)
// measured slower: nothing covers the stalls of a lone wavefront on its SIMD.
template <int D, int HID>
constexpr int mlp_nt() { return (D / 64) * (HID / 32) * 64 >= 512 ? 1 : 2; }

template <int D, int HID>
static hipError_t mlp_setup_one() {
  constexpr int NT = mlp_nt<D, HID>();
  hipError_t e = hipFuncSetAttribute(
      reinterpret_cast<const void*>(mlp_compress_kernel<D, HID, NT, 0>),
      hipFuncAttributeMaxDynamicSharedMemorySize, (int)mlp_lds_bytes<D, HID, NT>());
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(mlp_compress_kernel<D, HID, NT, 1>),
                            hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)mlp_lds_bytes<D, HID, NT>());
  return e;
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
  constexpr int NT = mlp_nt<D, HID>();
  const unsigned grid = (unsigned)std::min(mp.n_tiles, mp.max_grid);
  if (mp.activation == 0)
    mlp_compress_kernel<D, HID, NT, 0><<<grid, mlp_threads(NT), mlp_lds_bytes<D, HID, NT>(), s>>>(
        p, mp);
  else
    mlp_compress_kernel<D, HID, NT, 1><<<grid, mlp_threads(NT), mlp_lds_bytes<D, HID, NT>(), s>>>(
        p, mp);
  return hipGetLastError();
}

hipError_t launch_mlp_compress(const BatchParams& p, const MlpParams& mp, hipStream_t s) {
  if (mp.n_tiles <= 0) return hipSuccess;
  // the kernel addresses pool rows (head_dim elements each) with 32 bits
  if ((unsigned long long)p.n_layers * p.n_blocks * 2 * p.n_heads * 16 >= kNoRow)
    return hipErrorInvalidValue;
  if (p.head_dim == 128 && mp.hidden == 256) return mlp_launch_one<128, 256>(p, mp, s);
  if (p.head_dim == 128 && mp.hidden == 128) return mlp_launch_one<128, 128>(p, mp, s);
  if (p.head_dim == 64 && mp.hidden == 256) return mlp_launch_one<64, 256>(p, mp, s);
  if (p.head_dim == 64 && mp.hidden == 128) return mlp_launch_one<64, 128>(p, mp, s);
  return hipErrorInvalidValue;
}

}  // namespace fc
