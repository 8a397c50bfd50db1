// One-pass SnapKV-style score kernel for gfx950: the keys of a (layer, head)
// are read from HBM once.
//
// The row softmax needs every logit of a row before any column sum can be
// finished, so something has to stay on the chip between the pass that finds
// the row normalisers and the pass that forms the column sums.  Here it is K
// itself: a head is split along its tokens over a TEAM of G workgroups, small
// enough slices that every wavefront keeps its blocks (16 tokens, 4 KiB at
// d = 128) in registers, in MFMA operand layout.  Per head a workgroup
//   1. runs Q_win.K^T over its slice and reduces a (max, sum-of-exp) pair per
//      window row,
//   2. publishes its 64 pairs, collects those of the other G-1 members and
//      combines them into the row's log-sum-exp,
//   3. runs Q_win.K^T again from the registers and writes the un-pooled column
//      sums (4 bytes per token) to the score scratch.
// Max-pooling, selection and compaction follow in select_gather_kernel.
//
// Latency, not bandwidth, decides such a kernel, so it is software-pipelined
// and role-split.  Wavefronts 1..3 of a workgroup compute; they request the
// next head's blocks right after step 1 of this head, so HBM loads are in
// flight during step 2 and 3.  Loads of a wavefront return in order, which
// would put every poll of step 2 behind those HBM loads; wavefront 0 therefore
// holds no keys and does the exchange (and moves the window queries of the
// head after next into LDS, from where the compute wavefronts take their MFMA
// operands: a 16 KiB query tile per wavefront would not fit next to two sets
// of key registers).
//
// The exchange uses no fences (an agent-scope release writes back the whole
// L2; measured at 7-10 us per round against 2-2.6 us without): every datum is
// one relaxed 64-bit atomic store, agent scope, that carries its own tag
//     [ max: fp32 | sum: upper 24 bits of a positive fp32 | tag: 8 bits ]
// and readers poll the data until the tag is the current round's.  Two
// buffers alternate; a member can overwrite its round r entry (in round r+2)
// only after every member has published round r+1, which each does after it
// has read round r.  The sum loses 7 mantissa bits (relative 2^-17), far
// inside the 2e-3 tolerance of the scores.
//
// A waiting workgroup needs its partners to be running: the kernel is
// persistent and launched cooperatively (grid = what the device holds at once,
// team = consecutive workgroups in XCD-major order, so a team sits on one XCD
// and shares the queries and the exchange lines through that XCD's L2).
// Every wait is bounded: when it runs out the error flag is raised and the
// workgroup carries on with what it has, so every wavefront exits.
//
// Measured on MI355X (config-4 batch, per head and workgroup): step 1 takes
// 3.9 us, the exchange 5.5 us (a poll alone costs 3.3 us: the CU's vector
// memory path is one queue, and the polls stand behind the 60 KB of keys that
// the compute wavefronts have just requested), step 3 2.4 us.  That is
// 2.6 TB/s of key traffic, slower than reading K twice at full bandwidth; the
// two-pass kernels stay the default.

#include "fc_device.h"

#include <float.h>

namespace fc {

static constexpr int kSplitWaves = 3;  // compute wavefronts per workgroup (wavefront 0 communicates)
static constexpr int kSplitNBW = 5;    // blocks a compute wavefront holds
static constexpr int kSplitCap = kSplitWaves * kSplitNBW;  // blocks per workgroup per head
static constexpr int kSplitPollBatch = 32;
static constexpr int kSplitMaxSpins = 1 << 17;  // x (batch of L2 reads + sleep): a few tenths of a second

__host__ __device__ constexpr int split_capacity_blocks() { return kSplitCap; }

__device__ __forceinline__ uint64_t pack_stat(float m, float z, uint32_t tag) {
  // z >= 0: bits 30..7 of its fp32 pattern, rounded to nearest
  const uint32_t zb = (__float_as_uint(z) + 0x40u) >> 7;
  return ((uint64_t)__float_as_uint(m) << 32) | ((uint64_t)(zb & 0xFFFFFFu) << 8) | tag;
}
__device__ __forceinline__ float stat_max(uint64_t v) { return __uint_as_float((uint32_t)(v >> 32)); }
__device__ __forceinline__ float stat_sum(uint64_t v) {
  return __uint_as_float(((uint32_t)(v >> 8) & 0xFFFFFFu) << 7);
}

template <int D, int NT>
__global__ __launch_bounds__(kThreads, 2) void snapkv_split_kernel(BatchParams p) {
  constexpr int KS = D / 32;
  constexpr int NBW = kSplitNBW;
  constexpr int QN = NT * KS * 64;  // half8 entries of one query tile in operand order
  const int G = p.split_team;
  const int n_lh = p.n_layers * p.n_heads;
  static_assert(kWaves == kSplitWaves + 1, "one communication and kSplitWaves compute wavefronts");
  // XCD-major position of this workgroup (workgroup b runs on XCD b % 8)
  const int wpx = gridDim.x >> 3;
  const int pos = __builtin_amdgcn_readfirstlane((blockIdx.x & 7) * wpx + (blockIdx.x >> 3));
  const int n_teams = gridDim.x / G;
  const int team = pos / G;
  const int rank = pos - team * G;
  const int n_units = p.n_split * n_lh;
  if (team >= n_teams || team >= n_units) return;  // whole workgroup, before any barrier

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c16 = lane & 15;
  const int q4 = lane >> 4;
  const float c = p.scale_log2e;
  const size_t blk_stride = (size_t)2 * p.n_heads * 16 * D;

  __shared__ half8 sm_q[3][QN];
  __shared__ float sm_part[kSplitWaves][2][64];
  __shared__ float sm_fin[64];

  // what a wavefront needs to know about unit u = (request slot, layer-head)
  struct Unit {
    int rs, L, W, lh, nb, b0, b1, n_unmasked, n_prefix, old_off;
    int64_t q_off, raw_off;
  };
  // (every field is forced into scalar registers: the compiler does not see
  // that the descriptor index is the same for all lanes, and per-lane copies
  // would turn each use into a vector load that waits for all loads in flight)
  auto sgpr = [](int v) { return __builtin_amdgcn_readfirstlane(v); };
  auto sgpr64 = [&](int64_t v) {
    return (int64_t)(((uint64_t)(uint32_t)sgpr((int)(v >> 32)) << 32) | (uint32_t)sgpr((int)v));
  };
  auto unit_of = [&](int u) {
    const int rs = sgpr(u / n_lh);
    const ReqDesc& rd = p.descs[sgpr(p.order_split[rs])];
    Unit t;
    t.rs = rs;
    t.L = sgpr(rd.seq_len);
    t.W = sgpr(rd.window);
    t.lh = sgpr(u - rs * n_lh);
    t.nb = (t.L + 15) >> 4;
    const int bpw = (t.nb + G - 1) / G;  // <= kSplitCap, checked by the host
    t.b0 = min(t.nb, rank * bpw);
    t.b1 = min(t.nb, t.b0 + bpw);
    t.n_prefix = t.L - t.W;
    t.n_unmasked = t.n_prefix >> 4;
    t.old_off = sgpr(rd.old_off);
    t.q_off = sgpr64(rd.q_off);
    t.raw_off = sgpr64(rd.raw_off);
    return t;
  };
  // The unit `step` units after t.  A team's consecutive units mostly belong to
  // one request, and then only the layer-head changes: the descriptor (two
  // dependent scalar loads, a microsecond each when they miss) is re-read only
  // at a request boundary.
  auto unit_after = [&](const Unit& t, int step) {
    const int lh = t.lh + step;
    if (lh < n_lh) {
      Unit r = t;
      r.lh = lh;
      return r;
    }
    return unit_of(t.rs * n_lh + lh);
  };
  // window queries of a unit -> LDS in MFMA operand order (wavefront 0)
  auto move_queries = [&](const Unit& t, int buf) {
    const _Float16* qbase = p.q_window + t.q_off + (size_t)t.lh * t.W * D;
    half8 v[NT * KS];
#pragma unroll
    for (int e = 0; e < NT * KS; ++e) {
      const int row = (e / KS) * 16 + c16;
      const half8 z = {0, 0, 0, 0, 0, 0, 0, 0};
      v[e] = row < t.W ? load_half8(qbase + (size_t)row * D + (e % KS) * 32 + q4 * 8) : z;
    }
#pragma unroll
    for (int e = 0; e < NT * KS; ++e) sm_q[buf][e * 64 + lane] = v[e];
  };
  // Touches every 128-byte line of a unit's window queries so that they sit in
  // L2 when move_queries comes for them one unit later: wavefront 0 has one
  // in-order load queue for this and for the exchange, so nothing in it may
  // take an HBM round trip at the time the exchange starts.
  auto warm_queries = [&](const Unit& t) {
    const char* qb = reinterpret_cast<const char*>(p.q_window + t.q_off + (size_t)t.lh * t.W * D);
    const int bytes = t.W * D * 2;
    int sink = 0;
#pragma unroll
    for (int k = 0; k < (NT * 16 * D * 2) / (64 * 128); ++k) {
      const int off = (k * 64 + lane) * 128;
      if (off < bytes) sink += *reinterpret_cast<const volatile int*>(qb + off);
    }
    return sink;
  };
  // compute wavefront cw owns blocks b0 + cw + kSplitWaves * i, i < NBW
  const int cw = wave - 1;
  auto block_of = [&](const Unit& t, int i) { return t.b0 + cw + kSplitWaves * i; };
  // lane i < NBW: id of block i (0 if none).  Nothing may look at the value
  // here: it is requested behind the key loads of the unit before, and a use
  // would wait for all of them.  request_blocks clamps it.
  auto load_ids = [&](const Unit& t) {
    const int b = min(block_of(t, lane), t.b1 - 1);
    return p.old_ids[t.old_off + max(b, 0)];
  };
  // Keys travel as whole 1 KiB pieces (64 lanes x 16 contiguous bytes, which
  // the address unit takes at full rate; the MFMA operand pattern, 16 bytes
  // from each of 64 places, costs it a cycle per lane and made it the busiest
  // unit of the CU) and are turned into operand layout through a small LDS tile
  // of the wavefront's own, one block at a time, once they have landed.
  constexpr int LPR = D / 8;     // lanes per token row
  constexpr int RPI = 64 / LPR;  // rows per load instruction; 16 / RPI == KS instructions per block
  constexpr int PITCH = D * 2 + 16;  // bytes per tile row: rows 16 bytes apart in the banks
  __shared__ __attribute__((aligned(16))) char sm_tile[kSplitWaves][16 * PITCH];
  auto key_base = [&](const Unit& t) {
    const int layer = t.lh / p.n_heads;
    const int head = t.lh - layer * p.n_heads;
    return p.kv + (size_t)layer * p.n_blocks * blk_stride + (size_t)head * 16 * D + lane * 8;
  };

  half8 land[NBW][KS];  // blocks of the unit about to be scored (in flight or landed)
  half8 hold[NBW][KS];  // blocks of the unit being scored, kept for its second pass
  // Every slot is loaded and multiplied whether the wavefront has a block for
  // it or not (branches around the register tiles cost far more in copies than
  // the work they save); a slot without a block reads the pool's first chunk,
  // which stays in L2, and its logits are masked out.
  const _Float16* const spare = p.kv + lane * 8;
  auto request_blocks = [&](const Unit& t, int ids) {
    const _Float16* kb = key_base(t);
#pragma unroll
    for (int i = 0; i < NBW; ++i) {
      const _Float16* kp =
          block_of(t, i) < t.b1
              ? kb + (size_t)clamp_block(__builtin_amdgcn_readlane(ids, i), p.n_blocks) * blk_stride
              : spare;
#pragma unroll
      for (int j = 0; j < KS; ++j) land[i][j] = load_half8(kp + j * 512);
    }
  };
  // landed blocks, piece layout -> MFMA operand layout (lane: token lane % 16,
  // channels 32 ks + 8 (lane / 16) .. + 8), in place
  auto to_operand_layout = [&]() {
    char* tile = sm_tile[cw];
    const int wr = (lane / LPR) * PITCH + (lane % LPR) * 16;
    const int rd = c16 * PITCH + q4 * 16;
#pragma unroll
    for (int i = 0; i < NBW; ++i) {
#pragma unroll
      for (int j = 0; j < KS; ++j)
        *reinterpret_cast<half8*>(tile + wr + j * RPI * PITCH) = land[i][j];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        land[i][ks] = *reinterpret_cast<const half8*>(tile + rd + ks * 64);
    }
  };

  // this workgroup's (max, sum) of a row, from its compute wavefronts' partials
  auto workgroup_stat = [&](int row, float& mm, float& zz) {
    mm = -3.0e38f;
    zz = 0.f;
#pragma unroll
    for (int w = 0; w < kSplitWaves; ++w) mm = fmaxf(mm, sm_part[w][0][row]);
#pragma unroll
    for (int w = 0; w < kSplitWaves; ++w)
      zz += sm_part[w][1][row] * __builtin_amdgcn_exp2f(sm_part[w][0][row] - mm);
  };

  // The two roles run their own loops (so that neither carries the other's
  // registers) and meet at two barriers per unit:
  //   A  the workgroup's partial row statistics are in LDS
  //   B  the rows' log-sum-exps are in LDS
  // Query buffer n % 3 serves unit n; wavefront 0 refills it, two units ahead,
  // after barrier B of unit n - 1, when its last reader (pass 2 of unit n - 3)
  // is long done.
  if (wave == 0) {
    // ======================= communication wavefront =========================
    int u = team;
    int warm_sink = 0;
    Unit cur = unit_of(u);
    Unit ahead = cur;  // the unit whose queries are moved next (two after cur)
    move_queries(cur, 0);
    if (u + n_teams < n_units) {
      ahead = unit_after(ahead, n_teams);
      move_queries(ahead, 1);
    }
    if (u + 2 * n_teams < n_units) {
      ahead = unit_after(ahead, n_teams);
      warm_sink += warm_queries(ahead);
    }
    __syncthreads();  // prologue
    bool gave_up = false;  // a wait ran out: no further waiting, the results are void anyway
    for (int n = 0; u < n_units; ++n, u += n_teams) {
      const int W = cur.W;
      const uint32_t tag = 1u + (uint32_t)((n + 1) % 255);
      uint64_t* xbuf = p.split_xchg + (size_t)((n + 1) & 1) * gridDim.x * 64;
      __syncthreads();  // A
      // collect the team's pairs (this workgroup's own are published by its
      // first compute wavefront: a store in this wavefront's queue would have
      // to be acknowledged before the first poll could be looked at)
      const int row = lane;
      float gm = -3.0e38f, gz = 0.f;
      if (G == 1) {
        workgroup_stat(row, gm, gz);
      } else {
        const uint64_t* tb = xbuf + (size_t)team * G * 64 + row;
        for (int j0 = 0; j0 < G; j0 += kSplitPollBatch) {
          uint64_t v[kSplitPollBatch];
#pragma unroll
          for (int j = 0; j < kSplitPollBatch; ++j) v[j] = 0;
          uint32_t pending = G - j0 >= 32 ? 0xFFFFFFFFu : (1u << (G - j0)) - 1u;
          int spins = 0;
          while (pending && !gave_up) {
#pragma unroll
            for (int j = 0; j < kSplitPollBatch; ++j)
              if (pending & (1u << j))  // uniform
                v[j] = __hip_atomic_load(tb + (size_t)(j0 + j) * 64, __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int j = 0; j < kSplitPollBatch; ++j)
              if ((pending & (1u << j)) && __all((uint32_t)(v[j] & 0xFFu) == tag))
                pending &= ~(1u << j);
            if (pending) {
              if (++spins > kSplitMaxSpins) {
                __hip_atomic_fetch_or(p.error_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                gave_up = true;
                break;
              }
              __builtin_amdgcn_s_sleep(1);
            }
          }
          float bm = gm;
#pragma unroll
          for (int j = 0; j < kSplitPollBatch; ++j)
            if (j0 + j < G) bm = fmaxf(bm, stat_max(v[j]));
          gz *= __builtin_amdgcn_exp2f(gm - bm);
#pragma unroll
          for (int j = 0; j < kSplitPollBatch; ++j)
            if (j0 + j < G) gz += stat_sum(v[j]) * __builtin_amdgcn_exp2f(stat_max(v[j]) - bm);
          gm = bm;
        }
      }
      // log2 of the row's soft-max denominator; padded rows contribute exp2(-inf) = 0
      sm_fin[row] = row < W ? gm + log2f(gz) : INFINITY;
      __syncthreads();  // B
      // `ahead` is unit n + 2, warmed one unit ago; the one after it is warmed now
      if (u + 2 * n_teams < n_units) move_queries(ahead, (n + 2) % 3);
      if (u + 3 * n_teams < n_units) {
        ahead = unit_after(ahead, n_teams);
        warm_sink += warm_queries(ahead);
      }
      if (u + n_teams < n_units) cur = unit_after(cur, n_teams);
    }
    if (warm_sink == 0x7fffffff) sm_fin[0] = 0.f;  // keeps the warm-up loads alive
    return;
  }

  // =========================== compute wavefronts ============================
  int u = team;
  Unit cur = unit_of(u);
#pragma unroll
  for (int i = 0; i < NBW; ++i)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) hold[i][ks] = half8{0, 0, 0, 0, 0, 0, 0, 0};
  request_blocks(cur, load_ids(cur));
  // block ids of the unit after `cur`, requested one unit ahead of their use
  Unit nxt = u + n_teams < n_units ? unit_after(cur, n_teams) : cur;
  int ids_next = u + n_teams < n_units ? load_ids(nxt) : 0;
  __syncthreads();  // prologue

  for (int n = 0; u < n_units; ++n, u += n_teams) {
    const int qb = n % 3;
    const bool has_next = u + n_teams < n_units;
    to_operand_layout();
    // ---- pass 1 over the landed blocks: row maxima and normalisers ------------
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      float m = -3.0e38f, z = 0.f;
      floatx4 acc[NBW];
#pragma unroll
      for (int i = 0; i < NBW; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const half8 q = sm_q[qb][(nt * KS + ks) * 64 + lane];
#pragma unroll
        for (int i = 0; i < NBW; ++i)
          acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_f16(land[i][ks], q, acc[i], 0, 0, 0);
      }
      // mask, then one maximum over all of the wavefront's logits of this row
      // and one exponential per logit (c > 0, so max(c x) = c max(x))
#pragma unroll
      for (int i = 0; i < NBW; ++i) {
        const int b = block_of(cur, i);
        if (b >= cur.n_unmasked || b >= cur.b1) {  // uniform
          // query row at position L-W+row sees tokens up to its own position;
          // a slot without a block sees nothing
          const int limit = b < cur.b1 ? cur.n_prefix + nt * 16 + c16 : -1;
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (b * 16 + q4 * 4 + r > limit) acc[i][r] = -INFINITY;
        }
      }
      float mx = -INFINITY;
#pragma unroll
      for (int i = 0; i < NBW; ++i)
        if (block_of(cur, i) < cur.b1)  // uniform
          mx = fmaxf(mx, fmaxf(fmaxf(acc[i][0], acc[i][1]), fmaxf(acc[i][2], acc[i][3])));
      m = mx == -INFINITY ? -3.0e38f : mx * c;
#pragma unroll
      for (int i = 0; i < NBW; ++i)
        if (block_of(cur, i) < cur.b1)  // uniform
#pragma unroll
          for (int r = 0; r < 4; ++r) z += __builtin_amdgcn_exp2f(fmaf(acc[i][r], c, -m));
      // the four lanes that share a row hold disjoint tokens: merge them
#pragma unroll
      for (int o = 16; o <= 32; o <<= 1) {
        const float mo = __shfl_xor(m, o), zo = __shfl_xor(z, o);
        const float mn = fmaxf(m, mo);
        z = z * __builtin_amdgcn_exp2f(m - mn) + zo * __builtin_amdgcn_exp2f(mo - mn);
        m = mn;
      }
      if (q4 == 0) {
        sm_part[cw][0][nt * 16 + c16] = m;
        sm_part[cw][1][nt * 16 + c16] = z;
      }
    }
    __syncthreads();  // A
    if (cw == 0 && G > 1) {  // uniform: publish the workgroup's pairs
      float mm, zz;
      workgroup_stat(lane, mm, zz);
      const uint32_t tag = 1u + (uint32_t)((n + 1) % 255);
      uint64_t* xbuf = p.split_xchg + (size_t)((n + 1) & 1) * gridDim.x * 64;
      __hip_atomic_store(xbuf + (size_t)pos * 64 + lane, pack_stat(mm, zz, tag), __ATOMIC_RELAXED,
                         __HIP_MEMORY_SCOPE_AGENT);
    }

    // the landed blocks become the held ones; the next unit's are requested now,
    // so that they travel during the exchange and the second pass
#pragma unroll
    for (int i = 0; i < NBW; ++i)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) hold[i][ks] = land[i][ks];
    Unit nxt2 = nxt;
    if (has_next) {
      request_blocks(nxt, ids_next);
      // (behind those loads in the queue, so it costs no wait of its own)
      if (u + 2 * n_teams < n_units) {
        nxt2 = unit_after(nxt, n_teams);
        ids_next = load_ids(nxt2);
      }
    }
    __syncthreads();  // B

    // ---- pass 2 from the held blocks: column sums of the soft-maxed rows -------
    float colsum[NBW];
#pragma unroll
    for (int i = 0; i < NBW; ++i) colsum[i] = 0.f;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      float mrow[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) mrow[r] = sm_fin[nt * 16 + q4 * 4 + r];
      floatx4 acc[NBW];
#pragma unroll
      for (int i = 0; i < NBW; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const half8 q = sm_q[qb][(nt * KS + ks) * 64 + lane];
#pragma unroll
        for (int i = 0; i < NBW; ++i)
          acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_f16(q, hold[i][ks], acc[i], 0, 0, 0);
      }
#pragma unroll
      for (int i = 0; i < NBW; ++i)
        if (block_of(cur, i) < cur.b1)  // uniform
#pragma unroll
          for (int r = 0; r < 4; ++r)
            colsum[i] += __builtin_amdgcn_exp2f(fmaf(acc[i][r], c, -mrow[r]));
    }
    float* raw = p.raw_scores + cur.raw_off + (size_t)cur.lh * cur.L;
#pragma unroll
    for (int i = 0; i < NBW; ++i) {
      const int b = block_of(cur, i);
      float s2 = colsum[i];
      s2 += __shfl_xor(s2, 16);
      s2 += __shfl_xor(s2, 32);
      const int tok = b * 16 + c16;
      if (b < cur.b1 && q4 == 0 && tok < cur.n_prefix) raw[tok] = s2;
    }
    cur = nxt;
    nxt = nxt2;
  }
}


// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------

__global__ void zero_ints_kernel(int32_t* p, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

hipError_t launch_zero_ints(int32_t* p, int n, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  zero_ints_kernel<<<(n + 255) / 256, 256, 0, s>>>(p, n);
  return hipGetLastError();
}

template <int D>
static const void* split_kernel_ptr(int nt) {
  switch (nt) {
    case 1: return reinterpret_cast<const void*>(snapkv_split_kernel<D, 1>);
    case 2: return reinterpret_cast<const void*>(snapkv_split_kernel<D, 2>);
    case 3: return reinterpret_cast<const void*>(snapkv_split_kernel<D, 3>);
    case 4: return reinterpret_cast<const void*>(snapkv_split_kernel<D, 4>);
  }
  return nullptr;
}

static const void* split_kernel_for(int head_dim, int window) {
  const int nt = (window + 15) / 16;
  if (head_dim == 128) return split_kernel_ptr<128>(nt);
  if (head_dim == 64) return split_kernel_ptr<64>(nt);
  return nullptr;
}

int split_blocks_per_workgroup() { return kSplitCap; }

int split_grid_size(int head_dim, int window) {
  const void* fn = split_kernel_for(head_dim, window);
  if (!fn) return 0;
  int dev = 0, coop = 0, cus = 0, per_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&coop, hipDeviceAttributeCooperativeLaunch, dev) != hipSuccess || !coop)
    return 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
    return 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, kThreads, 0) != hipSuccess)
    return 0;
  if (per_cu > 2) per_cu = 2;
  return (cus * per_cu) & ~7;  // the XCD-major order assumes a multiple of 8
}

hipError_t launch_snapkv_split(const BatchParams& p, int grid, hipStream_t s) {
  const void* fn = split_kernel_for(p.head_dim, p.window);
  if (!fn || grid <= 0 || (grid & 7) || p.split_team < 1 || p.split_team > grid)
    return hipErrorInvalidValue;
  BatchParams copy = p;
  void* args[] = {&copy};
  return hipLaunchCooperativeKernel(fn, dim3(grid), dim3(kThreads), args, 0, s);
}

}  // namespace fc
