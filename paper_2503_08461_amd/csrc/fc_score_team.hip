// One-pass SnapKV-style score kernel for gfx950.
//
// The row softmax needs every logit of a row before any column sum can be
// finished, so a kernel that streams K once has to keep the logits somewhere
// until the normalisers are known.  Here they stay in registers: the MFMA
// accumulators of a workgroup hold the logits of up to kTeamCap tokens, and a
// (layer, head) that is longer than that is shared by a TEAM of g workgroups,
// each holding a contiguous run of pool blocks.  Team members exchange their
// per-query (max, sum-of-exp) pairs through global memory and one counter,
// then every member finishes its own columns from its own registers.  K is
// read from HBM exactly once; nothing but 4 bytes per token is written.
//
// Waiting on another workgroup is only safe if that workgroup is running, so
// the kernel is persistent and is launched co-resident (cooperative launch,
// grid = what the device can hold at once).  Every workgroup walks the same
// global job order (request, then round), so the earliest unfinished job
// always has all its members present and the grid drains.  The wait is
// bounded all the same: if it runs out, an error flag is raised and the
// workgroup moves on, so every wavefront exits.

#include "fc_device.h"

#include <float.h>

namespace fc {

// blocks held per wavefront for NT = ceil(window/16) query tiles; NT*4*NBW
// accumulator registers per lane, sized so that the kernel does not spill
__host__ __device__ constexpr int team_nbw(int nt) {
  return nt == 1 ? 20 : nt == 2 ? 14 : nt == 3 ? 10 : 8;
}

static constexpr int kMaxSpins = 1 << 21;  // about a second

template <int D, int NT>
__global__ __launch_bounds__(kThreads, 2) void snapkv_score_team_kernel(BatchParams p) {
  constexpr int KS = D / 32;
  constexpr int NBW = team_nbw(NT);
  const int n_lh = p.n_layers * p.n_heads;
  const int n_wg = gridDim.x;
  const int wg = blockIdx.x;
  const int W = p.window;  // the host admits one window size per batch to this kernel
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int c16 = lane & 15;
  const int q4 = lane >> 4;
  const float c = p.scale_log2e;

  // window queries in MFMA operand order: entry (nt*KS + ks)*64 + lane
  __shared__ half8 sm_q[NT * KS * 64];
  __shared__ float sm_m[kWaves][4][64];
  __shared__ float sm_z[kWaves][4][64];
  __shared__ float sm_final[64];

  for (int slot = 0; slot < p.n_snap; ++slot) {
    const ReqDesc rd = p.descs[p.order_snap[slot]];
    const int g = rd.team_size;
    const int n_teams = n_wg / g;
    if (wg >= n_teams * g) continue;  // left over for this request
    const int team = wg / g;
    const int member = wg - team * g;
    const int L = rd.seq_len;
    const int nb = (L + 15) >> 4;
    const int bpm = (nb + g - 1) / g;  // blocks per member
    const int b0m = member * bpm;
    const int b1m = min(nb, b0m + bpm);
    // each wavefront takes a contiguous run of the member's blocks
    const int bpw = (bpm + kWaves - 1) / kWaves;
    const int b0 = b0m + wave * bpw;
    const int b1 = min(b1m, b0 + bpw);
    const int n_unmasked = (L - W) >> 4;
    const int n_prefix = L - W;
    int32_t* counter = p.team_counters + rd.team_counter + team;
    float* stats = p.team_stats + rd.team_stats + (size_t)team * 2 * g * 128;
    // the wavefront's block ids, one per lane
    int my_id = 0;
    if (b0 + lane < b1) my_id = clamp_block(p.old_ids[rd.old_off + b0 + lane], p.n_blocks);

    int round = 0;
    for (int lh = team; lh < n_lh; lh += n_teams, ++round) {
      const int layer = lh / p.n_heads;
      const int head = lh - layer * p.n_heads;
      __syncthreads();  // the previous unit is done with the shared arrays

      const _Float16* qbase = p.q_window + rd.q_off + (size_t)lh * W * D;
      for (int e = threadIdx.x; e < NT * KS * 64; e += kThreads) {
        const int ln = e & 63;
        const int ks = (e >> 6) % KS;
        const int nt = (e >> 6) / KS;
        const int row = nt * 16 + (ln & 15);
        half8 v = {0, 0, 0, 0, 0, 0, 0, 0};
        if (row < W) v = load_half8(qbase + (size_t)row * D + ks * 32 + (ln >> 4) * 8);
        sm_q[e] = v;
      }
      const size_t blk_stride = (size_t)2 * p.n_heads * 16 * D;
      const _Float16* kbase = p.kv + (size_t)layer * p.n_blocks * blk_stride +
                              (size_t)head * 16 * D + (size_t)c16 * D + q4 * 8;

      // ---- the one pass over K: logits into registers, online row statistics
      floatx4 t[NBW][NT];
      float m[NT], z[NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        m[nt] = -3.0e38f;
        z[nt] = 0.f;
      }
      half8 kbuf[2][KS];
      if (b0 < b1) {
        const _Float16* kp = kbase + (size_t)__builtin_amdgcn_readlane(my_id, 0) * blk_stride;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) kbuf[0][ks] = load_half8(kp + ks * 32);
      }
      __syncthreads();  // sm_q is complete
#pragma unroll
      for (int k = 0; k < NBW; ++k) {
        const int b = b0 + k;
        if (k + 1 < NBW && b + 1 < b1) {
          const _Float16* kp =
              kbase + (size_t)__builtin_amdgcn_readlane(my_id, (k + 1 < NBW) ? k + 1 : 0) * blk_stride;
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) kbuf[(k + 1) & 1][ks] = load_half8(kp + ks * 32);
        }
        if (b < b1) {
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
              acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(
                  kbuf[k & 1][ks], sm_q[(nt * KS + ks) * 64 + lane], acc, 0, 0, 0);
            floatx4 tt;
#pragma unroll
            for (int r = 0; r < 4; ++r) tt[r] = acc[r] * c;
            if (b >= n_unmasked) {
              const int limit = n_prefix + nt * 16 + c16;  // query i sees tokens <= L-W+i
#pragma unroll
              for (int r = 0; r < 4; ++r)
                if (b * 16 + q4 * 4 + r > limit) tt[r] = -INFINITY;
            }
            const float bm = fmaxf(fmaxf(tt[0], tt[1]), fmaxf(tt[2], tt[3]));
            const float mn = fmaxf(m[nt], bm);
            float zz = z[nt] * __builtin_amdgcn_exp2f(m[nt] - mn);
#pragma unroll
            for (int r = 0; r < 4; ++r) zz += __builtin_amdgcn_exp2f(tt[r] - mn);
            z[nt] = zz;
            m[nt] = mn;
            t[k][nt] = tt;
          }
        }
      }

      // ---- this member's (max, sum) per query
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        sm_m[wave][q4][nt * 16 + c16] = m[nt];
        sm_z[wave][q4][nt * 16 + c16] = z[nt];
      }
      __syncthreads();
      float mm = -3.0e38f, zz = 0.f;
      if (threadIdx.x < 64) {
        const int row = threadIdx.x;
        for (int w = 0; w < kWaves; ++w)
          for (int q = 0; q < 4; ++q) mm = fmaxf(mm, sm_m[w][q][row]);
        for (int w = 0; w < kWaves; ++w)
          for (int q = 0; q < 4; ++q)
            zz += sm_z[w][q][row] * __builtin_amdgcn_exp2f(sm_m[w][q][row] - mm);
      }
      if (g > 1) {
        // ---- exchange with the other members of the team
        float* buf = stats + (size_t)(round & 1) * g * 128;
        if (threadIdx.x < 64) {
          __hip_atomic_store(buf + member * 128 + threadIdx.x * 2, mm, __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
          __hip_atomic_store(buf + member * 128 + threadIdx.x * 2 + 1, zz, __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        if (threadIdx.x == 0) {
          __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
          const int target = (round + 1) * g;
          int spins = 0;
          while (__hip_atomic_load(counter, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) < target) {
            __builtin_amdgcn_s_sleep(4);
            if (++spins > kMaxSpins) {
              __hip_atomic_store(p.error_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              break;
            }
          }
        }
        __syncthreads();
        if (threadIdx.x < 64) {
          float gm = -3.0e38f;
          for (int j = 0; j < g; ++j)
            gm = fmaxf(gm, __hip_atomic_load(buf + j * 128 + threadIdx.x * 2, __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT));
          float gz = 0.f;
          for (int j = 0; j < g; ++j) {
            const float mj = __hip_atomic_load(buf + j * 128 + threadIdx.x * 2, __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_AGENT);
            const float zj = __hip_atomic_load(buf + j * 128 + threadIdx.x * 2 + 1,
                                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            gz += zj * __builtin_amdgcn_exp2f(mj - gm);
          }
          mm = gm;
          zz = gz;
        }
      }
      if (threadIdx.x < 64)
        sm_final[threadIdx.x] = (threadIdx.x < W) ? mm + log2f(zz) : INFINITY;
      __syncthreads();

      // ---- column sums from the retained logits
      float mfin[NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) mfin[nt] = sm_final[nt * 16 + c16];
      float* raw = p.raw_scores + rd.raw_off + (size_t)lh * L;
#pragma unroll
      for (int k = 0; k < NBW; ++k) {
        const int b = b0 + k;
        if (b < b1 && b * 16 < n_prefix) {
          float s4[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int r = 0; r < 4; ++r) s4[r] += __builtin_amdgcn_exp2f(t[k][nt][r] - mfin[nt]);
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            s4[r] += __shfl_xor(s4[r], 1);
            s4[r] += __shfl_xor(s4[r], 2);
            s4[r] += __shfl_xor(s4[r], 4);
            s4[r] += __shfl_xor(s4[r], 8);
          }
          if (c16 == 0) {
            const int tok0 = b * 16 + q4 * 4;
#pragma unroll
            for (int r = 0; r < 4; ++r)
              if (tok0 + r < n_prefix) raw[tok0 + r] = s4[r];
          }
        }
      }
    }
  }
}

__global__ void zero_ints_kernel(int32_t* p, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

hipError_t launch_zero_ints(int32_t* p, int n, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  zero_ints_kernel<<<(n + 255) / 256, 256, 0, s>>>(p, n);
  return hipGetLastError();
}

int team_capacity_tokens(int window) {
  const int nt = (window + 15) / 16;
  return kWaves * team_nbw(nt) * 16;
}

template <int D>
static const void* team_kernel_ptr(int nt) {
  switch (nt) {
    case 1: return reinterpret_cast<const void*>(snapkv_score_team_kernel<D, 1>);
    case 2: return reinterpret_cast<const void*>(snapkv_score_team_kernel<D, 2>);
    case 3: return reinterpret_cast<const void*>(snapkv_score_team_kernel<D, 3>);
    case 4: return reinterpret_cast<const void*>(snapkv_score_team_kernel<D, 4>);
  }
  return nullptr;
}

static const void* team_kernel_for(int head_dim, int window) {
  const int nt = (window + 15) / 16;
  if (head_dim == 128) return team_kernel_ptr<128>(nt);
  if (head_dim == 64) return team_kernel_ptr<64>(nt);
  return nullptr;
}

int team_grid_size(int head_dim, int window) {
  const void* fn = team_kernel_for(head_dim, window);
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
  return cus * per_cu;
}

hipError_t launch_snapkv_score_team(const BatchParams& p, int grid, hipStream_t s) {
  const void* fn = team_kernel_for(p.head_dim, p.window);
  if (!fn || grid <= 0) return hipErrorInvalidValue;
  BatchParams copy = p;
  void* args[] = {&copy};
  return hipLaunchCooperativeKernel(fn, dim3(grid), dim3(kThreads), args, 0, s);
}

}  // namespace fc
