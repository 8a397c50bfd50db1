// Device-side helpers shared by the kernel translation units.
#pragma once

#include "fc_internal.h"

namespace fc {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

#ifndef FC_WAVES
#define FC_WAVES 4
#endif
static constexpr int kWaves = FC_WAVES;  // wavefronts per workgroup
static constexpr int kThreads = 64 * kWaves;

__device__ __forceinline__ int clamp_block(int blk, int n_blocks) {
  // Block ids come from caller-owned device memory; an id outside the pool
  // must not turn into an out-of-bounds access.
  return ((unsigned)blk < (unsigned)n_blocks) ? blk : 0;
}

// v + (the same register of another lane of the 16-lane row), by DPP control
template <int CTRL>
__device__ __forceinline__ float add_across_row(float v) {
  return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
// sum over the 16 lanes of a row, left in every one of them
__device__ __forceinline__ float row16_sum(float v) {
  v = add_across_row<0xB1>(v);   // quad_perm [1,0,3,2]
  v = add_across_row<0x4E>(v);   // quad_perm [2,3,0,1]
  v = add_across_row<0x141>(v);  // row_half_mirror: lane i <-> 7 - i of each 8
  v = add_across_row<0x140>(v);  // row_mirror: lane i <-> 15 - i
  return v;
}

__device__ __forceinline__ half8 load_half8(const _Float16* p) {
  return *reinterpret_cast<const half8*>(p);
}

// The same accesses with the non-temporal hint, for data that this kernel will
// not touch again: the line is the first to leave the caches, which keeps what
// IS read again (K between the two passes of the SnapKV score, the rows that
// the compaction re-reads) in L2 and in the memory-side cache for longer.
__device__ __forceinline__ half8 load_half8_nt(const _Float16* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const half8*>(p));
}

__device__ __forceinline__ void store_half8_nt(_Float16* p, half8 v) {
  __builtin_nontemporal_store(v, reinterpret_cast<half8*>(p));
}

__device__ __forceinline__ void store_half8(_Float16* p, half8 v) {
  *reinterpret_cast<half8*>(p) = v;
}

}  // namespace fc
