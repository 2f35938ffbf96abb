// Device helpers shared by the recurrent-mixer kernels (state access, lane reductions, bf16 unpacking).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace {

typedef __attribute__((ext_vector_type(4))) float f32x4;

// The state is touched exactly once per step, so it is loaded and stored with the non-temporal
// hint: measured back to back over 1 GiB of states on MI355X this is ~14 % faster than plain
// accesses, and a whole decode step (GDN, KDA, FA, SWA in turn) ~1 % faster.  Plain accesses only
// win when the same 128 MiB of state is stepped again while it still sits in the 256 MB last-level
// cache, which a model with dozens of recurrent layers never does.
__device__ __forceinline__ float4 load_state(const float* p) {
  const f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
  return float4{t[0], t[1], t[2], t[3]};
}
__device__ __forceinline__ void store_state(float* p, const float4& v) {
  const f32x4 t = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(t, reinterpret_cast<f32x4*>(p));
}

// Which tile the i-th of n workgroups visits.  Workgroups start in index order, so with the identity the ~1000
// resident ones sweep one contiguous 64 MiB window of the states; visiting four quarters of the tile list in turn
// keeps four windows a quarter of the list apart in flight, which the memory system serves faster once the list
// spans 256 MiB and more (one GDN step, identity against this order: 128 MiB of states 47.5 / 47.5 us, 256 MiB
// 95.2 / 92.3, 512 MiB 190.5 / 182.4, 1 GiB 390 / 366; two parts or eight are worse at some of these sizes).
__device__ __forceinline__ int interleaved_tile(int i, int n) { return (n & 3) ? i : (i & 3) * (n >> 2) + (i >> 2); }

// A per-(row, head) scalar read through the constant address space: the index is the same for the
// whole workgroup, so this becomes a scalar-cache load instead of 64 identical vector loads.  The
// gates are inputs and are not written while the kernel runs.
typedef const __attribute__((address_space(4))) float* const_f32_ptr;
__device__ __forceinline__ float load_uniform(const float* p, size_t i) {
  return reinterpret_cast<const_f32_ptr>(reinterpret_cast<uintptr_t>(p))[i];
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// Sum over the 8 lanes that share c8 (lane bits 3..5).  Lane l ^ 8 sits in the same row of 16 lanes: a row rotation
// by 8 (one DPP-modified add) fetches it without a trip through the LDS crossbar.
__device__ __forceinline__ float reduce_r8(float x) {
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x128 /* row_ror:8 */, 0xf, 0xf, false));
  x += __shfl_xor(x, 16);
  x += __shfl_xor(x, 32);
  return x;
}

// Orders this wavefront's LDS writes before its later LDS reads by other lanes (no other wavefront involved).
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

}  // namespace
