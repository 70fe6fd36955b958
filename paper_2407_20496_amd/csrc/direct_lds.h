// Direct global -> LDS copies (no registers in between) and the bookkeeping around them, shared by
// the kernels that stream gathered input rows through LDS (gfx950).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hinm {

typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void global_void_t;

__device__ __forceinline__ void copy16_to_lds(const void* src_lane, void* lds_wave_base) {
  // every lane copies 16 bytes; lane l lands at lds_wave_base + 16 l
  __builtin_amdgcn_global_load_lds((global_void_t*)src_lane, (lds_void_t*)lds_wave_base, 16, 0, 0);
}

__device__ __forceinline__ void copy4_to_lds(const void* src_lane, void* lds_wave_base) {
  // every lane copies 4 bytes; lane l lands at lds_wave_base + 4 l
  __builtin_amdgcn_global_load_lds((global_void_t*)src_lane, (lds_void_t*)lds_wave_base, 4, 0, 0);
}

// s_waitcnt vmcnt(n) with everything else left alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14,
// expcnt 6:4, lgkmcnt 11:8)
template <int N>
__device__ __forceinline__ void wait_copies_outstanding() {
  static_assert(N >= 0 && N < 64, "vmcnt range");
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}
// Outstanding copies allowed = `later` stages of (B + extra) copies each; extra is 0..3, later 0..2.
template <int B>
__device__ __forceinline__ void wait_copies_outstanding(int later, int extra) {
  if (later == 0) {
    wait_copies_outstanding<0>();
  } else if (later == 1) {
    switch (extra) {
      case 0: wait_copies_outstanding<B>(); break;
      case 1: wait_copies_outstanding<B + 1>(); break;
      case 2: wait_copies_outstanding<B + 2>(); break;
      default: wait_copies_outstanding<B + 3>(); break;
    }
  } else {
    switch (extra) {
      case 0: wait_copies_outstanding<2 * B>(); break;
      case 1: wait_copies_outstanding<2 * B + 2>(); break;
      case 2: wait_copies_outstanding<2 * B + 4>(); break;
      default: wait_copies_outstanding<2 * B + 6>(); break;
    }
  }
}

// 32-byte units of a row are stored at unit ^ swizzle(row & 3): the four rows a transposing read
// touches then sit on four different bank groups, for 16-lane as well as 32-lane LDS passes.
__host__ __device__ constexpr int swizzle_of_row(int r) { return ((r & 3) << 1) | (((r >> 1) ^ r) & 1); }

}  // namespace hinm
