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


// One wave's share of the gathered input rows of a stage, copied straight into LDS as NB-column row segments.
//   NB = 512: one wave-wide copy per row, lane = position of its 16 bytes in the 1024-byte segment;
//   NB = 256: one copy per pair of consecutive rows, lanes 0..31 the even row, 32..63 the odd one.
// A copy's source is a wave-uniform row base plus a per-lane byte offset that depends only on row % 4 (the
// swizzle of swizzle_of_row, applied on the source side because a direct copy writes LDS linearly): the
// offsets are computed once per kernel.  Lanes whose columns lie at or beyond N re-read the block's first
// columns instead; the accumulator columns they feed are never stored.
template <int NB>
struct RowSegmentCopy {
  static_assert(NB == 256 || NB == 512, "column block");
  uint32_t off[4];            // by row % 4 (NB = 512)
  uint32_t even_k, odd_k;     // NB = 256: this lane's offset in the k-th pair for even and odd k
  int half;                   // NB = 256: which row of a pair this lane copies

  __device__ __forceinline__ RowSegmentCopy(int lane, int n0, int N) {
    const int gpos = (NB == 512) ? lane : (lane & 31);
    half = (NB == 512) ? 0 : (lane >> 5);
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      const int granule = (((gpos >> 1) ^ swizzle_of_row(r4)) << 1) | (gpos & 1);  // which 16 bytes of the row segment
      off[r4] = (n0 + granule * 8 < N) ? granule * 16 : 0;
    }
    // lane in half h copies row 2 k + h, so row % 4 is h for even k and 2 + h for odd k
    even_k = half ? off[1] : off[0];
    odd_k = half ? off[3] : off[2];
  }

  // Issues the wave-wide copies K0 .. K0 + COPIES - 1 of the wave's share of a stage: row_base(j) = wave-uniform
  // source address of the wave's j-th row at the block's first column; row j lands at first_row + j * ROW_BYTES.
  // The wave's first row must have an index that is a multiple of four in the stage (it has: waves own 4, 8 or 16
  // consecutive rows); copy k covers row k (NB = 512) or rows 2 k and 2 k + 1 (NB = 256).
  template <int K0, int COPIES, int ROW_BYTES, class RowBase>
  __device__ __forceinline__ void issue_range(RowBase row_base, uint8_t* first_row) const {
#pragma unroll
    for (int k = K0; k < K0 + COPIES; ++k) {
      if constexpr (NB == 512) {
        copy16_to_lds(row_base(k) + off[k & 3], first_row + k * ROW_BYTES);
      } else {
        const uint8_t* be = row_base(2 * k);
        const uint8_t* bo = row_base(2 * k + 1);
        copy16_to_lds((half ? bo : be) + ((k & 1) ? odd_k : even_k), first_row + 2 * k * ROW_BYTES);
      }
    }
  }
  template <int COPIES, int ROW_BYTES, class RowBase>
  __device__ __forceinline__ void issue(RowBase row_base, uint8_t* first_row) const {
    issue_range<0, COPIES, ROW_BYTES>(row_base, first_row);
  }
};

}  // namespace hinm
