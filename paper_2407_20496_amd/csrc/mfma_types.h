// Register-level view of the gfx950 sparse matrix instructions used by the HiNM kernels.
//
// Both forms multiply a 4:2-compressed A (rows = output channels) by a dense B (columns = tokens):
//   16x16x64: A 16 rows x 64 dense k (32 stored), B 64 k x 16 columns, D 16 x 16 fp32 (4 registers)
//   32x32x32: A 32 rows x 32 dense k (16 stored), B 32 k x 32 columns, D 32 x 32 fp32 (16 registers)
//
// Operand layout, established by one-hot probing on MI355X (R = 16 or 32 rows/columns, lane l):
//   A  : lane l holds row l % R, lane group qa = l / R; 8 stored values = 4 groups of four dense k.
//   B  : lane l holds column l % R, lane group qb = l / R; 16 dense k values in slots 0..15.
//   D  : 16x16: lane l holds column l % 16, rows 4*(l/16) + reg.
//        32x32: lane l holds column l % 32, rows 8*(reg/4) + 4*(l/32) + reg % 4.
//   idx: 16 bits per lane and instruction, nibble g = p0 | p1 << 2 for the lane's g-th group (first
//        stored value sits at dense position p0, second at p1); ABID bit 0 selects the low or high
//        half of the 32-bit index register.
//   Pairing of k: the two groups in A slots 4*ps .. 4*ps+3 (ps = 0, 1) of lane group qa meet B slots
//        8*h .. 8*h+7 of lane group qb, where
//          32x32x32: qb = ps,                h = qa
//          16x16x64: qb = 2 * (qa % 2) + ps, h = qa / 2.
//   The NM nibble of the canonical packed format is exactly the hardware nibble.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hinm.h"

namespace hinm {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x8 __attribute__((ext_vector_type(8)));
// 16-byte global load that only promises 4-byte alignment
typedef uint32_t u32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));
typedef uint32_t u32x2_a4 __attribute__((ext_vector_type(2), aligned(4)));
typedef short i16x4 __attribute__((ext_vector_type(4)));

template <int DT, int ABID>
__device__ __forceinline__ f32x4 smfmac_16x16x64(u32x4 a, u32x8 b, f32x4 c, int idx) {
  if constexpr (DT == HINM_F16) {
    return __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x16, b), c, idx,
                                                    0, ABID);
  } else {
    return __builtin_amdgcn_smfmac_f32_16x16x64_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x16, b), c,
                                                     idx, 0, ABID);
  }
}

template <int DT, int ABID>
__device__ __forceinline__ f32x16 smfmac_32x32x32(u32x4 a, u32x8 b, f32x16 c, int idx) {
  if constexpr (DT == HINM_F16) {
    return __builtin_amdgcn_smfmac_f32_32x32x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x16, b), c, idx,
                                                    0, ABID);
  } else {
    return __builtin_amdgcn_smfmac_f32_32x32x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x16, b), c,
                                                     idx, 0, ABID);
  }
}

// LDS transposing read: within every group of 16 lanes the 64 16-bit elements addressed by the
// group (lane i supplies 4 consecutive elements) are viewed as a 4 x 16 row-major block and lane c
// receives column c, i.e. elements (row 0..3, column c).
__device__ __forceinline__ u32x2 lds_read_tr16(const void* lds_ptr) {
  typedef __attribute__((address_space(3))) i16x4 lds_i16x4;
  i16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)lds_ptr);
  return __builtin_bit_cast(u32x2, v);
}


// Four transposing LDS reads from one per-lane base address plus compile-time byte offsets, issued as
// raw instructions: the compiler would otherwise hold every such read until all direct-to-LDS
// copies in flight have landed, which serialises the copy pipeline.  The caller must execute
// lds_wait_tr() on the results before using them.
template <int O0, int O1, int O2, int O3>
__device__ __forceinline__ void lds_read_tr16_x4(uint32_t lds_addr, u32x2& r0, u32x2& r1, u32x2& r2, u32x2& r3) {
  static_assert(O0 >= 0 && O3 < 65536 && O1 < 65536 && O2 < 65536, "DS offset field is 16 bits");
  asm volatile(
      "ds_read_b64_tr_b16 %0, %4 offset:%5\n\t"
      "ds_read_b64_tr_b16 %1, %4 offset:%6\n\t"
      "ds_read_b64_tr_b16 %2, %4 offset:%7\n\t"
      "ds_read_b64_tr_b16 %3, %4 offset:%8"
      : "=&v"(r0), "=&v"(r1), "=&v"(r2), "=&v"(r3)
      : "v"(lds_addr), "n"(O0), "n"(O1), "n"(O2), "n"(O3));
}

// Waits for every LDS operation of this wave and ties the wait to the given registers, so that no
// use of them can be scheduled before it.
__device__ __forceinline__ void lds_wait_tr(u32x8& b0, u32x8& b1) {
  asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(b0), "+v"(b1));
}
__device__ __forceinline__ void lds_wait_tr(u32x8& b0) { asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(b0)); }

}  // namespace hinm
