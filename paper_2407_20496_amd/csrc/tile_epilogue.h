// Epilogue shared by the tile kernels whose waves each hold all V = 32 * RB rows of the tile for WC of the
// workgroup's NB columns in 32x32 MFMA accumulators (arXiv 2407.20496, Section 3.2: the tile's result goes to the
// output channels named by the output-channel order; Section 5.3: re-ordering at no run-time cost).
//   fp32 accumulators -> optional ReLU -> either fp32 straight from the registers, or rounded to the 16-bit
//   storage type, staged through LDS (row stride Y_STRIDE bytes) so that every output row leaves as one
//   contiguous segment, written with non-temporal 16-byte stores (the ragged tail element by element).
#pragma once

#include "mfma_types.h"

namespace hinm {

// acc[rb][cb][e]: D layout of the 32x32 MFMA, lane holds column lane % 32, rows 8 * (e / 4) + 4 * (lane / 32) + e % 4
// of row block rb, 32-column block cb of the wave.  `out_row_of(row)` names the row of Y for row `row` of the tile.
// The caller guarantees nothing: the barrier that ends the k loop's use of LDS is taken here.
template <int DT, int RB, int CBS, int NB, int WC, int THREADS, int Y_STRIDE, class OutRow>
__device__ __forceinline__ void store_tile_rows(const f32x16 (&acc)[RB][CBS], uint8_t* lds, void* Y, int64_t ldy, int N,
                                                int n0, bool relu, bool out_f32, OutRow out_row_of) {
  constexpr int V = 32 * RB;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int i32 = lane & 31;
  const int qh = lane >> 5;
  if (out_f32) {
    float* Yf = static_cast<float*>(Y);
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int64_t out_row = out_row_of(32 * rb + 8 * (e >> 2) + 4 * qh + (e & 3));
#pragma unroll
        for (int cb = 0; cb < CBS; ++cb) {
          const int n = n0 + wave * WC + cb * 32 + i32;
          float v = acc[rb][cb][e];
          if (relu) v = v > 0.f ? v : 0.f;
          if (n < N) Yf[out_row * ldy + n] = v;
        }
      }
    return;
  }
  __builtin_amdgcn_s_barrier();  // every wave is done reading the stages
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int cb = 0; cb < CBS; ++cb)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int row = 32 * rb + 8 * (e >> 2) + 4 * qh + (e & 3);
        const int col = wave * WC + cb * 32 + i32;
        float v = acc[rb][cb][e];
        if (relu) v = v > 0.f ? v : 0.f;
        *reinterpret_cast<uint16_t*>(lds + row * Y_STRIDE + col * 2) = float_to_bits<DT>(v);
      }
  __syncthreads();
  uint16_t* Yh = static_cast<uint16_t*>(Y);
  constexpr int LANES_PER_ROW = NB / 8;
  const int chunk = tid % LANES_PER_ROW;
  for (int row = tid / LANES_PER_ROW; row < V; row += THREADS / LANES_PER_ROW) {
    const int64_t out_row = out_row_of(row);
    const int n = n0 + chunk * 8;
    const u32x4 v = *reinterpret_cast<const u32x4*>(lds + row * Y_STRIDE + chunk * 16);
    uint16_t* dst = Yh + out_row * ldy + n;
    if (n + 8 <= N) {
      __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(dst));
    } else if (n < N) {
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
      for (int e = 0; e < N - n; ++e) dst[e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
    }
  }
}

}  // namespace hinm
