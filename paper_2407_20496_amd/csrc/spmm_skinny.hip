// HiNM product for few columns (decode-like shapes) and for V = 16 tiles
// (arXiv 2407.20496, Section 3.2: input rows are fetched through the vector index, here composed
// with pi_in on the fly; output rows are stored through pi_out).
//
// The work is bound by streaming the packed weights once from HBM.  One workgroup owns 16 rows of
// one tile and a block of 16 columns; its waves split the tile's kept columns in steps of 64 and
// each wave runs on its own: it streams its rows' stored values and NM nibbles straight into the A
// operand of the 16x16x64 sparse MFMA, gathers its 64 input rows (16 columns wide) into a private
// LDS slab, reads them back transposed as the B operand, and accumulates in fp32.  The per-wave
// partial tiles are summed in a fixed order through LDS, so results do not depend on timing.
#include "hinm_internal.h"
#include "mfma_types.h"

namespace hinm {
namespace {

constexpr int kRows = 16;   // rows per workgroup
constexpr int kCols = 16;   // columns per workgroup
constexpr int kStep = 64;   // kept columns per MFMA
constexpr int kUnroll = 4;  // k steps whose loads are issued together
// private LDS slab of one wave: 64 rows x 16 columns, 8-row blocks padded so that the four lane
// groups of a transposing read fall on different banks
constexpr int kSlabBytes = 8 * 384;

__device__ __forceinline__ int slab_row_offset(int row) { return row * 32 + (row >> 3) * 128; }

template <int DT, int NW>
__global__ __launch_bounds__(NW * 64) void spmm_skinny_kernel(
    const uint16_t* __restrict__ vals, const uint8_t* __restrict__ nm_idx, const int32_t* __restrict__ vec_idx,
    const int32_t* __restrict__ pi_in, const int32_t* __restrict__ pi_out, const uint16_t* __restrict__ X,
    int64_t ldx, void* __restrict__ Y, int64_t ldy, int V, int Kv, int N, bool relu, bool out_f32) {
  __shared__ __attribute__((aligned(16))) uint8_t slab_all[NW * kSlabBytes];
  __shared__ float partial[NW][kRows * kCols];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int row0 = blockIdx.x * kRows;  // first row of W handled here
  const int t = row0 / V;
  const int n0 = blockIdx.y * kCols;
  const int steps = (Kv + kStep - 1) / kStep;
  const int groups_total = Kv / 4;

  uint8_t* slab = slab_all + wave * kSlabBytes;
  const int i = lane & 15;   // A row / B column inside the block
  const int q = lane >> 4;   // lane group
  const int r = row0 + i;
  const uint16_t* vrow = vals + (size_t)r * (Kv / 2);
  const uint8_t* nrow = nm_idx + (size_t)r * (Kv / 8);
  const int32_t* vi = vec_idx + (size_t)t * Kv;
  const bool nm_pairs_aligned = ((Kv / 8) & 1) == 0;
  const bool x_vec_ok = (ldx % 8 == 0);

  f32x4 acc = {0.f, 0.f, 0.f, 0.f};

  for (int s_base = wave; s_base < steps; s_base += NW * kUnroll) {
    u32x4 a_reg[kUnroll];
    int idx_reg[kUnroll];
    u32x4 b_lo[kUnroll], b_hi[kUnroll];
    // ---- issue every global load of this batch --------------------------------------------
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int s = s_base + u * NW;
      a_reg[u] = u32x4{0, 0, 0, 0};
      idx_reg[u] = 0;
      b_lo[u] = u32x4{0, 0, 0, 0};
      b_hi[u] = u32x4{0, 0, 0, 0};
      if (s < steps) {
        // A: this lane's four groups 16 s + 4 q .. + 3  (stored values 32 s + 8 q .. + 7)
        const int g0 = 16 * s + 4 * q;
        if (g0 + 4 <= groups_total) {
          a_reg[u] = *reinterpret_cast<const u32x4_a4*>(vrow + 2 * g0);
          if (nm_pairs_aligned) idx_reg[u] = *reinterpret_cast<const uint16_t*>(nrow + (g0 >> 1));
          else idx_reg[u] = (int)nrow[g0 >> 1] | ((int)nrow[(g0 >> 1) + 1] << 8);
        } else if (g0 + 2 <= groups_total) {  // Kv % 8 == 0: the tail holds whole pairs of groups
          const u32x2 half = *reinterpret_cast<const u32x2_a4*>(vrow + 2 * g0);
          a_reg[u] = u32x4{half.x, half.y, 0, 0};
          idx_reg[u] = (int)nrow[g0 >> 1];
        }
        // B: lane fetches input row j = 64 s + lane of the tile, 16 columns wide
        const int j = kStep * s + lane;
        if (j < Kv) {
          int c = vi[j];
          if (pi_in) c = pi_in[c];
          const uint16_t* xr = X + (size_t)c * ldx + n0;
          if (x_vec_ok && n0 + 8 <= N) {
            b_lo[u] = *reinterpret_cast<const u32x4*>(xr);
          } else {
            uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
            for (int e = 0; e < 8; ++e)
              if (n0 + e < N) w[e >> 1] |= (uint32_t)xr[e] << (16 * (e & 1));
            b_lo[u] = u32x4{w[0], w[1], w[2], w[3]};
          }
          if (x_vec_ok && n0 + 16 <= N) {
            b_hi[u] = *reinterpret_cast<const u32x4*>(xr + 8);
          } else if (n0 + 8 < N) {
            uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
            for (int e = 0; e < 8; ++e)
              if (n0 + 8 + e < N) w[e >> 1] |= (uint32_t)xr[8 + e] << (16 * (e & 1));
            b_hi[u] = u32x4{w[0], w[1], w[2], w[3]};
          }
        }
      }
    }
    // ---- consume ---------------------------------------------------------------------------
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int s = s_base + u * NW;
      if (s < steps) {  // wave-uniform
        uint8_t* wr = slab + slab_row_offset(lane);
        *reinterpret_cast<u32x4*>(wr) = b_lo[u];
        *reinterpret_cast<u32x4*>(wr + 16) = b_hi[u];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        // B slots 8 h + 4 u2 .. + 3 of lane group q <- rows 32 h + 8 q + 4 u2 + (0..3), column i;
        // inside a 16-lane group lane i addresses row (i / 4) and columns 4 (i % 4) .. + 3.
        u32x8 b;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
#pragma unroll
          for (int u2 = 0; u2 < 2; ++u2) {
            const int row = 32 * h + 8 * q + 4 * u2 + (i >> 2);
            const u32x2 v = lds_read_tr16(slab + slab_row_offset(row) + (i & 3) * 8);
            b[(2 * h + u2) * 2] = v.x;
            b[(2 * h + u2) * 2 + 1] = v.y;
          }
        }
        acc = smfmac_16x16x64<DT, 0>(a_reg[u], b, acc, idx_reg[u]);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      }
    }
  }

  // ---- fixed-order reduction over the waves, epilogue ---------------------------------------
  // D layout: lane holds column lane % 16, rows 4 * (lane / 16) + reg.
#pragma unroll
  for (int reg = 0; reg < 4; ++reg) partial[wave][(4 * q + reg) * kCols + i] = acc[reg];
  __syncthreads();
  for (int e = threadIdx.x; e < kRows * kCols; e += NW * 64) {
    float sum = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) sum += partial[w][e];
    if (relu) sum = sum > 0.f ? sum : 0.f;
    const int row = e / kCols, col = e % kCols;
    if (n0 + col < N) {
      const int64_t out_row = pi_out ? pi_out[row0 + row] : (row0 + row);
      if (out_f32) static_cast<float*>(Y)[out_row * ldy + n0 + col] = sum;
      else static_cast<uint16_t*>(Y)[out_row * ldy + n0 + col] = float_to_bits<DT>(sum);
    }
  }
}

}  // namespace

bool spmm_skinny_supported(const SpmmArgs& a) {
  return a.s.V % 16 == 0 && (a.s.M / 16) <= 0x7FFFFFFF && (a.N + 15) / 16 <= 65535;
}

hipError_t launch_spmm_skinny(const SpmmArgs& a, hipStream_t stream) {
  dim3 grid(a.s.M / kRows, (a.N + kCols - 1) / kCols);
  auto v = static_cast<const uint16_t*>(a.vals);
  auto x = static_cast<const uint16_t*>(a.X);
  const int steps = (a.s.Kv + kStep - 1) / kStep;
#define HINM_LAUNCH_SKINNY(DT, NW)                                                                              \
  spmm_skinny_kernel<DT, NW><<<grid, NW * 64, 0, stream>>>(v, a.nm_idx, a.vec_idx, a.pi_in, a.pi_out, x, a.ldx, \
                                                           a.Y, a.ldy, a.s.V, a.s.Kv, a.N, a.relu, a.out_f32)
  if (a.s.dtype == HINM_F16) {
    if (steps >= 32) HINM_LAUNCH_SKINNY(HINM_F16, 8);
    else if (steps >= 4) HINM_LAUNCH_SKINNY(HINM_F16, 4);
    else HINM_LAUNCH_SKINNY(HINM_F16, 1);
  } else {
    if (steps >= 32) HINM_LAUNCH_SKINNY(HINM_BF16, 8);
    else if (steps >= 4) HINM_LAUNCH_SKINNY(HINM_BF16, 4);
    else HINM_LAUNCH_SKINNY(HINM_BF16, 1);
  }
#undef HINM_LAUNCH_SKINNY
  return hipGetLastError();
}

}  // namespace hinm
