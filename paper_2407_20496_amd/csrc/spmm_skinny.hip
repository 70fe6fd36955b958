// HiNM product for few columns (decode-like shapes) and for V = 16 tiles
// (arXiv 2407.20496, Section 3.2: input rows are fetched through the vector index, here composed
// with pi_in on the fly; output rows are stored through pi_out).
//
// The work is bound by streaming the packed weights once from HBM.  One workgroup owns 16 rows of
// one tile and a block of 16 columns; its waves split the tile's kept columns into contiguous
// ranges of 64-column steps and each wave runs on its own: it streams its rows' stored values and
// NM nibbles straight into the A operand of the 16x16x64 sparse MFMA, gathers its 64 input rows
// (16 columns wide) into a private LDS slab, reads them back transposed as the B operand, and
// accumulates in fp32.  All global loads of a batch of steps are issued before the first is used
// (weights first, then the index chain vec_idx -> pi_in -> X), without branches, so that every wave
// keeps several kilobytes in flight.  The per-wave partial tiles are summed in a fixed order
// through LDS, so results do not depend on timing.
#include "hinm_internal.h"
#include "mfma_types.h"

namespace hinm {
namespace {

constexpr int kRows = 16;   // rows per workgroup
constexpr int kCols = 16;   // columns per workgroup
constexpr int kStep = 64;   // kept columns per MFMA
// private LDS slab of one wave: 64 rows x 16 columns, 8-row blocks padded so that the four lane
// groups of a transposing read fall on different banks
constexpr int kSlabBytes = 8 * 384;

__device__ __forceinline__ int slab_row_offset(int row) { return row * 32 + (row >> 3) * 128; }

__device__ __forceinline__ void wave_sync_lds() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// B operand of one step from the wave's slab: slots 8 h + 4 u .. + 3 of lane group q hold rows
// 32 h + 8 q + 4 u + (0..3) at column i; inside a 16-lane group lane i addresses row (i / 4) and
// columns 4 (i % 4) .. + 3.
__device__ __forceinline__ u32x8 read_b_operand(const uint8_t* slab, int i, int q) {
  u32x8 b;
#pragma unroll
  for (int h = 0; h < 2; ++h)
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int row = 32 * h + 8 * q + 4 * u + (i >> 2);
      const u32x2 v = lds_read_tr16(slab + slab_row_offset(row) + (i & 3) * 8);
      b[(2 * h + u) * 2] = v.x;
      b[(2 * h + u) * 2 + 1] = v.y;
    }
  return b;
}

// XMODE: 0 = any N / ld (element loads, slow), 1 = the 16 columns are inside N and rows are
// 16-byte aligned, 2 = N == 1.  KB = steps whose loads are issued together.  RBW = 16-row blocks per
// workgroup (they share the gathered B operand).
template <int DT, int NW, int XMODE, int KB, int RBW>
__global__ __launch_bounds__(NW * 64) void spmm_skinny_kernel(
    const uint16_t* __restrict__ vals, const uint8_t* __restrict__ nm_idx, const int32_t* __restrict__ vec_idx,
    const int32_t* __restrict__ pi_in, const int32_t* __restrict__ pi_out, const uint16_t* __restrict__ X,
    int64_t ldx, void* __restrict__ Y, int64_t ldy, int V, int Kv, int N, bool relu, bool out_f32) {
  __shared__ __attribute__((aligned(16))) uint8_t slab_all[NW * kSlabBytes];
  static_assert(RBW * kRows * kCols * 4 <= kSlabBytes, "partial tiles must fit the slab");

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int row0 = blockIdx.x * (kRows * RBW);  // first row of W handled here
  const int t = row0 / V;
  const int n0 = blockIdx.y * kCols;
  const int full_steps = Kv / kStep;                       // steps with all 64 columns present
  const int steps = (Kv + kStep - 1) / kStep;
  const int per_wave = (full_steps + NW - 1) / NW;
  const int s_begin = wave * per_wave;
  const int s_end = min(full_steps, s_begin + per_wave);   // this wave's contiguous range of full steps

  uint8_t* slab = slab_all + wave * kSlabBytes;
  const int i = lane & 15;   // A row / B column inside the block
  const int q = lane >> 4;   // lane group
  const uint16_t* vrow = vals + (size_t)(row0 + i) * (Kv / 2);
  const uint8_t* nrow = nm_idx + (size_t)(row0 + i) * (Kv / 8);
  const size_t vblock = (size_t)kRows * (Kv / 2);  // distance between the 16-row blocks
  const size_t nblock = (size_t)kRows * (Kv / 8);
  const int32_t* vi = vec_idx + (size_t)t * Kv;
  const bool nm_pairs_aligned = ((Kv / 8) & 1) == 0;

  // output rows of the epilogue, fetched early: element e = threadIdx.x + k * blockDim.x
  constexpr int kOutPerThread = (RBW * kRows * kCols + NW * 64 - 1) / (NW * 64);
  int64_t out_row[kOutPerThread];
#pragma unroll
  for (int k = 0; k < kOutPerThread; ++k) {
    const int e = threadIdx.x + k * NW * 64;
    const int row = min(e / kCols, RBW * kRows - 1);
    out_row[k] = pi_out ? pi_out[row0 + row] : (row0 + row);
  }

  f32x4 acc[RBW];
#pragma unroll
  for (int rb = 0; rb < RBW; ++rb) acc[rb] = f32x4{0.f, 0.f, 0.f, 0.f};

  for (int sb = s_begin; sb < s_end; sb += KB) {
    u32x4 a_reg[KB][RBW];
    int idx_reg[KB][RBW];
    int col[KB];
    u32x4 b_lo[KB], b_hi[KB];
    // Loads come back in issue order, so the short index chain vec_idx -> pi_in goes first and the
    // bulk weight stream is issued behind it; the input rows are requested as soon as their indices
    // are known and arrive while the weights are still streaming.  (Steps past the wave's range
    // are clamped to its last step and zeroed before use.)
    // phase 1: vector-index entries, then the input-channel order
#pragma unroll
    for (int u = 0; u < KB; ++u) col[u] = vi[kStep * min(sb + u, s_end - 1) + lane];
    if (pi_in) {
#pragma unroll
      for (int u = 0; u < KB; ++u) col[u] = pi_in[col[u]];
    }
    __builtin_amdgcn_sched_barrier(0);
    // phase 2: stored values and NM nibbles
#pragma unroll
    for (int u = 0; u < KB; ++u) {
      const int s = min(sb + u, s_end - 1);
      const int g0 = 16 * s + 4 * q;  // this lane's four groups
#pragma unroll
      for (int rb = 0; rb < RBW; ++rb) {
        a_reg[u][rb] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_a4*>(vrow + rb * vblock + 2 * g0));  // read once
        const uint8_t* np = nrow + rb * nblock + (g0 >> 1);
        if (nm_pairs_aligned) idx_reg[u][rb] = *reinterpret_cast<const uint16_t*>(np);
        else idx_reg[u][rb] = (int)np[0] | ((int)np[1] << 8);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    // phase 3: input rows, 16 columns wide
#pragma unroll
    for (int u = 0; u < KB; ++u) {
      const uint16_t* xr = X + (size_t)col[u] * ldx + n0;
      if constexpr (XMODE == 1) {
        // Lanes 2 j and 2 j + 1 fetch the two 16-byte halves of one row (rows j and 32 + j of the step):
        // neighbouring lanes then fall into one cache line, which halves the tag look-ups that a gather of
        // rows scattered by the input-channel order costs.
        const int c_lo = __builtin_amdgcn_ds_bpermute((lane >> 1) * 4, col[u]);
        const int c_hi = __builtin_amdgcn_ds_bpermute((32 + (lane >> 1)) * 4, col[u]);
        b_lo[u] = *reinterpret_cast<const u32x4*>(X + (size_t)c_lo * ldx + n0 + 8 * (lane & 1));
        b_hi[u] = *reinterpret_cast<const u32x4*>(X + (size_t)c_hi * ldx + n0 + 8 * (lane & 1));
      } else if constexpr (XMODE == 2) {
        b_lo[u] = u32x4{(uint32_t)xr[0], 0, 0, 0};
        b_hi[u] = u32x4{0, 0, 0, 0};
      } else {
        uint32_t w[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (n0 + e < N) w[e >> 1] |= (uint32_t)xr[e] << (16 * (e & 1));
        b_lo[u] = u32x4{w[0], w[1], w[2], w[3]};
        b_hi[u] = u32x4{w[4], w[5], w[6], w[7]};
      }
    }
    // phase 4: multiply
#pragma unroll
    for (int u = 0; u < KB; ++u) {
      const bool live = sb + u < s_end;  // wave-uniform
      if constexpr (XMODE == 1) {  // half rows: see the loads
        *reinterpret_cast<u32x4*>(slab + slab_row_offset(lane >> 1) + 16 * (lane & 1)) = b_lo[u];
        *reinterpret_cast<u32x4*>(slab + slab_row_offset(32 + (lane >> 1)) + 16 * (lane & 1)) = b_hi[u];
      } else {
        uint8_t* wr = slab + slab_row_offset(lane);
        *reinterpret_cast<u32x4*>(wr) = b_lo[u];
        *reinterpret_cast<u32x4*>(wr + 16) = b_hi[u];
      }
      wave_sync_lds();
      u32x8 b = read_b_operand(slab, i, q);
      if (!live) b = u32x8{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
      for (int rb = 0; rb < RBW; ++rb) {
        const u32x4 a = live ? a_reg[u][rb] : u32x4{0, 0, 0, 0};
        acc[rb] = smfmac_16x16x64<DT, 0>(a, b, acc[rb], idx_reg[u][rb]);
      }
      wave_sync_lds();
    }
  }

  // ---- the ragged last step (Kv % 64 != 0), done by the last wave with guarded loads -----------
  if (steps > full_steps && wave == NW - 1) {
    const int s = full_steps;
    const int groups_total = Kv / 4;
    const int g0 = 16 * s + 4 * q;
    uint32_t w[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    const int j = kStep * s + lane;
    if (j < Kv) {
      int c = vi[j];
      if (pi_in) c = pi_in[c];
      const uint16_t* xr = X + (size_t)c * ldx + n0;
      for (int e = 0; e < 16; ++e)
        if (n0 + e < N) w[e >> 1] |= (uint32_t)xr[e] << (16 * (e & 1));
    }
    uint8_t* wr = slab + slab_row_offset(lane);
    *reinterpret_cast<u32x4*>(wr) = u32x4{w[0], w[1], w[2], w[3]};
    *reinterpret_cast<u32x4*>(wr + 16) = u32x4{w[4], w[5], w[6], w[7]};
    wave_sync_lds();
    const u32x8 b = read_b_operand(slab, i, q);
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb) {
      u32x4 a = {0, 0, 0, 0};
      int idx = 0;
      const uint16_t* vp = vrow + rb * vblock + 2 * g0;
      const uint8_t* np = nrow + rb * nblock + (g0 >> 1);
      if (g0 + 4 <= groups_total) {
        a = *reinterpret_cast<const u32x4_a4*>(vp);
        idx = (int)np[0] | ((int)np[1] << 8);
      } else if (g0 + 2 <= groups_total) {  // Kv % 8 == 0: the tail holds whole pairs of groups
        const u32x2 half = *reinterpret_cast<const u32x2_a4*>(vp);
        a = u32x4{half.x, half.y, 0, 0};
        idx = (int)np[0];
      }
      acc[rb] = smfmac_16x16x64<DT, 0>(a, b, acc[rb], idx);
    }
  }

  // ---- fixed-order reduction over the waves, epilogue ---------------------------------------
  // D layout: lane holds column lane % 16, rows 4 * (lane / 16) + reg.
  // (the slab is free now; its first kilobytes take this wave's partial tiles)
  wave_sync_lds();
  float* partial = reinterpret_cast<float*>(slab);
#pragma unroll
  for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
    for (int reg = 0; reg < 4; ++reg) partial[(16 * rb + 4 * q + reg) * kCols + i] = acc[rb][reg];
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kOutPerThread; ++k) {
    const int e = threadIdx.x + k * NW * 64;
    if (e < RBW * kRows * kCols) {
      float sum = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) sum += reinterpret_cast<const float*>(slab_all + w * kSlabBytes)[e];
      if (relu) sum = sum > 0.f ? sum : 0.f;
      const int c = e % kCols;
      if (n0 + c < N) {
        if (out_f32) static_cast<float*>(Y)[out_row[k] * ldy + n0 + c] = sum;
        else static_cast<uint16_t*>(Y)[out_row[k] * ldy + n0 + c] = float_to_bits<DT>(sum);
      }
    }
  }
}

template <int DT, int NW, int KB, int RBW>
void launch_modes(const SpmmArgs& a, hipStream_t stream) {
  auto v = static_cast<const uint16_t*>(a.vals);
  auto x = static_cast<const uint16_t*>(a.X);
  const int col_blocks = (a.N + kCols - 1) / kCols;
  const int full_blocks = (a.ldx % 8 == 0) ? a.N / kCols : 0;  // column blocks eligible for vector loads
#define HINM_SKINNY(MODE, GRID_Y, X_PTR, Y_OFF)                                                                 \
  spmm_skinny_kernel<DT, NW, MODE, KB, RBW><<<dim3(a.s.M / (kRows * RBW), GRID_Y), NW * 64, 0, stream>>>(       \
      v, a.nm_idx, a.vec_idx, a.pi_in, a.pi_out, X_PTR, a.ldx,                                                  \
      a.out_f32 ? static_cast<void*>(static_cast<float*>(a.Y) + (Y_OFF))                                        \
                : static_cast<void*>(static_cast<uint16_t*>(a.Y) + (Y_OFF)),                                    \
      a.ldy, a.s.V, a.s.Kv, a.N - (Y_OFF), a.relu, a.out_f32)
  if (a.N == 1) {
    HINM_SKINNY(2, 1, x, 0);
    return;
  }
  if (full_blocks > 0) HINM_SKINNY(1, full_blocks, x, 0);
  if (col_blocks > full_blocks) {
    const int off = full_blocks * kCols;  // ragged remainder: shift the column origin
    HINM_SKINNY(0, col_blocks - full_blocks, x + off, off);
  }
#undef HINM_SKINNY
}

template <int DT, int RBW>
void launch_waves(const SpmmArgs& a, hipStream_t stream) {
  const int full_steps = a.s.Kv / kStep;
  // Prefer one batch per wave (every load of the wave in flight at once): waves x batch >= steps.
  if (full_steps <= 4) launch_modes<DT, 1, 4, RBW>(a, stream);
  else if (full_steps <= 16) launch_modes<DT, 4, 4, RBW>(a, stream);
  else if (full_steps <= 32) launch_modes<DT, 8, 4, RBW>(a, stream);
  else if (full_steps <= 64) launch_modes<DT, 16, 4, RBW>(a, stream);
  else launch_modes<DT, 16, 6, RBW>(a, stream);
}

}  // namespace

bool spmm_skinny_supported(const SpmmArgs& a) {
  return a.s.V % 16 == 0 && (a.N + 15) / 16 <= 65535;
}

hipError_t launch_spmm_skinny(const SpmmArgs& a, hipStream_t stream) {
  // Two 16-row blocks per workgroup share the gathered input rows; used when there are enough
  // rows that the grid still fills the chip in one round.
  const bool two = (a.s.V % 32 == 0) && (a.s.M / 32 >= 320);
  if (a.s.dtype == HINM_F16) {
    if (two) launch_waves<HINM_F16, 2>(a, stream);
    else launch_waves<HINM_F16, 1>(a, stream);
  } else {
    if (two) launch_waves<HINM_BF16, 2>(a, stream);
    else launch_waves<HINM_BF16, 1>(a, stream);
  }
  return hipGetLastError();
}

}  // namespace hinm
