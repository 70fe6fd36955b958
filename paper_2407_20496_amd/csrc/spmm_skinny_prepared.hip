// HiNM product for few columns (N <= 32, decode-like shapes) from the device-tuned layer form
// (arXiv 2407.20496, Section 3.2; layout in prepared_layout.h).
//
// The work is one pass over the packed weights, bound by HBM, and HBM only delivers its bandwidth
// when (nearly) the whole weight matrix is requested at once.  One workgroup owns one 32-row block
// of one tile; its waves take the tile's 64-column steps round-robin and every wave issues ALL the
// loads of its steps before it uses the first: the gather-table entries first (a short dependent
// chain), then the stored values and NM nibbles (already in MFMA lane order: every load instruction
// reads one contiguous kilobyte, straight into the A operand of the 32x32x32 sparse MFMA), then the
// input rows named by the table.  The input rows pass through a private LDS slab and come back
// transposed as the B operand; accumulation is fp32.  The per-wave partial tiles are added in a
// fixed order through LDS, so results do not depend on timing.  No workspace, no second kernel.
//
// For a single column (N = 1) the whole input vector is small: the workgroup copies it into LDS once
// (requested before everything else, so it arrives while the weight stream is in flight) and the
// rows named by the table are then picked from LDS.  Picking them from global memory instead costs
// one address-unit cycle per lane and load (64 different lines), queued behind the weight stream.
#include "hinm_internal.h"
#include "mfma_types.h"
#include "prepared_layout.h"

namespace hinm {
namespace {

constexpr int kSlabBytes = 64 * 64;  // 64 gathered rows x 32 columns x 16 bit, per wave
constexpr int kXPieces = 2;          // N = 1: 16-byte pieces of the input vector a thread copies into LDS
constexpr int kXLdsMaxBytes = 64 * 1024;

__device__ __forceinline__ void wave_sync_lds() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Two 1024-thread workgroups fit a compute unit only at 64 registers per lane (8 waves per SIMD):
// the configurations that are a few registers away from that are held to it, because a grid of
// T * RB workgroups that needs a second round costs more than the registers give.
template <int NWV, int KB, int NG, int RBW, bool XS>
constexpr int min_waves_per_simd() {
  return (NWV == 16 && KB == 2 && RBW == 1 && NG <= 2 && !XS) ? 8 : 1;
}

// NWV waves per workgroup, KB steps per wave and batch (a wave with more steps runs several batches),
// NG = 16-byte pieces fetched per input row (8 columns each), XS = input vector staged in LDS
template <int DT, int NWV, int KB, int NG, int RBW, bool XS>
__global__ __launch_bounds__(NWV * 64, (min_waves_per_simd<NWV, KB, NG, RBW, XS>())) void spmm_skinny_prepared_kernel(
    const uint8_t* __restrict__ prep_blocks, const int32_t* __restrict__ gather, const int32_t* __restrict__ out_rows,
    const uint16_t* __restrict__ X, int64_t ldx, void* __restrict__ Y, int64_t ldy, int RB, int S64, int N, int K,
    bool relu, bool out_f32) {
  // NWV slabs (later NWV x 32 x N floats), then the input vector when x_in_lds
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int rb = blockIdx.x * RBW;  // first of the RBW row blocks this workgroup owns
  const int t = blockIdx.y;
  const int Kp = S64 * 64;
  const int V = 32 * RB;

  const int32_t* gt = gather + (size_t)t * Kp;
  const uint8_t* a_blocks = prep_blocks + ((size_t)t * S64 * RB + rb) * kPrepBlockBytes;  // step s: + s * RB blocks
  const size_t step_stride = (size_t)RB * kPrepBlockBytes;
  uint8_t* slab = lds + wave * kSlabBytes;
  const int granules = (N + 7) / 8;  // 16-byte pieces of an input row that hold real columns (<= NG)
  // slab rows are 64 bytes; the pieces beyond NG stay zero for the whole kernel
  if (NG < 4) {
#pragma unroll
    for (int p = NG; p < 4; ++p) *reinterpret_cast<u32x4*>(slab + lane * 64 + p * 16) = u32x4{0, 0, 0, 0};
  }
  const bool single_column = (N == 1);
  // XS (N = 1, contiguous X, K % 8 == 0): elements 8 c .. 8 c + 7 of the input vector go to x_lds as
  // one 16-byte piece; every thread moves up to kXPieces pieces (the launcher checks that this covers
  // K).  No branch around a load: loads in separate blocks would each wait for the one before.
  static_assert(!XS || (NG == 1 && RBW == 1), "the input vector is staged for single columns only");
  uint16_t* x_lds = reinterpret_cast<uint16_t*>(lds + NWV * kSlabBytes);
  u32x4 x_mine[XS ? kXPieces : 1];
  if constexpr (XS) {
#pragma unroll
    for (int r = 0; r < kXPieces; ++r) {
      const int c = min((int)threadIdx.x + r * NWV * 64, K / 8 - 1);  // past the end: re-read the last piece, unused
      x_mine[r] = *reinterpret_cast<const u32x4*>(X + 8 * (size_t)c);
    }
  }

  const int i32 = lane & 31;
  const int qh = lane >> 5;
  const int i16 = lane & 15;
  // output rows of the epilogue, fetched early
  const int my_row = threadIdx.x & 31;
  int64_t out_row[RBW];
#pragma unroll
  for (int k = 0; k < RBW; ++k) out_row[k] = out_rows[t * V + 32 * (rb + k) + my_row];

  f32x16 acc[RBW];
#pragma unroll
  for (int k = 0; k < RBW; ++k)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[k][e] = 0.f;

  struct Batch {
    u32x4 a_val[KB][RBW][2];
    int a_idx[KB][RBW];
    int row[KB];
  };
  // loads return in issue order: the short index chain goes first, the bulk weight stream behind it
  // (steps past the end are clamped: loaded again, multiplied by zero)
  auto load_batch = [&](int sb, Batch& bt) {
#pragma unroll
    for (int u = 0; u < KB; ++u) bt.row[u] = gt[64 * min(sb + u * NWV, S64 - 1) + lane];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < KB; ++u) {
      const uint8_t* blk = a_blocks + (size_t)min(sb + u * NWV, S64 - 1) * step_stride;
#pragma unroll
      for (int k = 0; k < RBW; ++k) {
        bt.a_val[u][k][0] = *reinterpret_cast<const u32x4*>(blk + k * kPrepBlockBytes + lane * 16);
        bt.a_val[u][k][1] = *reinterpret_cast<const u32x4*>(blk + k * kPrepBlockBytes + 1024 + lane * 16);
        bt.a_idx[u][k] = *reinterpret_cast<const int*>(blk + k * kPrepBlockBytes + kPrepIdxOffset + lane * 4);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  auto multiply_batch = [&](int sb, const Batch& bt) {
    u32x4 b_reg[KB][NG];
    // input rows: up to 32 columns (four 16-byte pieces) per gathered row; padded kept columns read zeros
#pragma unroll
    for (int u = 0; u < KB; ++u) {
      const int g = bt.row[u];
      const uint16_t* xr = X + (size_t)max(g, 0) * ldx;
#pragma unroll
      for (int p = 0; p < NG; ++p) b_reg[u][p] = u32x4{0, 0, 0, 0};
      if constexpr (XS) {
        if (g >= 0) b_reg[u][0] = u32x4{(uint32_t)x_lds[g], 0, 0, 0};
      } else if (single_column) {
        if (g >= 0) b_reg[u][0] = u32x4{(uint32_t)xr[0], 0, 0, 0};
      } else {
#pragma unroll
        for (int p = 0; p < NG; ++p)
          if (g >= 0 && p < granules) b_reg[u][p] = *reinterpret_cast<const u32x4*>(xr + 8 * p);
      }
    }
#pragma unroll
    for (int u = 0; u < KB; ++u) {
      const bool live = sb + u * NWV < S64;  // wave-uniform
#pragma unroll
      for (int p = 0; p < NG; ++p) *reinterpret_cast<u32x4*>(slab + lane * 64 + p * 16) = b_reg[u][p];
      wave_sync_lds();
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        // B slots 8 h + 4 v .. + 3 of lane group qb <- rows 16 h + 8 qb + 4 v + (0..3) of the substep;
        // lanes 0..15 / 16..31 of a 32-lane half read columns 0..15 / 16..31
        u32x8 b;
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int v = 0; v < 2; ++v) {
            const int r = 32 * sub + 16 * h + 8 * qh + 4 * v + (i16 >> 2);
            const u32x2 w = lds_read_tr16(slab + r * 64 + (i32 & 16) * 2 + (i16 & 3) * 8);
            b[(2 * h + v) * 2] = w.x;
            b[(2 * h + v) * 2 + 1] = w.y;
          }
        if (!live) b = u32x8{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int k = 0; k < RBW; ++k) {
          const u32x4 a = live ? bt.a_val[u][k][sub] : u32x4{0, 0, 0, 0};
          if (sub == 0) acc[k] = smfmac_32x32x32<DT, 0>(a, b, acc[k], bt.a_idx[u][k]);
          else acc[k] = smfmac_32x32x32<DT, 1>(a, b, acc[k], bt.a_idx[u][k]);
        }
      }
      wave_sync_lds();
    }
  };
  if constexpr (XS) {
    Batch bt;
    load_batch(wave, bt);  // every wave, also one without steps: the barrier below is for all of them
    // the input vector was requested first, so this waits for it alone, not for the weight stream
#pragma unroll
    for (int r = 0; r < kXPieces; ++r) {
      const int c = threadIdx.x + r * NWV * 64;
      if (8 * c < K) *reinterpret_cast<u32x4*>(x_lds + 8 * c) = x_mine[r];
    }
    __syncthreads();
    for (int sb = wave; sb < S64; sb += NWV * KB) {
      if (sb != wave) load_batch(sb, bt);
      multiply_batch(sb, bt);
    }
  } else {
    for (int sb = wave; sb < S64; sb += NWV * KB) {
      Batch bt;
      load_batch(sb, bt);
      multiply_batch(sb, bt);
    }
  }

  // ---- sum over the waves (fixed order), epilogue ------------------------------------------------------
  // D layout: lane holds column lane % 32, rows 8 * (reg / 4) + 4 * (lane / 32) + reg % 4.
  __syncthreads();  // slabs are no longer needed
  float* wave_part = reinterpret_cast<float*>(lds);  // [NWV][RBW][32][N]
  const int elems = RBW * 32 * N;
  if (i32 < N) {
#pragma unroll
    for (int k = 0; k < RBW; ++k)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int r = 8 * (e >> 2) + 4 * qh + (e & 3);
        wave_part[wave * elems + (k * 32 + r) * N + i32] = acc[k][e];
      }
  }
  __syncthreads();
  // thread -> (row = threadIdx % 32, columns threadIdx / 32, + blockDim / 32, ...)
#pragma unroll
  for (int k = 0; k < RBW; ++k)
    for (int c = threadIdx.x >> 5; c < N; c += (NWV * 64) >> 5) {
      const int e = (k * 32 + my_row) * N + c;
      float sum = 0.f;
#pragma unroll
      for (int w = 0; w < NWV; ++w) sum += wave_part[w * elems + e];
      if (relu) sum = sum > 0.f ? sum : 0.f;
      if (out_f32) static_cast<float*>(Y)[out_row[k] * ldy + c] = sum;
      else static_cast<uint16_t*>(Y)[out_row[k] * ldy + c] = float_to_bits<DT>(sum);
    }
}

template <int DT, int NWV, int KB, int NG, int RBW, bool XS>
void launch_kernel(const PreparedArgs& a, const PreparedLayout& L, size_t lds_bytes, hipStream_t stream) {
  const uint8_t* base = static_cast<const uint8_t*>(a.prepared);
  constexpr auto kernel = spmm_skinny_prepared_kernel<DT, NWV, KB, NG, RBW, XS>;
  if (a.plan) {
    plan_record(a.plan, "spmm_skinny_prepared_kernel<DT=%d,NWV=%d,KB=%d,NG=%d,RBW=%d,XS=%d> grid=%dx%d block=%d lds=%d", DT,
                NWV, KB, NG, RBW, (int)XS, L.RB / RBW, L.T, NWV * 64, (int)lds_bytes);
    return;
  }
  if (raise_lds_limit<kernel>((int)(NWV * kSlabBytes + kXLdsMaxBytes)) != hipSuccess)
    return;  // the error stays pending and is reported by the caller's hipGetLastError
  kernel<<<dim3(L.RB / RBW, L.T), NWV * 64, lds_bytes, stream>>>(
      base + L.a_offset, reinterpret_cast<const int32_t*>(base + L.gather_offset),
      reinterpret_cast<const int32_t*>(base + L.pi_out_offset), static_cast<const uint16_t*>(a.X), a.ldx, a.Y, a.ldy,
      L.RB, L.S, a.N, a.s.K, a.relu, a.out_f32);
}

template <int DT, int NWV, int KB, int NG, int RBW>
void launch_one(const PreparedArgs& a, const PreparedLayout& L, hipStream_t stream) {
  const size_t slabs = (size_t)NWV * kSlabBytes;
  const size_t parts = (size_t)NWV * RBW * 32 * a.N * 4;
  const size_t front = slabs > parts ? slabs : parts;
  if constexpr (NG == 1 && RBW == 1) {
    // staging the input vector is worth its workgroup barrier once a wave gathers for more than two steps
    const size_t x_bytes = ((size_t)a.s.K * 2 + 15) / 16 * 16;
    const bool stage_x = a.N == 1 && a.ldx == 1 && a.s.K % 8 == 0 && L.S > 2 * NWV &&
                         (reinterpret_cast<uintptr_t>(a.X) & 15u) == 0 && a.s.K <= 8 * kXPieces * NWV * 64 &&
                         x_bytes <= (size_t)kXLdsMaxBytes;
    if (stage_x) {
      launch_kernel<DT, NWV, KB, NG, RBW, true>(a, L, front > slabs + x_bytes ? front : slabs + x_bytes, stream);
      return;
    }
  }
  launch_kernel<DT, NWV, KB, NG, RBW, false>(a, L, front, stream);
}

template <int DT, int NG, int RBW>
void launch_rbw(const PreparedArgs& a, hipStream_t stream) {
  const PreparedLayout L = prepared_layout(a.s);
  // waves x batch >= steps where possible: every load of the workgroup is in flight at once
  // batch sizes are capped so that a 1024-thread workgroup (128 registers per lane) does not spill
  constexpr int KB_BIG = (RBW == 1) ? (NG == 1 ? 6 : 4) : (NG <= 2 ? 3 : 2);
  constexpr int KB_MID = KB_BIG < 4 ? KB_BIG : 4;
  if (L.S <= 4) launch_one<DT, 4, 1, NG, RBW>(a, L, stream);
  else if (L.S <= 16) launch_one<DT, 8, 2, NG, RBW>(a, L, stream);
  else if (L.S <= 32) launch_one<DT, 16, 2, NG, RBW>(a, L, stream);
  else if (L.S <= 64) launch_one<DT, 16, KB_MID, NG, RBW>(a, L, stream);
  else launch_one<DT, 16, KB_BIG, NG, RBW>(a, L, stream);
}

template <int DT, int NG>
void launch_ng(const PreparedArgs& a, hipStream_t stream) {
  // Two row blocks per workgroup share the gathered input rows; worth it when rows are wide enough
  // for the gather to matter and the grid still covers the chip.
  const PreparedLayout L = prepared_layout(a.s);
  const bool two = (L.RB % 2 == 0) && (NG >= 2) && ((int64_t)L.T * L.RB / 2 >= 160);
  if (two) launch_rbw<DT, NG, 2>(a, stream);
  else launch_rbw<DT, NG, 1>(a, stream);
}

template <int DT>
void launch_dt(const PreparedArgs& a, hipStream_t stream) {
  if (a.N <= 8) launch_ng<DT, 1>(a, stream);
  else if (a.N <= 16) launch_ng<DT, 2>(a, stream);
  else launch_ng<DT, 4>(a, stream);
}

}  // namespace

size_t skinny_prepared_workspace_bytes(const hinm_shape&, int) { return 0; }

hipError_t launch_spmm_skinny_prepared(const PreparedArgs& a, hipStream_t stream) {
  if (a.s.dtype == HINM_F16) launch_dt<HINM_F16>(a, stream);
  else launch_dt<HINM_BF16>(a, stream);
  if (a.plan) return hipSuccess;  // a dry run launched nothing
  return hipGetLastError();
}

}  // namespace hinm
