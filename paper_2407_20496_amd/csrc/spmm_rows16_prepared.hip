// HiNM product for few columns from the device-tuned layer form, 16 output channels per workgroup
// (arXiv 2407.20496, Section 3.2; layout in prepared_layout.h).
//
// spmm_skinny_prepared_kernel gives every workgroup a 32-row block of a tile; a layer with few tiles
// (4096 rows at V = 128: 128 blocks) then leaves half of the 256 compute units idle.  This kernel
// halves the granularity: one workgroup owns 16 rows and a block of 16 columns and uses the 16x16x64
// sparse MFMA, whose A operand for lane (row i, lane group q) is exactly the 16 bytes the prepared
// block holds for lane 32 (q % 2) + i of substep q / 2 -- so the prepared form is read in place, four
// contiguous 256-byte segments per step.  Otherwise it works like the canonical-array kernel for few
// columns: the waves split the tile's steps into contiguous ranges, every wave issues all loads of a
// batch of steps before it uses the first, gathered rows pass through a private LDS slab and come
// back transposed, and the per-wave partial tiles are added in a fixed order through LDS.
#include "hinm_internal.h"
#include "mfma_types.h"
#include "prepared_layout.h"
#include "direct_lds.h"

namespace hinm {
namespace {

constexpr int kRows = 16;   // rows per workgroup
constexpr int kCols = 16;   // columns per workgroup
constexpr int kStep = 64;   // kept columns per MFMA
// private LDS slab of one wave: 64 rows x 16 columns, 8-row blocks padded so that the four lane
// groups of a transposing read fall on different banks
constexpr int kSlabBytes = 8 * 384;
constexpr int kXPieces = 4;                 // XMODE 3: 16-byte pieces of the input vector per thread
constexpr int kXLdsMaxBytes = 48 * 1024;

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

// XMODE: 0 = any N / ld (element loads, slow), 1 = rows are 16-byte aligned (ld % 8 == 0; columns beyond N
// are computed on whatever the padding holds and never stored), 2 = N == 1, 3 = N == 1 with the input vector staged in LDS (a 64-lane gather of 2-byte
// elements from global memory costs the address unit one cycle per lane; the vector is small, so the
// workgroup copies it whole, requested before everything else, and picks from LDS), 4 = 16 columns with all K
// input rows resident in LDS (32 bytes each, copied once per workgroup with direct-to-LDS loads: rows
// scattered by the input-channel order otherwise cost a whole 128-byte line each on the way from L2).
// KB = steps whose loads are issued together.  RBW = 1: the workgroup owns 16 rows; RBW = 2: both halves of a
// 32-row block, which share the gathered input rows; RBW = 4: two neighbouring 32-row blocks of one tile (V % 64 == 0).
// CB = 16-column blocks per workgroup (XMODE 1 only): with two or four, a step's weights, gather entries and
// cache lines of input rows serve 32 or 64 columns.
template <int DT, int NW, int XMODE, int KB, int RBW, int CB = 1>
__global__ __launch_bounds__(NW * 64) void spmm_rows16_prepared_kernel(
    const uint8_t* __restrict__ prep_blocks, const int32_t* __restrict__ gather, const int32_t* __restrict__ out_rows,
    const uint8_t* __restrict__ zeros, const uint16_t* __restrict__ X, int64_t ldx, void* __restrict__ Y, int64_t ldy,
    int V, int RB, int S64, int N, int K, bool relu, bool out_f32) {
  // a wave's slab holds its gathered rows, later its partial tiles (a kilobyte per 16 rows)
  constexpr int kTiles = RBW * CB;  // 16 x 16 output tiles of the workgroup
  constexpr int kSlab = (XMODE != 4 && kTiles * kRows * kCols * 4 > kSlabBytes) ? kTiles * kRows * kCols * 4 : kSlabBytes;
  __shared__ __attribute__((aligned(16))) uint8_t slab_all[NW * kSlab];
  extern __shared__ __attribute__((aligned(16))) uint16_t x_lds[];  // XMODE 3: K elements + 8 zeros; 4: K rows + a zero row
  static_assert(RBW == 1 || RBW == 2 || RBW == 4, "half a 32-row block, one, or two neighbours");
  static_assert(CB == 1 || ((CB == 2 || CB == 4) && XMODE == 1), "several column blocks only with paired-lane vector loads");
  uint8_t* x_bytes = reinterpret_cast<uint8_t*>(x_lds);

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int row0 = blockIdx.x * (kRows * RBW);  // first row of the layer handled here
  const int t = row0 / V;
  const int rb32 = (row0 % V) / 32;     // 32-row block of the prepared form that holds these rows
  const int hf = (row0 % 32) / 16;      // ... and which half of it (0 when the workgroup owns both)
  const int n0 = blockIdx.y * (kCols * CB);
  const int per_wave = (S64 + NW - 1) / NW;
  const int s_begin = wave * per_wave;
  const int s_end = min(S64, s_begin + per_wave);  // this wave's contiguous range of steps (all steps are full: padded)

  uint8_t* slab = slab_all + wave * kSlab;
  const int i = lane & 15;   // A row / B column inside the block
  const int q = lane >> 4;   // lane group: groups 4 q .. 4 q + 3 of the step = substep q / 2, quad q % 2
  // this lane's 16 bytes inside a (tile, step, row block) block of the prepared form, and its index word
  const int lane32 = 32 * (q & 1) + 16 * hf + i;
  const uint8_t* a_lane = prep_blocks + ((size_t)t * S64 * RB + rb32) * kPrepBlockBytes + (q >> 1) * 1024 + lane32 * 16;
  const uint8_t* idx_lane = prep_blocks + ((size_t)t * S64 * RB + rb32) * kPrepBlockBytes + kPrepIdxOffset + lane32 * 4;
  const size_t step_stride = (size_t)RB * kPrepBlockBytes;
  const int32_t* gt = gather + (size_t)t * S64 * 64;

  // output rows of the epilogue, fetched early: element e = threadIdx.x + k * blockDim.x
  constexpr int kOutPerThread = (kTiles * kRows * kCols + NW * 64 - 1) / (NW * 64);
  int64_t out_row[kOutPerThread];
#pragma unroll
  for (int k = 0; k < kOutPerThread; ++k) {
    const int e = min((int)threadIdx.x + k * NW * 64, kTiles * kRows * kCols - 1);
    const int row = (e / kCols) % (RBW * kRows);  // element e: column block, then row, then column
    out_row[k] = out_rows[row0 + row];
  }

  f32x4 acc[CB][RBW];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb)
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb) acc[cb][rb] = f32x4{0.f, 0.f, 0.f, 0.f};

  // XMODE 3: this thread's 16-byte pieces of the input vector (requested now, written to LDS after the first
  // batch of weight loads has been issued); every wave passes the barrier exactly once
  u32x4 x_mine[kXPieces];
  bool x_staged = XMODE != 3 && XMODE != 4;
  if constexpr (XMODE == 3) {
#pragma unroll
    for (int r = 0; r < kXPieces; ++r) {
      const int piece = min((int)threadIdx.x + r * NW * 64, K / 8 - 1);  // beyond the vector: its last piece again
      x_mine[r] = reinterpret_cast<const u32x4*>(X)[piece];
    }
  }
  // XMODE 4: wave-wide copies of 32 rows x 32 bytes (lane l: row l / 2, half l % 2), requested before everything
  // else; rows past K repeat the last row and are never addressed; the zero row sits behind the last copy
  const int x_copies = (K + 31) / 32;
  const int x_zero_row = 32 * x_copies;
  if constexpr (XMODE == 4) {
    for (int j = wave; j < x_copies; j += NW) {
      const int r = min(32 * j + (lane >> 1), K - 1);
      copy16_to_lds(X + (size_t)r * ldx + n0 + 8 * (lane & 1), x_bytes + (size_t)j * 1024);
    }
    if (threadIdx.x < 8) reinterpret_cast<uint32_t*>(x_bytes + (size_t)x_zero_row * 32)[threadIdx.x] = 0u;
  }
  auto stage_x = [&]() {
    if constexpr (XMODE == 4) {
      wait_copies_outstanding<0>();  // this wave's copies (and its other loads) have landed
      __syncthreads();               // ... and everyone's
    }
    if constexpr (XMODE == 3) {
#pragma unroll
      for (int r = 0; r < kXPieces; ++r) {
        const int piece = (int)threadIdx.x + r * NW * 64;
        if (piece < K / 8) reinterpret_cast<u32x4*>(x_lds)[piece] = x_mine[r];
      }
      if (threadIdx.x < 8) x_lds[K + threadIdx.x] = 0;  // where padded kept columns read
      __syncthreads();
    }
    x_staged = true;
  };

  // XMODE 1: whether this lane's 16-byte piece of column block cb lies inside the row (ldx % 8 == 0)
  bool piece_in_row[CB];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) piece_in_row[cb] = n0 + kCols * cb + 8 * (lane & 1) + 8 <= (int)ldx;
  for (int sb = s_begin; sb < s_end; sb += KB) {
    u32x4 a_reg[KB][RBW];
    int idx_reg[KB][RBW];
    int col[KB];
    u32x4 b_lo[KB][CB], b_hi[KB][CB];
    // Loads come back in issue order: the gather-table entries go first, the bulk weight stream is issued
    // behind them, and the input rows are requested as soon as their indices are known and arrive while the
    // weights are still streaming.  (Steps past the wave's range are clamped to its last step and zeroed
    // before use.)
    // phase 1: gather-table entries (vector index composed with the input-channel order; -1 = padding)
#pragma unroll
    for (int u = 0; u < KB; ++u) col[u] = gt[kStep * min(sb + u, s_end - 1) + lane];
    __builtin_amdgcn_sched_barrier(0);
    // phase 2: stored values and NM nibbles, 16 bytes + one index word per lane and step
#pragma unroll
    for (int u = 0; u < KB; ++u) {
      const size_t off = (size_t)min(sb + u, s_end - 1) * step_stride;
#pragma unroll
      for (int rb = 0; rb < RBW; ++rb) {  // the second half sits 16 lanes further in the block
        // 16-row block rb: half rb % 2 of 32-row block rb / 2 (the second half sits 16 lanes further); the
        // weights are read once, so they are kept from displacing the input rows and tables in the caches
        const size_t blk = (size_t)(rb >> 1) * kPrepBlockBytes;
        a_reg[u][rb] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(a_lane + off + blk + (rb & 1) * 256));
        const uint32_t word = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(idx_lane + off + blk + (rb & 1) * 64));
        idx_reg[u][rb] = (int)((q >> 1) ? (word >> 16) : (word & 0xFFFFu));
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    if (!x_staged) stage_x();
    // phase 3: input rows, 16 columns wide
#pragma unroll
    for (int u = 0; u < KB; ++u) {
      const uint16_t* xr = (col[u] >= 0) ? X + (size_t)col[u] * ldx + n0 : reinterpret_cast<const uint16_t*>(zeros);
      if constexpr (XMODE == 4) {
        const uint8_t* xl = x_bytes + (size_t)(col[u] >= 0 ? col[u] : x_zero_row) * 32;
        b_lo[u][0] = *reinterpret_cast<const u32x4*>(xl);
        b_hi[u][0] = *reinterpret_cast<const u32x4*>(xl + 16);
      } else if constexpr (XMODE == 3) {
        b_lo[u][0] = u32x4{(uint32_t)x_lds[col[u] >= 0 ? col[u] : K], 0, 0, 0};
        b_hi[u][0] = u32x4{0, 0, 0, 0};
      } else if constexpr (XMODE == 1) {
        // Lanes 2 j and 2 j + 1 fetch the two 16-byte halves of one row (rows j and 32 + j of the step):
        // neighbouring lanes then fall into one cache line, which halves the tag look-ups that a gather of
        // rows scattered by the input-channel order costs.
        const int c_lo = __builtin_amdgcn_ds_bpermute((lane >> 1) * 4, col[u]);
        const int c_hi = __builtin_amdgcn_ds_bpermute((32 + (lane >> 1)) * 4, col[u]);
        // (a piece of a ragged last block may lie past the end of the row: its columns are beyond N then, and
        // it reads the zero row instead; whatever else a piece holds beyond N never reaches a stored column)
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
          const uint16_t* r_lo = (c_lo >= 0 && piece_in_row[cb]) ? X + (size_t)c_lo * ldx + n0 + kCols * cb : reinterpret_cast<const uint16_t*>(zeros);
          const uint16_t* r_hi = (c_hi >= 0 && piece_in_row[cb]) ? X + (size_t)c_hi * ldx + n0 + kCols * cb : reinterpret_cast<const uint16_t*>(zeros);
          b_lo[u][cb] = *reinterpret_cast<const u32x4*>(r_lo + 8 * (lane & 1));
          b_hi[u][cb] = *reinterpret_cast<const u32x4*>(r_hi + 8 * (lane & 1));
        }
      } else if constexpr (XMODE == 2) {
        b_lo[u][0] = u32x4{(uint32_t)xr[0], 0, 0, 0};
        b_hi[u][0] = u32x4{0, 0, 0, 0};
      } else {
        uint32_t w[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (n0 + e < N) w[e >> 1] |= (uint32_t)xr[e] << (16 * (e & 1));
        b_lo[u][0] = u32x4{w[0], w[1], w[2], w[3]};
        b_hi[u][0] = u32x4{w[4], w[5], w[6], w[7]};
      }
    }
    // phase 4: multiply
#pragma unroll
    for (int u = 0; u < KB; ++u) {
      const bool live = sb + u < s_end;  // wave-uniform
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) {
        if constexpr (XMODE == 1) {  // half rows: see the loads
          *reinterpret_cast<u32x4*>(slab + slab_row_offset(lane >> 1) + 16 * (lane & 1)) = b_lo[u][cb];
          *reinterpret_cast<u32x4*>(slab + slab_row_offset(32 + (lane >> 1)) + 16 * (lane & 1)) = b_hi[u][cb];
        } else {
          uint8_t* wr = slab + slab_row_offset(lane);
          *reinterpret_cast<u32x4*>(wr) = b_lo[u][cb];
          *reinterpret_cast<u32x4*>(wr + 16) = b_hi[u][cb];
        }
        wave_sync_lds();
        u32x8 b = read_b_operand(slab, i, q);
        if (!live) b = u32x8{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int rb = 0; rb < RBW; ++rb) {
          const u32x4 a = live ? a_reg[u][rb] : u32x4{0, 0, 0, 0};
          acc[cb][rb] = smfmac_16x16x64<DT, 0>(a, b, acc[cb][rb], idx_reg[u][rb]);
        }
        wave_sync_lds();
      }
    }
  }

  if (!x_staged) stage_x();  // a wave without steps still owes the barrier

  // ---- fixed-order reduction over the waves, epilogue ---------------------------------------
  // D layout: lane holds column lane % 16, rows 4 * (lane / 16) + reg.
  // (the slab is free now; its first kilobytes take this wave's partial tiles)
  wave_sync_lds();
  // XMODE 4: the partial tiles (a kilobyte each) go where the input rows were, once nobody reads them
  constexpr int kPartialStride = (XMODE == 4) ? kTiles * kRows * kCols * 4 : kSlab;
  if constexpr (XMODE == 4) __syncthreads();
  uint8_t* partial_all = (XMODE == 4) ? x_bytes : slab_all;
  float* partial = reinterpret_cast<float*>(partial_all + wave * kPartialStride);
#pragma unroll
  for (int cb = 0; cb < CB; ++cb)
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
      for (int reg = 0; reg < 4; ++reg) partial[(16 * (cb * RBW + rb) + 4 * q + reg) * kCols + i] = acc[cb][rb][reg];
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kOutPerThread; ++k) {
    const int e = threadIdx.x + k * NW * 64;
    if (e < kTiles * kRows * kCols) {
      float sum = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) sum += reinterpret_cast<const float*>(partial_all + w * kPartialStride)[e];
      if (relu) sum = sum > 0.f ? sum : 0.f;
      const int c = kCols * (e / (RBW * kRows * kCols)) + e % kCols;
      if (n0 + c < N) {
        if (out_f32) static_cast<float*>(Y)[out_row[k] * ldy + n0 + c] = sum;
        else static_cast<uint16_t*>(Y)[out_row[k] * ldy + n0 + c] = float_to_bits<DT>(sum);
      }
    }
  }
}

template <int DT, int NW, int KB, int RBW>
void launch_modes(const PreparedArgs& a, const PreparedLayout& L, int blocks_per_wg, hipStream_t stream) {
  const uint8_t* base = static_cast<const uint8_t*>(a.prepared);
  auto x = static_cast<const uint16_t*>(a.X);
  const int col_blocks = (a.N + kCols - 1) / kCols;
#define HINM_ROWS16(MODE, GRID_Y, X_PTR, Y_OFF, LDS) HINM_ROWS16_CB(MODE, 1, KB, GRID_Y, X_PTR, Y_OFF, LDS)
#define HINM_ROWS16_CB(MODE, CBV, KBV, GRID_Y, X_PTR, Y_OFF, LDS)                                                \
  if (a.plan)                                                                                                    \
    plan_record(a.plan, "spmm_rows16_prepared_kernel<DT=%d,NW=%d,XMODE=%d,KB=%d,RBW=%d,CB=%d> grid=%dx%d block=%d", \
                DT, NW, MODE, KBV, RBW, CBV, a.s.M / (kRows * RBW), (int)(GRID_Y), NW * 64);                     \
  else                                                                                                           \
    spmm_rows16_prepared_kernel<DT, NW, MODE, KBV, RBW, CBV>                                                     \
      <<<dim3(a.s.M / (kRows * RBW), GRID_Y), NW * 64, LDS, stream>>>(                                           \
          base + L.a_offset, reinterpret_cast<const int32_t*>(base + L.gather_offset),                           \
          reinterpret_cast<const int32_t*>(base + L.pi_out_offset), base + L.zero_offset, X_PTR, a.ldx,          \
          a.out_f32 ? static_cast<void*>(static_cast<float*>(a.Y) + (Y_OFF))                                     \
                    : static_cast<void*>(static_cast<uint16_t*>(a.Y) + (Y_OFF)),                                 \
          a.ldy, a.s.V, L.RB, L.S, a.N - (Y_OFF), a.s.K, a.relu, a.out_f32)
  if (a.N == 1) {
    // staging the input vector pays once a wave gathers for more than four steps (4096 x 11008 at 50 %:
    // 10.4 -> 9.9 us; with four steps per wave and 688 workgroups it costs 0.8 us instead)
    const size_t x_bytes = ((size_t)a.s.K + 8) * 2;
    const bool stage = a.ldx == 1 && a.s.K % 8 == 0 && (reinterpret_cast<uintptr_t>(a.X) & 15u) == 0 &&
                       a.s.K <= 8 * kXPieces * NW * 64 && x_bytes <= (size_t)kXLdsMaxBytes && L.S > 4 * NW;
    if (stage) {
      // slabs (static) plus the vector (dynamic) can exceed the default 64 KB of a workgroup
      if (!a.plan && raise_lds_limit<spmm_rows16_prepared_kernel<DT, NW, 3, KB, RBW>>(kXLdsMaxBytes) != hipSuccess)
        return;  // the error stays pending and is reported by the caller's hipGetLastError
      HINM_ROWS16(3, 1, x, 0, x_bytes);
    } else {
      HINM_ROWS16(2, 1, x, 0, 0);
    }
    return;
  }
  // rows of X that start on 16-byte boundaries: vector loads for every block, the ragged last one included
  if constexpr (NW <= 8) {  // (sixteen waves leave 128 registers per lane: not enough for several blocks)
    if (blocks_per_wg == 4 && a.ldx % 8 == 0) {  // (batches of two steps: four blocks of input rows per step)
      HINM_ROWS16_CB(1, 4, 2, (col_blocks + 3) / 4, x, 0, 0);
      return;
    }
    if (blocks_per_wg == 2 && a.ldx % 8 == 0) {
      HINM_ROWS16_CB(1, 2, KB, (col_blocks + 1) / 2, x, 0, 0);
      return;
    }
  }
  if (a.ldx % 8 == 0) {
    HINM_ROWS16(1, col_blocks, x, 0, 0);
  } else {
    HINM_ROWS16(0, col_blocks, x, 0, 0);
  }
#undef HINM_ROWS16
#undef HINM_ROWS16_CB
}

// The layer's input rows resident in LDS (XMODE 4): 16 columns, 64 rows per workgroup.
inline size_t resident_lds_bytes(int K) { return (size_t)((K + 31) / 32) * 1024 + 32; }
// The same region later takes the waves' partial tiles (four 16 x 16 fp32 tiles = 4096 bytes per wave), which
// for short input vectors is the larger of the two.
inline size_t resident_dynamic_lds_bytes(int K, int NW) {
  const size_t partials = (size_t)NW * 4 * kRows * kCols * 4;
  return resident_lds_bytes(K) > partials ? resident_lds_bytes(K) : partials;
}

template <int DT, int NW>
void launch_resident(const PreparedArgs& a, const PreparedLayout& L, hipStream_t stream) {
  constexpr auto kernel = spmm_rows16_prepared_kernel<DT, NW, 4, 4, 4>;
  if (a.plan) {
    plan_record(a.plan, "spmm_rows16_prepared_kernel<DT=%d,NW=%d,XMODE=4,KB=4,RBW=4,CB=1> grid=%dx1 block=%d lds=%d", DT,
                NW, a.s.M / 64, NW * 64, (int)resident_dynamic_lds_bytes(a.s.K, NW));
    return;
  }
  if (raise_lds_limit<kernel>(160 * 1024 - NW * kSlabBytes) != hipSuccess)
    return;  // the error stays pending and is reported by the caller's hipGetLastError
  const uint8_t* base = static_cast<const uint8_t*>(a.prepared);
  kernel<<<dim3(a.s.M / 64, 1), NW * 64, resident_dynamic_lds_bytes(a.s.K, NW), stream>>>(
      base + L.a_offset, reinterpret_cast<const int32_t*>(base + L.gather_offset),
      reinterpret_cast<const int32_t*>(base + L.pi_out_offset), base + L.zero_offset,
      static_cast<const uint16_t*>(a.X), a.ldx, a.Y, a.ldy, a.s.V, L.RB, L.S, a.N, a.s.K, a.relu, a.out_f32);
}

// Launch shape beyond the template choice by N: 16-row blocks per workgroup, waves, column blocks per workgroup.
struct Rows16Plan {
  int rbw;
  int nw;
  int blocks_per_wg;  // 16-column blocks: 1, 2 or 4
};

Rows16Plan plan_rows16(const PreparedArgs& a) {
  const PreparedLayout L = prepared_layout(a.s);
  Rows16Plan p;
  // Several 16-row blocks in one workgroup share the gathered input rows: both halves of a 32-row block when
  // the grid then still holds 256 workgroups (column blocks count: 4096 x 4096 at N = 128 22.8 -> 17.1 us), two
  // neighbouring 32-row blocks under the same condition on layers of at least 2048 rows and beyond one column
  // block (-> 13.0 us; 8192 x 8192 at N = 128 62.8 -> 47.8 us; with fewer rows the shorter grid loses: 768 x 3072
  // at N = 384 9.2 -> 12.0 us).
  const int64_t col_blocks = (a.N + kCols - 1) / kCols;
  const bool quad = a.N > kCols && a.s.V % 64 == 0 && a.s.M >= 2048 && (a.s.M / 64) * col_blocks >= 256;
  const bool both = a.N > 4 && (a.s.M / 32) * col_blocks >= 256;
  p.rbw = quad ? 4 : both ? 2 : 1;
  // one batch per wave where possible (every load of the wave in flight at once): waves x batch >= steps ...
  const int nw_steps = L.S <= 4 ? 1 : L.S <= 16 ? 4 : L.S <= 32 ? 8 : 16;
  p.nw = nw_steps;
  p.blocks_per_wg = 1;
  if (a.N > kCols) {
    // ... but no more waves than the chip can hold at once: with many workgroups (several column blocks, or
    // a tall layer) the parallelism is already there, and fewer waves per workgroup mean fewer partial tiles
    // to sum and more of each wave's own loads in flight one after another (4096 x 4096 at N = 128, 2048
    // workgroups: 32.8 us with eight waves, 22.7 us with one).  About eight waves per compute unit in total.
    const int64_t row_wgs = a.s.M / (kRows * p.rbw);
    // Two or four column blocks per workgroup: a step's weights, gather entries and the 128-byte cache lines of
    // its input rows then serve 32 or 64 columns (11008 x 4096 at N = 128 42.3 -> 31.1 -> 24.8 us, 8192 x 8192
    // at N = 256 89.5 -> 69.3 -> 45.0 us).  It needs a grid that still covers most of the chip (160 workgroups;
    // with 96..159 it measured slower: 4096 x 4096 at N = 64, 128 workgroups left, 7.9 -> 9.5 us) and at least
    // eight steps (from there on never slower under that condition; 8192 x 1024 with 512 kept columns at
    // N = 256: 17.7 -> 13.5 us).
    if (a.ldx % 8 == 0 && L.S >= 8) {
      if (col_blocks >= 3 && row_wgs * ((col_blocks + 3) / 4) >= 160) p.blocks_per_wg = 4;
      else if (row_wgs * ((col_blocks + 1) / 2) >= 160) p.blocks_per_wg = 2;
    }
    const int64_t wgs = row_wgs * ((col_blocks + p.blocks_per_wg - 1) / p.blocks_per_wg);
    while (p.nw > 1 && wgs * p.nw > 2048) p.nw >>= 1;
    if (p.blocks_per_wg > 1 && p.nw > 8) {  // sixteen waves leave too few registers for several blocks
      p.blocks_per_wg = 1;
      p.nw = nw_steps;
      while (p.nw > 1 && row_wgs * col_blocks * p.nw > 2048) p.nw >>= 1;
    }
  }
  return p;
}

template <int DT, int RBW>
void launch_waves(const PreparedArgs& a, const Rows16Plan& plan, hipStream_t stream) {
  const PreparedLayout L = prepared_layout(a.s);
  const int blocks = plan.blocks_per_wg;
  const bool deep = L.S > 64;  // batches of six steps for long k loops
  switch (plan.nw) {
    case 1: return launch_modes<DT, 1, 4, RBW>(a, L, blocks, stream);
    case 2: return launch_modes<DT, 2, 4, RBW>(a, L, blocks, stream);
    case 4: return launch_modes<DT, 4, 4, RBW>(a, L, blocks, stream);
    case 8: return launch_modes<DT, 8, 4, RBW>(a, L, blocks, stream);
    default:
      if (deep) launch_modes<DT, 16, 6, RBW>(a, L, 1, stream);
      else launch_modes<DT, 16, 4, RBW>(a, L, 1, stream);
  }
}

template <int DT>
void launch_dt(const PreparedArgs& a, hipStream_t stream) {
  // 16 columns and a layer whose input fits in LDS beside the slabs: no gather from global memory at all.
  // Each workgroup then owns 64 rows, so the layer needs enough of them to keep most of the chip streaming,
  // and copying the 32 K bytes of input has to be small beside the workgroup's weights (11008 x 4096:
  // 12.4 -> 10.3 us with 2048 kept columns, 7.4 -> 7.9 us with 1024).
  const PreparedLayout L = prepared_layout(a.s);
  if (spmm_rows16_resident_supported(a) && (a.tile_variant == 19 || (a.s.M / 64 >= 160 && L.S > 16))) {
    if (L.S <= 16) launch_resident<DT, 4>(a, L, stream);
    else launch_resident<DT, 8>(a, L, stream);
    return;
  }
  const Rows16Plan plan = plan_rows16(a);
  if (plan.rbw == 4) launch_waves<DT, 4>(a, plan, stream);
  else if (plan.rbw == 2) launch_waves<DT, 2>(a, plan, stream);
  else launch_waves<DT, 1>(a, plan, stream);
}

}  // namespace

int spmm_rows16_prepared_blocks_per_wg(const PreparedArgs& a) { return plan_rows16(a).blocks_per_wg; }

bool spmm_rows16_resident_supported(const PreparedArgs& a) {
  const PreparedLayout L = prepared_layout(a.s);
  if (a.N != 16 || a.ldx % 8 != 0 || (reinterpret_cast<uintptr_t>(a.X) & 15u) != 0) return false;
  if (a.s.V % 64 != 0 || L.S > 32 || a.tile_variant == 11) return false;
  const int NW = L.S <= 16 ? 4 : 8;
  return resident_dynamic_lds_bytes(a.s.K, NW) + (size_t)NW * kSlabBytes <= 160 * 1024;
}

hipError_t launch_spmm_rows16_prepared(const PreparedArgs& a, hipStream_t stream) {
  if (a.s.dtype == HINM_F16) launch_dt<HINM_F16>(a, stream);
  else launch_dt<HINM_BF16>(a, stream);
  if (a.plan) return hipSuccess;  // a dry run launched nothing
  return hipGetLastError();
}

}  // namespace hinm
