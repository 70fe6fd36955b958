// HiNM sparse GEMM with fused channel permutation for many columns
// (arXiv 2407.20496, Section 3.2 and Section 5.3).
//
// One workgroup computes one tile of V = 32 * RB consecutive output channels for a block of 256
// columns.  The tile's kept input channels are walked in steps of KS = 32 * KSUB:
//   global -> LDS : the KS input rows named by the vector index composed with pi_in are gathered
//                   (each a contiguous 512-byte row segment) together with the tile's stored
//                   values and NM nibbles for that step; this is where the channel permutation is
//                   absorbed, at no cost beyond the vector-index lookup the format needs anyway;
//   LDS -> MFMA   : every wave owns 64 of the 256 columns and all V rows; A fragments are plain
//                   16-byte LDS reads, B fragments use the transposing LDS read, the NM nibbles
//                   go unchanged into the index operand of the 32x32x32 sparse MFMA;
//   epilogue      : fp32 accumulators -> optional ReLU -> 16-bit, staged through LDS so that every
//                   output row leaves as one contiguous 512-byte segment to row pi_out[r] of Y.
// Global loads for step s+1 are in flight while step s is multiplied (registers -> other LDS stage).
#include "hinm_internal.h"
#include "mfma_types.h"
#include "direct_lds.h"
#include "tile_epilogue.h"

#include <type_traits>

namespace hinm {
namespace {

constexpr int kNB = 256;       // columns per workgroup
constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int kCB = 2;         // 32-column blocks per wave
constexpr int kBStride = kNB * 2 + 64;  // bytes per gathered row in LDS (+64: rows 4 apart hit distinct banks)
constexpr int kYStride = kNB * 2 + 16;  // bytes per staged output row

template <int KSUB>
struct StageLayout {
  static constexpr int KS = 32 * KSUB;
  static constexpr int a_val_bytes = KS;            // KS/2 stored values per row and step
  static constexpr int a_nm_offset = a_val_bytes;   // then KS/8 bytes of nibbles
  static constexpr int a_stride = a_val_bytes + 16; // 48 or 80: 16 consecutive rows hit 16 distinct 16-byte bank groups
  static constexpr int b_bytes = KS * kBStride;
  __host__ __device__ static constexpr int a_bytes(int V) { return V * a_stride; }
  __host__ __device__ static constexpr int stage_bytes(int V) { return b_bytes + a_bytes(V); }
  __host__ __device__ static constexpr int total_bytes(int V) {
    const int two = 2 * stage_bytes(V);
    const int epi = V * kYStride;
    return two > epi ? two : epi;
  }
};

template <int DT, int RB, int KSUB>
__global__ __launch_bounds__(kThreads) void spmm_tile_kernel(
    const uint16_t* __restrict__ vals, const uint8_t* __restrict__ nm_idx, const int32_t* __restrict__ vec_idx,
    const int32_t* __restrict__ pi_in, const int32_t* __restrict__ pi_out, const uint16_t* __restrict__ X,
    int64_t ldx, void* __restrict__ Y, int64_t ldy, int T, int Kv, int N, int n_blocks, int work_per_xcd,
    bool relu, bool out_f32) {
  using L = StageLayout<KSUB>;
  constexpr int V = 32 * RB;
  constexpr int KS = L::KS;
  constexpr int B_PIECES = KS / 8;                 // 16-byte pieces of B per thread and step
  constexpr int A_PIECES_TOTAL = V * KS / 16;      // 16-byte pieces of stored values per step
  constexpr int A_PIECES = (A_PIECES_TOTAL + kThreads - 1) / kThreads;
  constexpr int NM_WORDS_TOTAL = V * KSUB;         // one dword of nibbles per row and 32-column substep
  constexpr int NM_WORDS = (NM_WORDS_TOTAL + kThreads - 1) / kThreads;

  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

  // ---- which (column block, tile) this workgroup owns: consecutive workgroup ids go to
  // different XCDs, so give every XCD a contiguous run of the column-block-major work list; the
  // tiles that run together on one XCD then share one column panel of X in that XCD's L2.
  const int xcd = blockIdx.x & 7;
  const int slot = blockIdx.x >> 3;
  const int work = xcd * work_per_xcd + slot;
  if (slot >= work_per_xcd || work >= n_blocks * T) return;
  const int nb = work / T;
  const int t = work % T;
  const int n0 = nb * kNB;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int steps = (Kv + KS - 1) / KS;

  const int32_t* vi = vec_idx + (size_t)t * Kv;
  const uint16_t* vtile = vals + (size_t)t * V * (Kv / 2);
  const uint8_t* ntile = nm_idx + (size_t)t * V * (Kv / 8);

  // ---- per-thread roles in the global -> LDS copy --------------------------------------------
  // B piece q of this thread: row 8 q + tid / 32 of the step, 16-byte column chunk tid % 32
  const int b_row0 = tid >> 5;
  const int b_chunk = tid & 31;
  const bool b_cols_ok = n0 + b_chunk * 8 < N;  // chunk starts inside the matrix (ldx % 8 == 0 keeps it in bounds)

  u32x4 b_regs[B_PIECES];
  u32x4 a_regs[A_PIECES];
  uint32_t nm_regs[NM_WORDS];
  int g_next[B_PIECES];   // X rows of step s + 1
  int g_next2[B_PIECES];  // X rows of step s + 2 (after pi_in)
  int v_next3[B_PIECES];  // vector-index entries of step s + 3

  auto load_vec_idx = [&](int step, int (&out)[B_PIECES]) {
#pragma unroll
    for (int q = 0; q < B_PIECES; ++q) {
      const int j = step * KS + 8 * q + b_row0;
      out[q] = (j < Kv) ? vi[j] : -1;
    }
  };
  auto apply_pi_in = [&](const int (&in)[B_PIECES], int (&out)[B_PIECES]) {
#pragma unroll
    for (int q = 0; q < B_PIECES; ++q) out[q] = (in[q] >= 0 && pi_in) ? pi_in[in[q]] : in[q];
  };
  auto load_step = [&](int step, const int (&rows)[B_PIECES]) {
#pragma unroll
    for (int q = 0; q < B_PIECES; ++q) {
      b_regs[q] = u32x4{0, 0, 0, 0};
      if (rows[q] >= 0 && b_cols_ok)
        b_regs[q] = *reinterpret_cast<const u32x4*>(X + (size_t)rows[q] * ldx + n0 + b_chunk * 8);
    }
#pragma unroll
    for (int q = 0; q < A_PIECES; ++q) {
      const int p = tid + q * kThreads;
      a_regs[q] = u32x4{0, 0, 0, 0};
      if (p < A_PIECES_TOTAL) {
        const int row = p / (KS / 16), c = p % (KS / 16);  // 16-byte piece c of the row's KS bytes
        const int val0 = step * (KS / 2) + c * 8;          // first stored value of the piece
        if (val0 * 2 + 16 <= Kv)                            // whole piece inside the row (Kv % 32 == 0)
          a_regs[q] = *reinterpret_cast<const u32x4_a4*>(vtile + (size_t)row * (Kv / 2) + val0);
      }
    }
#pragma unroll
    for (int q = 0; q < NM_WORDS; ++q) {
      const int p = tid + q * kThreads;
      nm_regs[q] = 0;
      if (p < NM_WORDS_TOTAL) {
        const int row = p / KSUB, sub = p % KSUB;
        const int byte0 = step * (KS / 8) + sub * 4;
        if (byte0 * 8 + 32 <= Kv) nm_regs[q] = *reinterpret_cast<const uint32_t*>(ntile + (size_t)row * (Kv / 8) + byte0);
      }
    }
  };
  auto store_step = [&](uint8_t* stage) {
    uint8_t* bs = stage;
    uint8_t* as = stage + L::b_bytes;
#pragma unroll
    for (int q = 0; q < B_PIECES; ++q)
      *reinterpret_cast<u32x4*>(bs + (8 * q + b_row0) * kBStride + b_chunk * 16) = b_regs[q];
#pragma unroll
    for (int q = 0; q < A_PIECES; ++q) {
      const int p = tid + q * kThreads;
      if (p < A_PIECES_TOTAL) {
        const int row = p / (KS / 16), c = p % (KS / 16);
        *reinterpret_cast<u32x4*>(as + row * L::a_stride + c * 16) = a_regs[q];
      }
    }
#pragma unroll
    for (int q = 0; q < NM_WORDS; ++q) {
      const int p = tid + q * kThreads;
      if (p < NM_WORDS_TOTAL) {
        const int row = p / KSUB, sub = p % KSUB;
        *reinterpret_cast<uint32_t*>(as + row * L::a_stride + L::a_nm_offset + sub * 4) = nm_regs[q];
      }
    }
  };

  // ---- MFMA roles -------------------------------------------------------------------------------
  const int i32 = lane & 31;  // A row / B column inside a 32-block
  const int qh = lane >> 5;   // lane group (qa for A, qb for B)
  const int i16 = lane & 15;
  f32x16 acc[RB][kCB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int cb = 0; cb < kCB; ++cb)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[rb][cb][e] = 0.f;

  auto compute_step = [&](const uint8_t* stage) {
    const uint8_t* bs = stage;
    const uint8_t* as = stage + L::b_bytes;
#pragma unroll
    for (int sub = 0; sub < KSUB; ++sub) {
      u32x4 a[RB];
      int idx[RB];
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        const uint8_t* row = as + (32 * rb + i32) * L::a_stride;
        // lane group qa holds groups 4 qa .. 4 qa + 3 of the substep: stored values 8 qa .. 8 qa + 7
        a[rb] = *reinterpret_cast<const u32x4*>(row + sub * 32 + qh * 16);
        idx[rb] = *reinterpret_cast<const uint16_t*>(row + L::a_nm_offset + sub * 4 + qh * 2);
      }
#pragma unroll
      for (int cb = 0; cb < kCB; ++cb) {
        // B slots 8 h + 4 u .. + 3 of lane group qb <- rows 16 h + 8 qb + 4 u + (0..3) of the substep
        u32x8 b;
        const int col_byte = (wave * 64 + cb * 32 + (i32 & 16) + (i16 & 3) * 4) * 2;
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int u = 0; u < 2; ++u) {
            const int row = sub * 32 + 16 * h + 8 * qh + 4 * u + (i16 >> 2);
            const u32x2 v = lds_read_tr16(bs + row * kBStride + col_byte);
            b[(2 * h + u) * 2] = v.x;
            b[(2 * h + u) * 2 + 1] = v.y;
          }
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) acc[rb][cb] = smfmac_32x32x32<DT, 0>(a[rb], b, acc[rb][cb], idx[rb]);
      }
    }
  };

  // ---- pipeline ---------------------------------------------------------------------------------
  uint8_t* stage0 = lds;
  uint8_t* stage1 = lds + L::stage_bytes(V);
  {
    int v0[B_PIECES], v1[B_PIECES], v2[B_PIECES];
    load_vec_idx(0, v0);
    load_vec_idx(1, v1);
    load_vec_idx(2, v2);
    int g0[B_PIECES];
    apply_pi_in(v0, g0);
    apply_pi_in(v1, g_next);
    apply_pi_in(v2, g_next2);
    load_vec_idx(3, v_next3);
    load_step(0, g0);
    store_step(stage0);
  }
  __syncthreads();
  for (int s = 0; s < steps; ++s) {
    uint8_t* cur = (s & 1) ? stage1 : stage0;
    uint8_t* nxt = (s & 1) ? stage0 : stage1;
    const bool more = s + 1 < steps;
    if (more) load_step(s + 1, g_next);
    // rotate the index pipeline: rows of step s+2 are ready, translate step s+3, fetch step s+4
#pragma unroll
    for (int q = 0; q < B_PIECES; ++q) g_next[q] = g_next2[q];
    apply_pi_in(v_next3, g_next2);
    load_vec_idx(s + 4, v_next3);
    compute_step(cur);
    if (more) store_step(nxt);
    __syncthreads();
  }

  // ---- epilogue -----------------------------------------------------------------------------------
  store_tile_rows<DT, RB, kCB, kNB, 64, kThreads, kYStride>(acc, lds, Y, ldy, N, n0, relu, out_f32,
                                                            [&](int row) -> int64_t { const int r = t * V + row; return pi_out ? pi_out[r] : r; });
}

// ---------------------------------------------------------------------------------------------
// Direct-to-LDS variant for Kv % 64 == 0 (the common case): stages of 64 kept columns, two buffers,
// NB in {256, 512} columns per workgroup, every wave 64 columns and all V rows.
//   B : the 64 input rows of a stage arrive as contiguous NB-column segments straight from global
//       memory into LDS; the row numbers (vector index composed with pi_in) are wave-uniform scalar
//       loads, fetched two stages and translated one stage ahead.  32-byte units of a row are
//       XOR-swizzled by row % 4 on the source address, for the transposing reads.
//   A : the tile's stored values of the stage, 64 bytes per row of the canonical array, copied the
//       same way with the four 16-byte chunks of row r stored at chunk ^ ((r / 4) % 4), so that the
//       fragment reads of 16 consecutive rows cover all banks once; and its NM nibbles, one dword
//       per row and 32-column substep, with 4-byte copies into a [substep][row] array.
// One barrier per stage; a stage is multiplied while the copies of the next one are in flight.
// Same results as the register-staged kernel above; about 2.5x faster on large layers.
// ---------------------------------------------------------------------------------------------
template <int RB, int NB, int WC>
struct TileDmaCfg {
  static constexpr int V = 32 * RB;
  static constexpr int NW = NB / WC;                          // waves; each owns WC of the NB columns
  static constexpr int THREADS = NW * 64;
  static constexpr int CBS = WC / 32;                         // 32-column accumulator blocks per wave
  static constexpr int ROW_BYTES = NB * 2;
  static constexpr int B_BYTES = 64 * ROW_BYTES;
  static constexpr int A_VAL_BYTES = V * 64;                 // 32 stored values per row and stage
  static constexpr int A_NM_BYTES = V * 8;                   // one dword of nibbles per row and 32-column substep
  static constexpr int STAGE_BYTES = B_BYTES + A_VAL_BYTES + A_NM_BYTES;
  static constexpr int ROWS_PER_WAVE = 64 / NW;
  static constexpr int B_PER_WAVE = (NB == 512) ? ROWS_PER_WAVE : ROWS_PER_WAVE / 2;
  static constexpr int A_VAL_INSTR = V / 16;                 // wave-wide 16-byte copies: 16 rows x 64 bytes each
  static constexpr int A_NM_INSTR = V / 32;                  // wave-wide 4-byte copies: 64 dwords each
  static constexpr int A_INSTR = A_VAL_INSTR + A_NM_INSTR;
  static constexpr int A_ROUNDS = (A_INSTR + NW - 1) / NW;
  static constexpr int Y_STRIDE = NB * 2 + 16;
  static constexpr int EPI_BYTES = V * Y_STRIDE;
  static constexpr int LDS_BYTES = (2 * STAGE_BYTES > EPI_BYTES) ? 2 * STAGE_BYTES : EPI_BYTES;
  static_assert(NB == 256 || NB == 512, "column block");
  static_assert(WC == 64 || WC == 32, "columns per wave");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS of a compute unit");
};

template <int DT, int RB, int NB, int WC>
__global__ __launch_bounds__(NB / WC * 64) void spmm_tile_dma_kernel(
    const uint16_t* __restrict__ vals, const uint8_t* __restrict__ nm_idx, const int32_t* __restrict__ vec_idx,
    const int32_t* __restrict__ pi_in,
    const int32_t* __restrict__ pi_out, const uint16_t* __restrict__ X, int64_t ldx, void* __restrict__ Y,
    int64_t ldy, int T, int Kv, int N, int n_blocks, int work_per_xcd, bool relu, bool out_f32) {
  using C = TileDmaCfg<RB, NB, WC>;
  constexpr int V = C::V;
  constexpr int NW = C::NW;
  constexpr int CBS = C::CBS;
  constexpr int RPW = C::ROWS_PER_WAVE;
  extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];

  const int xcd = blockIdx.x & 7;
  const int slot = blockIdx.x >> 3;
  const int work = xcd * work_per_xcd + slot;
  if (slot >= work_per_xcd || work >= n_blocks * T) return;
  const int nb = work / T;
  const int t = work % T;
  const int n0 = nb * NB;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int stages_total = Kv / 64;

  const int32_t* vi = vec_idx + (size_t)t * Kv;
  const uint8_t* a_tile = reinterpret_cast<const uint8_t*>(vals + (size_t)t * V * (Kv / 2));   // Kv bytes per row
  const uint8_t* nm_tile = nm_idx + (size_t)t * V * (Kv / 8);

  // ---- copy roles (B as in the sparse tile kernel) -------------------------------------------------
  const RowSegmentCopy<NB> b_copy(lane, n0, N);
  // A values: wave-wide copy number i moves rows 16 i .. 16 i + 15; lane l lands at 16 l = row 16 i + l / 4,
  // chunk position l % 4, and fetches chunk (l % 4) ^ ((row / 4) % 4) of that row's 64 bytes.
  // A nibbles: copy number k moves dwords 64 k .. 64 k + 63 of the stage's [substep][row] array.
  uint32_t a_src_off[C::A_ROUNDS];
#pragma unroll
  for (int m = 0; m < C::A_ROUNDS; ++m) {
    const int instr = wave + m * NW;
    if (instr < C::A_VAL_INSTR) {
      const int row = 16 * instr + (lane >> 2);
      const int chunk = (lane & 3) ^ ((row >> 2) & 3);
      a_src_off[m] = (uint32_t)row * (uint32_t)Kv + (uint32_t)chunk * 16u;
    } else {
      const int d = min(64 * (instr - C::A_VAL_INSTR) + lane, 2 * V - 1);
      const int sub = d / V, row = d % V;
      a_src_off[m] = (uint32_t)row * (uint32_t)(Kv / 8) + (uint32_t)sub * 4u;
    }
  }

  typedef int rows_t __attribute__((ext_vector_type(RPW), aligned(4)));  // the vector index only promises 4-byte alignment
  auto load_vec_idx = [&](int stage_idx) -> rows_t {  // wave-uniform: scalar load
    const int st = min(stage_idx, stages_total - 1);
    return *reinterpret_cast<const rows_t*>(vi + st * 64 + wave * RPW);
  };
  auto apply_pi_in = [&](rows_t v) -> rows_t {
    if (!pi_in) return v;
    rows_t g;
#pragma unroll
    for (int k = 0; k < RPW; ++k) g[k] = pi_in[v[k]];
    return g;
  };
  const uint8_t* x_block = reinterpret_cast<const uint8_t*>(X + n0);
  auto row_base = [&](int g) -> const uint8_t* { return x_block + (size_t)g * ldx * 2; };  // wave-uniform
  auto b_buffer = [&](int stage_idx) -> uint8_t* { return lds + (stage_idx & 1) * C::STAGE_BYTES; };
  auto a_buffer = [&](int stage_idx) -> uint8_t* { return lds + (stage_idx & 1) * C::STAGE_BYTES + C::B_BYTES; };
  auto issue_stage = [&](int stage_idx, const rows_t rows) {
    uint8_t* bs = b_buffer(stage_idx);
    b_copy.template issue<C::B_PER_WAVE, C::ROW_BYTES>([&](int j) { return row_base(rows[j]); },
                                                        bs + wave * RPW * C::ROW_BYTES);
    uint8_t* as = a_buffer(stage_idx);
#pragma unroll
    for (int m = 0; m < C::A_ROUNDS; ++m) {
      const int instr = wave + m * NW;  // wave-uniform
      if (instr < C::A_VAL_INSTR)
        copy16_to_lds(a_tile + (size_t)stage_idx * 64 + a_src_off[m], as + instr * 1024);
      else if (instr < C::A_INSTR)
        copy4_to_lds(nm_tile + (size_t)stage_idx * 8 + a_src_off[m],
                     as + C::A_VAL_BYTES + (instr - C::A_VAL_INSTR) * 256);
    }
  };

  // ---- MFMA roles -------------------------------------------------------------------------------------
  const int i32 = lane & 31;
  const int qh = lane >> 5;
  const int i16 = lane & 15;
  const int sw_lane = swizzle_of_row(i16 >> 2);
  const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_void_t*)lds;
  uint32_t b_lane_off[CBS];
#pragma unroll
  for (int cb = 0; cb < CBS; ++cb)
    b_lane_off[cb] = (8 * qh + (i16 >> 2)) * C::ROW_BYTES +
                     (((wave * (WC / 16) + cb * 2 + (i32 >> 4)) ^ sw_lane) * 32) + (i16 & 3) * 8;
  // A fragment of the 32-column substep q: chunk 2 q + qh of row i32 (+ 32 rb), at its swizzled place;
  // its four NM nibbles: half qh of the dword of (substep q, row)
  uint32_t a_lane_off[2], nm_lane_off[2];
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    a_lane_off[q] = i32 * 64 + (((2 * q + qh) ^ ((i32 >> 2) & 3)) * 16);
    nm_lane_off[q] = C::A_VAL_BYTES + (q * V + i32) * 4 + qh * 2;
  }

  f32x16 acc[RB][CBS];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int cb = 0; cb < CBS; ++cb)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[rb][cb][e] = 0.f;

  // B slots 8 h + 4 u .. + 3 of lane group qh <- rows 16 h + 8 qh + 4 u + (0..3) of the 32-column substep
  auto compute_sub = [&](int stage_idx, auto sub_tag) {
    constexpr int Q = decltype(sub_tag)::value;
    const uint32_t stage_addr = lds_base + (uint32_t)(b_buffer(stage_idx) - lds);
    const uint8_t* as = a_buffer(stage_idx);
    constexpr int R0 = (Q * 32 + 0) * C::ROW_BYTES, R1 = (Q * 32 + 4) * C::ROW_BYTES,
                  R2 = (Q * 32 + 16) * C::ROW_BYTES, R3 = (Q * 32 + 20) * C::ROW_BYTES;
    u32x2 r[CBS][4];
#pragma unroll
    for (int cb = 0; cb < CBS; ++cb)
      lds_read_tr16_x4<R0, R1, R2, R3>(stage_addr + b_lane_off[cb], r[cb][0], r[cb][1], r[cb][2], r[cb][3]);
    u32x4 a[RB];
    int idx[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      a[rb] = *reinterpret_cast<const u32x4*>(as + rb * 2048 + a_lane_off[Q]);
      idx[rb] = *reinterpret_cast<const uint16_t*>(as + rb * 128 + nm_lane_off[Q]);
    }
    u32x8 b0 = u32x8{r[0][0].x, r[0][0].y, r[0][1].x, r[0][1].y, r[0][2].x, r[0][2].y, r[0][3].x, r[0][3].y};
    u32x8 b1 = b0;
    if constexpr (CBS == 2) {
      b1 = u32x8{r[CBS - 1][0].x, r[CBS - 1][0].y, r[CBS - 1][1].x, r[CBS - 1][1].y,
                 r[CBS - 1][2].x, r[CBS - 1][2].y, r[CBS - 1][3].x, r[CBS - 1][3].y};
      lds_wait_tr(b0, b1);
    } else {
      lds_wait_tr(b0);
    }
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      acc[rb][0] = smfmac_32x32x32<DT, 0>(a[rb], b0, acc[rb][0], idx[rb]);
      if constexpr (CBS == 2) acc[rb][1] = smfmac_32x32x32<DT, 0>(a[rb], b1, acc[rb][1], idx[rb]);
    }
  };

  // ---- pipeline -----------------------------------------------------------------------------------------
  issue_stage(0, apply_pi_in(load_vec_idx(0)));
  rows_t rows_next = apply_pi_in(load_vec_idx(1));  // translated rows of stage s + 1
  rows_t vec_next2 = load_vec_idx(2);                // vector-index entries of stage s + 2
  for (int s = 0; s < stages_total; ++s) {
    wait_copies_outstanding<0>();  // this wave's copies of stage s have landed
    __builtin_amdgcn_s_barrier();  // ... and everyone's; everyone is also done reading the other buffer
    if (s + 1 < stages_total) issue_stage(s + 1, rows_next);
    rows_next = apply_pi_in(vec_next2);
    vec_next2 = load_vec_idx(s + 3);
    compute_sub(s, std::integral_constant<int, 0>{});
    compute_sub(s, std::integral_constant<int, 1>{});
  }

  // ---- epilogue -------------------------------------------------------------------------------------------
  store_tile_rows<DT, RB, CBS, NB, WC, C::THREADS, C::Y_STRIDE>(acc, lds, Y, ldy, N, n0, relu, out_f32,
                                                                  [&](int row) -> int64_t { const int r = t * V + row; return pi_out ? pi_out[r] : r; });
}

template <int DT, int RB, int KSUB>
hipError_t launch_one(const SpmmArgs& a, hipStream_t stream) {
  using L = StageLayout<KSUB>;
  constexpr int V = 32 * RB;
  const int T = a.s.M / V;
  const int n_blocks = (a.N + kNB - 1) / kNB;
  const int64_t work = (int64_t)n_blocks * T;
  const int work_per_xcd = (int)((work + 7) / 8);
  const size_t lds_bytes = L::total_bytes(V);
  constexpr auto kernel = spmm_tile_kernel<DT, RB, KSUB>;
  if (hipError_t e = raise_lds_limit<kernel>((int)lds_bytes); e != hipSuccess) return e;
  kernel<<<dim3((unsigned)(work_per_xcd * 8)), kThreads, lds_bytes, stream>>>(
      static_cast<const uint16_t*>(a.vals), a.nm_idx, a.vec_idx, a.pi_in, a.pi_out,
      static_cast<const uint16_t*>(a.X), a.ldx, a.Y, a.ldy, T, a.s.Kv, a.N, n_blocks, work_per_xcd, a.relu,
      a.out_f32);
  return hipGetLastError();
}

template <int DT, int RB, int NB, int WC>
hipError_t launch_dma(const SpmmArgs& a, hipStream_t stream) {
  using C = TileDmaCfg<RB, NB, WC>;
  const int T = a.s.M / C::V;
  const int n_blocks = (a.N + NB - 1) / NB;
  const int64_t work = (int64_t)n_blocks * T;
  const int work_per_xcd = (int)((work + 7) / 8);
  constexpr auto kernel = spmm_tile_dma_kernel<DT, RB, NB, WC>;
  if (hipError_t e = raise_lds_limit<kernel>(C::LDS_BYTES); e != hipSuccess) return e;
  kernel<<<dim3((unsigned)(work_per_xcd * 8)), C::THREADS, C::LDS_BYTES, stream>>>(
      static_cast<const uint16_t*>(a.vals), a.nm_idx, a.vec_idx, a.pi_in, a.pi_out, static_cast<const uint16_t*>(a.X),
      a.ldx, a.Y, a.ldy, T, a.s.Kv, a.N, n_blocks, work_per_xcd, a.relu, a.out_f32);
  return hipGetLastError();
}

template <int DT, int RB>
hipError_t launch_rb(const SpmmArgs& a, hipStream_t stream) {
  if (a.s.Kv % 64 != 0) return launch_one<DT, RB, 2>(a, stream);
  // 512-column blocks halve the re-reads of the stored values when there are enough of them to fill the chip
  const int64_t wide_blocks = (int64_t)(a.s.M / (32 * RB)) * ((a.N + 511) / 512);
  // Waves of 32 columns (twice as many per workgroup) cover the latency of a stage's copies better and read
  // 40 % more from LDS per MFMA: better unless the layer is large enough to be bound by that throughput.
  if (a.N >= 1024 && wide_blocks >= 256)
    return wide_blocks <= 1024 ? launch_dma<DT, RB, 512, 32>(a, stream) : launch_dma<DT, RB, 512, 64>(a, stream);
  return launch_dma<DT, RB, 256, 32>(a, stream);
}

template <int DT>
hipError_t launch_dt(const SpmmArgs& a, hipStream_t stream) {
  switch (a.s.V) {
    case 32: return launch_rb<DT, 1>(a, stream);
    case 64: return launch_rb<DT, 2>(a, stream);
    case 96: return launch_rb<DT, 3>(a, stream);
    case 128: return launch_rb<DT, 4>(a, stream);
  }
  return hipErrorInvalidValue;
}

}  // namespace

bool spmm_tile_supported(const SpmmArgs& a) {
  const int V = a.s.V;
  if (!(V == 32 || V == 64 || V == 96 || V == 128)) return false;
  if (a.s.Kv % 32 != 0) return false;
  if (a.ldx % 8 != 0 || a.ldy % 8 != 0) return false;
  if ((reinterpret_cast<uintptr_t>(a.nm_idx) & 3u) != 0) return false;
  const int64_t work = (int64_t)((a.N + kNB - 1) / kNB) * (a.s.M / V);
  return work < (1ll << 28);
}

hipError_t launch_spmm_tile(const SpmmArgs& a, hipStream_t stream) {
  return a.s.dtype == HINM_F16 ? launch_dt<HINM_F16>(a, stream) : launch_dt<HINM_BF16>(a, stream);
}

}  // namespace hinm
