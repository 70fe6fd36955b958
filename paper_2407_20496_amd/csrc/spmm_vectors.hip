// Product of a layer that carries the column-vector mask alone (arXiv 2407.20496, Section 3.1 first
// step; Section 5.1.2: during gradual pruning a layer stays in this state until the target vector
// sparsity is reached and only then receives the 2:4 mask), with the same fused channel orders as
// the HiNM product (Section 3.2, Section 5.3):
//     Y[pi_out[r]][n] = sum_j vals_v[r][j] * X[pi_in[vec_idx[r / V][j]]][n].
// Every surviving entry is stored, so this is a dense contraction over the gathered input rows and
// runs on the dense 32x32x16 MFMA.
//
// Two tile kernels with the same decomposition (one workgroup = one tile of V = 32 * RB consecutive
// output channels x a block of columns, every wave 64 columns and all V rows): the direct-to-LDS
// kernel further down for Kv % 64 == 0, and a register-staged one for every other Kv, which walks
// 256-column blocks in steps of 32 kept columns:
//   global -> LDS : the 32 input rows named by the vector index composed with pi_in (each a
//                   contiguous 512-byte row segment) and the tile's 32 stored values per row;
//   LDS -> MFMA   : every wave owns 64 of the 256 columns and all V rows; A fragments are plain
//                   16-byte LDS reads, B fragments use the transposing LDS read;
//   epilogue      : fp32 accumulators -> optional ReLU -> 16-bit, staged through LDS so that every
//                   output row leaves as one contiguous 512-byte segment to row pi_out[r] of Y.
// Global loads for step s+1 are in flight while step s is multiplied (registers -> other LDS stage).
// A plain kernel (one thread per output) covers every other legal shape and serves as cross-check.
#include "hinm_internal.h"
#include "mfma_types.h"
#include "direct_lds.h"
#include "tile_epilogue.h"

#include <type_traits>

namespace hinm {
namespace {

// Operand layout of the dense 32x32x16 MFMA (lane l): A holds row l % 32, k = 8 * (l / 32) + 0..7;
// B holds column l % 32, the same eight k; D as for the sparse 32x32 form.
template <int DT>
__device__ __forceinline__ f32x16 mfma_32x32x16(u32x4 a, u32x4 b, f32x16 c) {
  if constexpr (DT == HINM_F16) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0,
                                                  0);
  } else {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                   0, 0);
  }
}

constexpr int kNB = 256;  // columns per workgroup
constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int kCB = 2;                  // 32-column blocks per wave
constexpr int kKS = 32;                 // kept columns per step
constexpr int kBStride = kNB * 2 + 64;  // bytes per gathered row in LDS (+64: rows 4 apart hit distinct banks)
constexpr int kYStride = kNB * 2 + 16;  // bytes per staged output row
constexpr int kAStride = kKS * 2 + 16;  // 80: 16 consecutive rows hit 16 distinct 16-byte bank groups
constexpr int kBBytes = kKS * kBStride;

__host__ __device__ constexpr int stage_bytes(int V) { return kBBytes + V * kAStride; }
__host__ __device__ constexpr int total_lds_bytes(int V) {
  const int two = 2 * stage_bytes(V);
  const int epi = V * kYStride;
  return two > epi ? two : epi;
}

template <int DT, int RB>
__global__ __launch_bounds__(kThreads) void spmm_vectors_kernel(
    const uint16_t* __restrict__ vals_v, const int32_t* __restrict__ vec_idx, const int32_t* __restrict__ pi_in,
    const int32_t* __restrict__ pi_out, const uint16_t* __restrict__ X, int64_t ldx, void* __restrict__ Y,
    int64_t ldy, int T, int Kv, int N, int n_blocks, int work_per_xcd, bool relu, bool out_f32) {
  constexpr int V = 32 * RB;
  constexpr int B_PIECES = kKS / 8;             // 16-byte pieces of B per thread and step
  constexpr int A_PIECES_TOTAL = V * kKS / 8;   // 16-byte pieces of stored values per step
  constexpr int A_PIECES = (A_PIECES_TOTAL + kThreads - 1) / kThreads;

  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

  // consecutive workgroup ids go to different XCDs: give every XCD a contiguous run of the
  // column-block-major work list, so the tiles running together share one column panel of X in L2
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
  const int steps = (Kv + kKS - 1) / kKS;

  const int32_t* vi = vec_idx + (size_t)t * Kv;
  const uint16_t* vtile = vals_v + (size_t)t * V * Kv;

  // B piece q of this thread: row 8 q + tid / 32 of the step, 16-byte column chunk tid % 32
  const int b_row0 = tid >> 5;
  const int b_chunk = tid & 31;
  const bool b_cols_ok = n0 + b_chunk * 8 < N;  // chunk starts inside the matrix (ldx % 8 == 0 keeps it in bounds)

  u32x4 b_regs[B_PIECES];
  u32x4 a_regs[A_PIECES];
  int g_next[B_PIECES];   // X rows of step s + 1
  int g_next2[B_PIECES];  // X rows of step s + 2 (after pi_in)
  int v_next3[B_PIECES];  // vector-index entries of step s + 3

  auto load_vec_idx = [&](int step, int (&out)[B_PIECES]) {
#pragma unroll
    for (int q = 0; q < B_PIECES; ++q) {
      const int j = step * kKS + 8 * q + b_row0;
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
        const int row = p / (kKS / 8), c = p % (kKS / 8);  // 16-byte piece c of the row's 64 bytes
        const int j0 = step * kKS + c * 8;                  // first kept column of the piece
        if (j0 + 8 <= Kv)                                    // whole piece inside the row (Kv % 8 == 0)
          a_regs[q] = *reinterpret_cast<const u32x4*>(vtile + (size_t)row * Kv + j0);
      }
    }
  };
  auto store_step = [&](uint8_t* stage) {
    uint8_t* bs = stage;
    uint8_t* as = stage + kBBytes;
#pragma unroll
    for (int q = 0; q < B_PIECES; ++q)
      *reinterpret_cast<u32x4*>(bs + (8 * q + b_row0) * kBStride + b_chunk * 16) = b_regs[q];
#pragma unroll
    for (int q = 0; q < A_PIECES; ++q) {
      const int p = tid + q * kThreads;
      if (p < A_PIECES_TOTAL) {
        const int row = p / (kKS / 8), c = p % (kKS / 8);
        *reinterpret_cast<u32x4*>(as + row * kAStride + c * 16) = a_regs[q];
      }
    }
  };

  const int i32 = lane & 31;  // A row / B column inside a 32-block
  const int qh = lane >> 5;   // which eight k of the substep this lane holds
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
    const uint8_t* as = stage + kBBytes;
#pragma unroll
    for (int sub = 0; sub < kKS / 16; ++sub) {
      u32x4 a[RB];
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
        a[rb] = *reinterpret_cast<const u32x4*>(as + (32 * rb + i32) * kAStride + sub * 32 + qh * 16);
#pragma unroll
      for (int cb = 0; cb < kCB; ++cb) {
        // B slots 4 u .. 4 u + 3 <- rows 16 sub + 8 qh + 4 u + (0..3) of the step, column of this lane
        u32x4 b;
        const int col_byte = (wave * 64 + cb * 32 + (i32 & 16) + (i16 & 3) * 4) * 2;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const int row = sub * 16 + 8 * qh + 4 * u + (i16 >> 2);
          const u32x2 v = lds_read_tr16(bs + row * kBStride + col_byte);
          b[2 * u] = v.x;
          b[2 * u + 1] = v.y;
        }
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) acc[rb][cb] = mfma_32x32x16<DT>(a[rb], b, acc[rb][cb]);
      }
    }
  };

  uint8_t* stage0 = lds;
  uint8_t* stage1 = lds + stage_bytes(V);
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
// Direct-to-LDS variant (Kv % 64 == 0): stages of 64 kept columns, two buffers.
//   B : the 64 input rows of a stage arrive as contiguous NB-column segments straight from global
//       memory into LDS; the row numbers (vector index composed with pi_in) are wave-uniform scalar
//       loads, fetched two stages and translated one stage ahead.  32-byte units of a row are
//       XOR-swizzled by row % 4 on the source address, for the transposing reads.
//   A : the tile's V x 64 stored values of the stage, 128 bytes per row, copied the same way; the
//       eight 16-byte chunks of row r are stored at chunk ^ ((r / 2) % 8), so that the 16-byte
//       fragment reads of 16 consecutive rows cover all banks once.
// One barrier per stage; a stage is multiplied while the copies of the next one are in flight.
// ---------------------------------------------------------------------------------------------
template <int RB, int NB, int WC>
struct DmaCfg {
  static constexpr int V = 32 * RB;
  static constexpr int NW = NB / WC;                          // waves; each owns WC of the NB columns
  static constexpr int THREADS = NW * 64;
  static constexpr int CBS = WC / 32;                         // 32-column accumulator blocks per wave
  static constexpr int ROW_BYTES = NB * 2;
  static constexpr int B_BYTES = 64 * ROW_BYTES;
  static constexpr int A_BYTES = V * 128;
  static constexpr int STAGE_BYTES = B_BYTES + A_BYTES;
  static constexpr int ROWS_PER_WAVE = 64 / NW;
  static constexpr int B_PER_WAVE = (NB == 512) ? ROWS_PER_WAVE : ROWS_PER_WAVE / 2;
  static constexpr int A_INSTR = V / 8;                      // wave-wide copies of 8 rows x 128 bytes
  static constexpr int A_ROUNDS = (A_INSTR + NW - 1) / NW;
  static constexpr int Y_STRIDE = NB * 2 + 16;
  static constexpr int EPI_BYTES = V * Y_STRIDE;
  static constexpr int LDS_BYTES = (2 * STAGE_BYTES > EPI_BYTES) ? 2 * STAGE_BYTES : EPI_BYTES;
  static_assert(NB == 256 || NB == 512, "column block");
  static_assert(WC == 64 || WC == 32, "columns per wave");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS of a compute unit");
};

template <int DT, int RB, int NB, int WC>
__global__ __launch_bounds__(NB / WC * 64) void spmm_vectors_dma_kernel(
    const uint16_t* __restrict__ vals_v, const int32_t* __restrict__ vec_idx, const int32_t* __restrict__ pi_in,
    const int32_t* __restrict__ pi_out, const uint16_t* __restrict__ X, int64_t ldx, void* __restrict__ Y,
    int64_t ldy, int T, int Kv, int N, int n_blocks, int work_per_xcd, bool relu, bool out_f32) {
  using C = DmaCfg<RB, NB, WC>;
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
  const uint8_t* a_tile = reinterpret_cast<const uint8_t*>(vals_v + (size_t)t * V * Kv);

  // ---- copy roles (B as in the sparse tile kernel) -------------------------------------------------
  const RowSegmentCopy<NB> b_copy(lane, n0, N);
  // A: wave-wide copy number i moves rows 8 i .. 8 i + 7; lane l lands at 16 l = row 8 i + l / 8,
  // chunk position l % 8, and fetches chunk (l % 8) ^ ((row / 2) % 8) of that row
  uint32_t a_src_off[C::A_ROUNDS];
#pragma unroll
  for (int m = 0; m < C::A_ROUNDS; ++m) {
    const int row = min(8 * (wave + m * NW) + (lane >> 3), V - 1);
    const int chunk = (lane & 7) ^ ((row >> 1) & 7);
    a_src_off[m] = (uint32_t)row * (uint32_t)Kv * 2u + (uint32_t)chunk * 16u;
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
    const uint8_t* a_stage = a_tile + (size_t)stage_idx * 128;
#pragma unroll
    for (int m = 0; m < C::A_ROUNDS; ++m) {
      const int instr = wave + m * NW;
      if (instr < C::A_INSTR) copy16_to_lds(a_stage + a_src_off[m], as + instr * 1024);  // wave-uniform condition
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
  // A fragment of the 16-column substep q: chunk 2 q + qh of row i32 (+ 32 rb), at its swizzled place
  uint32_t a_lane_off[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) a_lane_off[q] = i32 * 128 + (((2 * q + qh) ^ ((i32 >> 1) & 7)) * 16);

  f32x16 acc[RB][CBS];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int cb = 0; cb < CBS; ++cb)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[rb][cb][e] = 0.f;

  // two consecutive 16-column substeps (q0, q0 + 1) at a time: one group of four transposing reads
  // per 32-column block brings the B fragments of both
  auto compute_pair = [&](int stage_idx, auto pair_tag) {
    constexpr int Q0 = 2 * decltype(pair_tag)::value;
    const uint32_t stage_addr = lds_base + (uint32_t)(b_buffer(stage_idx) - lds);
    const uint8_t* as = a_buffer(stage_idx);
    constexpr int R0 = (Q0 * 16 + 0) * C::ROW_BYTES, R1 = (Q0 * 16 + 4) * C::ROW_BYTES,
                  R2 = (Q0 * 16 + 16) * C::ROW_BYTES, R3 = (Q0 * 16 + 20) * C::ROW_BYTES;
    u32x2 r[CBS][4];
#pragma unroll
    for (int cb = 0; cb < CBS; ++cb)
      lds_read_tr16_x4<R0, R1, R2, R3>(stage_addr + b_lane_off[cb], r[cb][0], r[cb][1], r[cb][2], r[cb][3]);
    u32x4 a[2][RB];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
        a[h][rb] = *reinterpret_cast<const u32x4*>(as + rb * 4096 + a_lane_off[Q0 + h]);
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
    for (int h = 0; h < 2; ++h) {
      const u32x4 bf0 = u32x4{b0[4 * h], b0[4 * h + 1], b0[4 * h + 2], b0[4 * h + 3]};
      const u32x4 bf1 = u32x4{b1[4 * h], b1[4 * h + 1], b1[4 * h + 2], b1[4 * h + 3]};
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        acc[rb][0] = mfma_32x32x16<DT>(a[h][rb], bf0, acc[rb][0]);
        if constexpr (CBS == 2) acc[rb][1] = mfma_32x32x16<DT>(a[h][rb], bf1, acc[rb][1]);
      }
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
    compute_pair(s, std::integral_constant<int, 0>{});
    compute_pair(s, std::integral_constant<int, 1>{});
  }

  // ---- epilogue -------------------------------------------------------------------------------------------
  store_tile_rows<DT, RB, CBS, NB, WC, C::THREADS, C::Y_STRIDE>(acc, lds, Y, ldy, N, n0, relu, out_f32,
                                                                  [&](int row) -> int64_t { const int r = t * V + row; return pi_out ? pi_out[r] : r; });
}

// One thread per output element, fp32 fused multiply-adds in ascending vector-index order.
template <int DT>
__global__ __launch_bounds__(256) void spmm_vectors_plain_kernel(
    const uint16_t* __restrict__ vals_v, const int32_t* __restrict__ vec_idx, const int32_t* __restrict__ pi_in,
    const int32_t* __restrict__ pi_out, const uint16_t* __restrict__ X, int64_t ldx, void* __restrict__ Y,
    int64_t ldy, int M, int V, int Kv, int N, bool relu, bool out_f32) {
  const int n = blockIdx.x * 64 + (threadIdx.x & 63);
  const int r = blockIdx.y * 4 + (threadIdx.x >> 6);
  if (n >= N || r >= M) return;
  const uint16_t* vr = vals_v + (size_t)r * Kv;
  const int32_t* vi = vec_idx + (size_t)(r / V) * Kv;
  float acc = 0.f;
  for (int j = 0; j < Kv; ++j) {
    int c = vi[j];
    if (pi_in) c = pi_in[c];
    acc = __builtin_fmaf(bits_to_float<DT>(vr[j]), bits_to_float<DT>(X[(size_t)c * ldx + n]), acc);
  }
  if (relu) acc = acc > 0.f ? acc : 0.f;
  const int64_t row = pi_out ? pi_out[r] : r;
  if (out_f32) static_cast<float*>(Y)[row * ldy + n] = acc;
  else static_cast<uint16_t*>(Y)[row * ldy + n] = float_to_bits<DT>(acc);
}

template <int DT, int RB>
hipError_t launch_one(const VectorsArgs& a, hipStream_t stream) {
  constexpr int V = 32 * RB;
  const int T = a.s.M / V;
  const int n_blocks = (a.N + kNB - 1) / kNB;
  const int64_t work = (int64_t)n_blocks * T;
  const int work_per_xcd = (int)((work + 7) / 8);
  const size_t lds_bytes = total_lds_bytes(V);
  constexpr auto kernel = spmm_vectors_kernel<DT, RB>;
  if (hipError_t e = raise_lds_limit<kernel>((int)lds_bytes); e != hipSuccess) return e;
  kernel<<<dim3((unsigned)(work_per_xcd * 8)), kThreads, lds_bytes, stream>>>(
      static_cast<const uint16_t*>(a.vals_v), a.vec_idx, a.pi_in, a.pi_out, static_cast<const uint16_t*>(a.X), a.ldx,
      a.Y, a.ldy, T, a.s.Kv, a.N, n_blocks, work_per_xcd, a.relu, a.out_f32);
  return hipGetLastError();
}

template <int DT, int RB, int NB, int WC>
hipError_t launch_dma(const VectorsArgs& a, hipStream_t stream) {
  using C = DmaCfg<RB, NB, WC>;
  const int T = a.s.M / C::V;
  const int n_blocks = (a.N + NB - 1) / NB;
  const int64_t work = (int64_t)n_blocks * T;
  const int work_per_xcd = (int)((work + 7) / 8);
  constexpr auto kernel = spmm_vectors_dma_kernel<DT, RB, NB, WC>;
  if (hipError_t e = raise_lds_limit<kernel>(C::LDS_BYTES); e != hipSuccess) return e;
  kernel<<<dim3((unsigned)(work_per_xcd * 8)), C::THREADS, C::LDS_BYTES, stream>>>(
      static_cast<const uint16_t*>(a.vals_v), a.vec_idx, a.pi_in, a.pi_out, static_cast<const uint16_t*>(a.X), a.ldx,
      a.Y, a.ldy, T, a.s.Kv, a.N, n_blocks, work_per_xcd, a.relu, a.out_f32);
  return hipGetLastError();
}

template <int DT, int RB>
hipError_t launch_rb(const VectorsArgs& a, hipStream_t stream) {
  switch (spmm_vectors_variant(a)) {
    case 2: return launch_dma<DT, RB, 256, 64>(a, stream);
    case 3: return launch_dma<DT, RB, 512, 64>(a, stream);
    case 4: return launch_dma<DT, RB, 256, 32>(a, stream);
    case 5: return launch_dma<DT, RB, 512, 32>(a, stream);
    default: return launch_one<DT, RB>(a, stream);
  }
}

template <int DT>
hipError_t launch_dt(const VectorsArgs& a, hipStream_t stream) {
  switch (a.s.V) {
    case 32: return launch_rb<DT, 1>(a, stream);
    case 64: return launch_rb<DT, 2>(a, stream);
    case 96: return launch_rb<DT, 3>(a, stream);
    case 128: return launch_rb<DT, 4>(a, stream);
  }
  return hipErrorInvalidValue;
}

}  // namespace

// 1 = register-staged kernel, 2 / 3 = direct-to-LDS kernel with 256- / 512-column blocks and 64-column waves,
// 4 / 5 = the same blocks with 32-column waves (twice as many waves per workgroup).
int spmm_vectors_variant(const VectorsArgs& a) {
  if (a.variant) return a.variant;
  if (a.s.Kv % 64 != 0) return 1;
  // 512-column blocks halve the re-reads of the stored values; they pay when there are enough of them to
  // fill the chip and the k loop is long enough to amortise the larger start-up and epilogue
  const int64_t wide_blocks = (int64_t)(a.s.M / a.s.V) * ((a.N + 511) / 512);
  // Waves of 32 columns (twice as many per workgroup) cover the latency of a stage's copies better and read
  // more from LDS per MFMA: 5 to 20 % faster on every shape measured except the largest (16384 x 16384 x 8192).
  const int wide = wide_blocks <= 1024 ? 5 : 3;
  if (a.N >= 1024 && wide_blocks >= 256 && a.s.Kv >= 1024) return wide;
  if (a.N >= 1024 && wide_blocks >= 192 && a.s.V == 128) return wide;  // measured on 3072 x 768, N = 4096: 34.0 -> 23.3 us
  return 4;
}

bool spmm_vectors_mfma_supported(const VectorsArgs& a) {
  const int V = a.s.V;
  if (!(V == 32 || V == 64 || V == 96 || V == 128)) return false;
  if (a.ldx % 8 != 0 || a.ldy % 8 != 0) return false;
  if (a.variant < 0 || a.variant > 5 || (a.variant >= 2 && a.s.Kv % 64 != 0)) return false;
  const int64_t work = (int64_t)((a.N + kNB - 1) / kNB) * (a.s.M / V);
  return work < (1ll << 28);
}

hipError_t launch_spmm_vectors_mfma(const VectorsArgs& a, hipStream_t stream) {
  return a.s.dtype == HINM_F16 ? launch_dt<HINM_F16>(a, stream) : launch_dt<HINM_BF16>(a, stream);
}

hipError_t launch_spmm_vectors_plain(const VectorsArgs& a, hipStream_t stream) {
  dim3 grid((a.N + 63) / 64, (a.s.M + 3) / 4);
  if (grid.y > 65535u) return hipErrorInvalidConfiguration;
  auto v = static_cast<const uint16_t*>(a.vals_v);
  auto x = static_cast<const uint16_t*>(a.X);
  if (a.s.dtype == HINM_F16)
    spmm_vectors_plain_kernel<HINM_F16><<<grid, 256, 0, stream>>>(v, a.vec_idx, a.pi_in, a.pi_out, x, a.ldx, a.Y, a.ldy,
                                                                  a.s.M, a.s.V, a.s.Kv, a.N, a.relu, a.out_f32);
  else
    spmm_vectors_plain_kernel<HINM_BF16><<<grid, 256, 0, stream>>>(v, a.vec_idx, a.pi_in, a.pi_out, x, a.ldx, a.Y,
                                                                   a.ldy, a.s.M, a.s.V, a.s.Kv, a.N, a.relu, a.out_f32);
  return hipGetLastError();
}

}  // namespace hinm
