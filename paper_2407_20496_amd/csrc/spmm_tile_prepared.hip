// HiNM sparse GEMM with fused channel permutation, many columns, from the device-tuned layer form
// (arXiv 2407.20496, Section 3.2 and Section 5.3; layout in prepared_layout.h).
//
// One workgroup computes one tile of V = 32 * RB output channels for a block of NB columns.  The
// tile's kept input channels are walked in stages of KS = 32 * KSUB columns, ST stages deep:
//   global -> LDS : direct-to-LDS loads, no registers in between.  The KS input rows named by the
//                   gather table (vector index composed with the input-channel order) arrive as
//                   contiguous NB-column row segments; the tile's stored values and NM nibbles for
//                   the stage are one contiguous chunk already in MFMA lane order.  Channel
//                   re-ordering costs nothing here: the table lookup is the one the format needs.
//   LDS -> MFMA   : every wave owns 64 of the NB columns and all V rows; A fragments are linear
//                   16-byte LDS reads, B fragments use the transposing LDS read on rows whose
//                   32-byte units are XOR-swizzled (applied on the source address of the copy) so
//                   that the four rows of one read fall on different banks; the NM nibbles go
//                   unchanged into the index operand of the 32x32x32 sparse MFMA.
//   epilogue      : fp32 accumulators -> optional ReLU -> 16 bit, staged through LDS so that every
//                   output row leaves as one contiguous segment to row pi_out[r] of Y.
// The stage being multiplied, and the ST - 1 stages in flight behind it, are separated by one
// workgroup barrier per stage and by explicit counts of outstanding copies.
#include "hinm_internal.h"
#include "mfma_types.h"
#include "prepared_layout.h"
#include "direct_lds.h"
#include "tile_epilogue.h"

#include <type_traits>

namespace hinm {
namespace {

template <int RB, int NB, int KSUB, int ST, int WC>
struct TileCfg {
  static constexpr int NW = NB / WC;                            // waves; each owns WC of the NB columns
  static constexpr int CBS = WC / 32;                           // 32-column accumulator blocks per wave
  static constexpr int THREADS = NW * 64;
  static constexpr int KS = 32 * KSUB;
  static constexpr int ROW_BYTES = NB * 2;
  static constexpr int B_BYTES = KS * ROW_BYTES;
  static constexpr int STEPS = (KSUB + 1) / 2;                   // 64-column steps per stage (KSUB = 1: half a step)
  static constexpr int SUBS = KSUB / STEPS;                      // 32-column substeps per step and stage
  static constexpr int A_RB_BYTES = SUBS * 1024 + 256;           // per step and row block: values of its substeps + nibbles
  static constexpr int A_GRANULES = STEPS * RB * (SUBS * 64 + 16);
  static constexpr int A_INSTR = (A_GRANULES + 63) / 64;         // wave-wide copies for A per stage
  static constexpr int A_BYTES = A_INSTR * 1024;                 // rounded up: the last copy may overshoot
  // LDS: ST buffers for the gathered rows (B), then ST buffers for the stored values (A).  (Requesting
  // the A chunk one stage earlier than its rows, with a third A buffer, was measured slower on every
  // shape: 5 to 10 %.)
  static constexpr int STAGES_BYTES = ST * (B_BYTES + A_BYTES);
  static constexpr int B_PER_WAVE = (NB == 512 ? KS : KS / 2) / NW;  // wave-wide copies for B per wave and stage
  static constexpr int ROWS_PER_WAVE = KS / NW;
  static constexpr int Y_STRIDE = NB * 2 + 16;
  static constexpr int EPI_BYTES = 32 * RB * Y_STRIDE;
  static constexpr int LDS_BYTES = (STAGES_BYTES > EPI_BYTES) ? STAGES_BYTES : EPI_BYTES;
  static_assert(NB == 256 || NB == 512, "column block");
  static_assert(WC == 64 || WC == 32, "columns per wave");
  static_assert(KSUB == 1 || KSUB == 2 || KSUB == 4, "half a step, one step or two steps per stage");
  static_assert(B_PER_WAVE * NW * (NB == 512 ? 1 : 2) == KS, "copy split");
  static_assert(ST == 2 || B_PER_WAVE == 4 * KSUB, "deeper pipelines: the wait table assumes four copies per substep");
  static_assert(ST >= 2 && ST <= 4 && (A_INSTR + NW - 1) / NW <= 3, "wait table covers these");
  // 512-column blocks, two stages: the copies of the next stage are issued in KSUB chunks, one in front of every
  // substep of the current stage (the stored values with the first), instead of in one burst behind the barrier.
  // Measured on 16384 x 16384 at N = 8192: 1455 -> 1388 us; 11008 x 4096 at N = 2048: 96.9 -> 92.4 us.  For
  // 256-column blocks the same split is neutral to 10 % slower, and uneven splits or the stored values in a later
  // chunk are slower everywhere.
  static constexpr bool CHUNKED_ISSUE = NB == 512 && ST == 2 && KSUB >= 2 && B_PER_WAVE % KSUB == 0;
};

// PART 0 is the product.  PART 1 and 2 are measurement aids (hinm_calib_tile_part): the same launch with only the
// copy stream (no LDS reads, no MFMAs), or only the LDS reads and MFMAs (no copies after the prologue, so the
// operands are whatever the first stages left in LDS); neither stores anything.
template <int DT, int RB, int NB, int KSUB, int ST, int WC, int PART = 0>
__global__ __launch_bounds__(NB / WC * 64) void spmm_tile_prepared_kernel(
    const uint8_t* __restrict__ prep_blocks, const int32_t* __restrict__ gather, const int32_t* __restrict__ out_rows,
    const uint8_t* __restrict__ zeros, const uint16_t* __restrict__ X, int64_t ldx, void* __restrict__ Y, int64_t ldy,
    int T, int S64, int N, int n_blocks, int work_per_xcd, bool relu, bool out_f32) {
  using C = TileCfg<RB, NB, KSUB, ST, WC>;
  constexpr int CBS = C::CBS;
  constexpr int V = 32 * RB;
  constexpr int NW = C::NW;
  constexpr int KS = C::KS;
  extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];

  // Consecutive workgroup ids go to different XCDs: give every XCD a contiguous run of the
  // column-block-major work list, so the tiles running together on one XCD share a column panel of
  // X in that XCD's L2.
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
  const int stages_total = (KSUB == 4) ? S64 / 2 : S64 * (2 / KSUB);  // stages of KS columns (KSUB = 4: S64 is even)
  const int Kp = S64 * 64;

  const int32_t* gt = gather + (size_t)t * Kp;
  const uint8_t* a_tile = prep_blocks + (size_t)t * S64 * RB * kPrepBlockBytes;

  // ---- copy roles ---------------------------------------------------------------------------------
  // B: this wave copies rows [wave * ROWS_PER_WAVE, +ROWS_PER_WAVE) of every stage.
  //    NB = 512: one copy per row, lane = 16-byte granule position in the row;
  //    NB = 256: one copy per row pair, lanes 0..31 the even row, 32..63 the odd row.
  // A copy's source is a wave-uniform row base (X row from the gather table, or the zero row for
  // padded kept columns) plus a per-lane byte offset that depends only on row % 4 (the swizzle):
  // the offsets are computed once.  Lanes whose columns lie beyond N re-read the block's first
  // columns instead: those accumulator columns are never stored.
  const RowSegmentCopy<NB> b_copy(lane, n0, N);
  // A: wave-wide copies number wave, wave + NW, ... of the stage's chunk; per-lane source offsets
  constexpr int A_ROUNDS = (C::A_INSTR + NW - 1) / NW;
  uint32_t a_src_off[A_ROUNDS];
  uint32_t a_src_odd_stage[A_ROUNDS];  // KSUB == 1: extra offset on odd stages (second half of the values)
#pragma unroll
  for (int m = 0; m < A_ROUNDS; ++m) {
    const int gran = min((wave + m * NW) * 64 + lane, C::A_GRANULES - 1);  // overshoot re-reads the last granule
    if constexpr (KSUB >= 2) {
      a_src_off[m] = gran * 16;
      a_src_odd_stage[m] = 0;
    } else {
      const int rb = gran / 80, r = gran % 80;
      a_src_off[m] = rb * kPrepBlockBytes + ((r < 64) ? r * 16 : kPrepIdxOffset + (r - 64) * 16);
      a_src_odd_stage[m] = (r < 64) ? 1024 : 0;
    }
  }
  typedef int rows_t __attribute__((ext_vector_type(C::ROWS_PER_WAVE)));
  auto load_rows = [&](int stage_idx) -> rows_t {
    // the wave's ROWS_PER_WAVE consecutive gather-table entries of a stage (wave-uniform: scalar load)
    const int st = min(stage_idx, stages_total - 1);
    return *reinterpret_cast<const rows_t*>(gt + st * KS + wave * C::ROWS_PER_WAVE);
  };
  const uint8_t* x_block = reinterpret_cast<const uint8_t*>(X + n0);
  auto row_base = [&](int g) -> const uint8_t* {  // wave-uniform
    return (g >= 0) ? x_block + (size_t)g * ldx * 2 : zeros;
  };
  auto b_buffer = [&](int stage_idx) -> uint8_t* { return lds + (stage_idx % ST) * C::B_BYTES; };
  auto a_buffer = [&](int stage_idx) -> uint8_t* { return lds + ST * C::B_BYTES + (stage_idx % ST) * C::A_BYTES; };
  auto issue_b = [&](int stage_idx, const rows_t rows) {
    uint8_t* stage = b_buffer(stage_idx);
    b_copy.template issue<C::B_PER_WAVE, C::ROW_BYTES>([&](int j) { return row_base(rows[j]); },
                                                        stage + wave * C::ROWS_PER_WAVE * C::ROW_BYTES);
  };
  auto issue_a = [&](int stage_idx) {
    uint8_t* a_lds = a_buffer(stage_idx);
    const uint8_t* a_stage = (KSUB >= 2) ? a_tile + (size_t)stage_idx * C::STEPS * RB * kPrepBlockBytes
                                         : a_tile + (size_t)(stage_idx >> 1) * RB * kPrepBlockBytes;
#pragma unroll
    for (int m = 0; m < A_ROUNDS; ++m) {
      const int instr = wave + m * NW;
      if (instr < C::A_INSTR) {  // wave-uniform
        const uint32_t off = a_src_off[m] + ((stage_idx & 1) ? a_src_odd_stage[m] : 0u);
        copy16_to_lds(a_stage + off, a_lds + instr * 1024);
      }
    }
  };
  const int extra_copies = (C::A_INSTR - wave + NW - 1) / NW;  // A copies of this wave per stage

  // ---- MFMA roles -----------------------------------------------------------------------------------
  const int i32 = lane & 31;  // A row / B column inside a 32-block
  const int qh = lane >> 5;   // lane group
  const int i16 = lane & 15;
  const int sw_lane = swizzle_of_row(i16 >> 2);
  int b_col_off[CBS];
#pragma unroll
  for (int cb = 0; cb < CBS; ++cb)
    b_col_off[cb] = (((wave * (WC / 16) + cb * 2 + (i32 >> 4)) ^ sw_lane) * 32) + (i16 & 3) * 8;
  const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_void_t*)lds;
  // per-lane part of the transposing-read address: row 8 qb + (i16 / 4), swizzled column unit
  uint32_t b_lane_off[CBS];
#pragma unroll
  for (int cb = 0; cb < CBS; ++cb) b_lane_off[cb] = (8 * qh + (i16 >> 2)) * C::ROW_BYTES + b_col_off[cb];

  f32x16 acc[RB][CBS];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int cb = 0; cb < CBS; ++cb)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[rb][cb][e] = 0.f;

  // B slots 8 h + 4 u .. + 3 of lane group qb <- rows 16 h + 8 qb + 4 u + (0..3) of the substep
  auto read_b = [&](uint32_t stage_addr, int cb, auto sub_tag) -> u32x8 {
    constexpr int Q = decltype(sub_tag)::value;  // 32-column substep of the stage
    constexpr int R0 = (Q * 32 + 0) * C::ROW_BYTES, R1 = (Q * 32 + 4) * C::ROW_BYTES,
                  R2 = (Q * 32 + 16) * C::ROW_BYTES, R3 = (Q * 32 + 20) * C::ROW_BYTES;
    u32x2 r0, r1, r2, r3;
    lds_read_tr16_x4<R0, R1, R2, R3>(stage_addr + b_lane_off[cb], r0, r1, r2, r3);
    return u32x8{r0.x, r0.y, r1.x, r1.y, r2.x, r2.y, r3.x, r3.y};
  };

  auto compute_sub = [&](int stage_idx, auto sub_tag) {
    const uint8_t* stage = b_buffer(stage_idx);
    // Q = 32-column substep of the stage; it belongs to step Q / SUBS of the stage and is substep
    // SUB of that step (the substep picks the half of the step's index word, ABID)
    constexpr int Q = decltype(sub_tag)::value;
    constexpr int STEP = Q / C::SUBS, SUB = Q % C::SUBS;
    const uint8_t* as = a_buffer(stage_idx);
    const uint32_t stage_addr = lds_base + (uint32_t)(stage - lds);
    u32x8 b0 = read_b(stage_addr, 0, sub_tag);
    u32x8 b1 = b0;
    if constexpr (CBS == 2) b1 = read_b(stage_addr, 1, sub_tag);
    u32x4 a[RB];
    int idx[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const uint8_t* blk = as + (STEP * RB + rb) * C::A_RB_BYTES;
      a[rb] = *reinterpret_cast<const u32x4*>(blk + SUB * 1024 + lane * 16);
      idx[rb] = *reinterpret_cast<const int*>(blk + C::SUBS * 1024 + lane * 4);
      // the index register holds the nibbles of both substeps of a 64-column step
      if (KSUB == 1 && (stage_idx & 1)) idx[rb] = (int)((uint32_t)idx[rb] >> 16);
    }
    if constexpr (CBS == 2) lds_wait_tr(b0, b1);
    else lds_wait_tr(b0);
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      if constexpr (SUB == 1) {
        acc[rb][0] = smfmac_32x32x32<DT, 1>(a[rb], b0, acc[rb][0], idx[rb]);
        if constexpr (CBS == 2) acc[rb][1] = smfmac_32x32x32<DT, 1>(a[rb], b1, acc[rb][1], idx[rb]);
      } else {
        acc[rb][0] = smfmac_32x32x32<DT, 0>(a[rb], b0, acc[rb][0], idx[rb]);
        if constexpr (CBS == 2) acc[rb][1] = smfmac_32x32x32<DT, 0>(a[rb], b1, acc[rb][1], idx[rb]);
      }
    }
  };
  auto compute_stage = [&](int stage_idx) {
    compute_sub(stage_idx, std::integral_constant<int, 0>{});
    if constexpr (KSUB >= 2) compute_sub(stage_idx, std::integral_constant<int, 1>{});
    if constexpr (KSUB == 4) {
      compute_sub(stage_idx, std::integral_constant<int, 2>{});
      compute_sub(stage_idx, std::integral_constant<int, 3>{});
    }
  };

  // ---- pipeline ---------------------------------------------------------------------------------------
  // Issue order: B(0) A(0) B(1) A(1) ... up to the pipeline depth, then per iteration s the copies
  // of stage s + ST - 1.  Copies complete in issue order.
#pragma unroll
  for (int p = 0; p < ST - 1; ++p)
    if (p < stages_total) {
      issue_b(p, load_rows(p));
      issue_a(p);
    }
  rows_t rows_next = load_rows(ST - 1);
  for (int s = 0; s < stages_total; ++s) {
    // stage s must have landed; the stages issued after it may still be in flight
    const int later = min(ST - 2, stages_total - 1 - s);
    if constexpr (ST == 2) wait_copies_outstanding<0>();
    else wait_copies_outstanding<C::B_PER_WAVE>(later, extra_copies);
    __builtin_amdgcn_s_barrier();
    const int nxt = s + ST - 1;
    if constexpr (C::CHUNKED_ISSUE) {
      constexpr int CH = C::B_PER_WAVE / KSUB;
      const bool more = PART != 2 && nxt < stages_total;  // uniform over the workgroup
      const rows_t rows_now = rows_next;
      rows_next = load_rows(nxt + 1);
      uint8_t* rows_lds = b_buffer(nxt) + wave * C::ROWS_PER_WAVE * C::ROW_BYTES;
      auto base_of = [&](int j) { return row_base(rows_now[j]); };
      if (more) {
        b_copy.template issue_range<0, CH, C::ROW_BYTES>(base_of, rows_lds);
        issue_a(nxt);
      }
      if constexpr (PART != 1) compute_sub(s, std::integral_constant<int, 0>{});
      if (more) b_copy.template issue_range<CH, CH, C::ROW_BYTES>(base_of, rows_lds);
      if constexpr (PART != 1) compute_sub(s, std::integral_constant<int, 1>{});
      if constexpr (KSUB == 4) {
        if (more) b_copy.template issue_range<2 * CH, CH, C::ROW_BYTES>(base_of, rows_lds);
        if constexpr (PART != 1) compute_sub(s, std::integral_constant<int, 2>{});
        if (more) b_copy.template issue_range<3 * CH, CH, C::ROW_BYTES>(base_of, rows_lds);
        if constexpr (PART != 1) compute_sub(s, std::integral_constant<int, 3>{});
      }
    } else {
      if (PART != 2 && nxt < stages_total) {
        issue_b(nxt, rows_next);
        issue_a(nxt);
      }
      rows_next = load_rows(nxt + 1);
      if constexpr (PART != 1) compute_stage(s);
    }
  }
  if constexpr (PART != 0) {
    // keeps the accumulators alive without ever storing them: no launch has a negative column count
    if (N >= 0) return;
  }

  // ---- epilogue -------------------------------------------------------------------------------------
  store_tile_rows<DT, RB, CBS, NB, WC, C::THREADS, C::Y_STRIDE>(
      acc, lds, Y, ldy, N, n0, relu, out_f32, [&](int row) -> int64_t { return out_rows[t * V + row]; });
}

// Launches the tiles [tile_base, tile_base + tile_count) of the layer (tile_count < 0: all of them).  The kernel
// numbers its tiles from zero: the tables it indexes by tile are handed over already advanced to tile_base.
template <int DT, int RB, int NB, int KSUB, int ST, int WC = 64, int PART = 0>
hipError_t launch_cfg(const PreparedArgs& a, hipStream_t stream, int tile_base = 0, int tile_count = -1) {
  using C = TileCfg<RB, NB, KSUB, ST, WC>;
  const PreparedLayout L = prepared_layout(a.s);
  const int T = tile_count < 0 ? L.T : tile_count;
  const int n_blocks = (a.N + NB - 1) / NB;
  const int64_t work = (int64_t)n_blocks * T;
  const int work_per_xcd = (int)((work + 7) / 8);
  constexpr auto kernel = spmm_tile_prepared_kernel<DT, RB, NB, KSUB, ST, WC, PART>;
  if (a.plan) {
    plan_record(a.plan, "spmm_tile_prepared_kernel<DT=%d,RB=%d,NB=%d,KSUB=%d,ST=%d,WC=%d%s> tiles=%d..%d grid=%d block=%d lds=%d",
                DT, RB, NB, KSUB, ST, WC, PART == 1 ? ",copies only" : PART == 2 ? ",LDS reads and MFMAs only" : "", tile_base, tile_base + T - 1, work_per_xcd * 8, C::THREADS, C::LDS_BYTES);
    return hipSuccess;
  }
  if (hipError_t e = raise_lds_limit<kernel>(C::LDS_BYTES); e != hipSuccess) return e;
  const uint8_t* base = static_cast<const uint8_t*>(a.prepared);
  const size_t tb = (size_t)tile_base;
  kernel<<<dim3((unsigned)(work_per_xcd * 8)), C::THREADS, C::LDS_BYTES, stream>>>(
      base + L.a_offset + tb * L.S * RB * kPrepBlockBytes,
      reinterpret_cast<const int32_t*>(base + L.gather_offset) + tb * L.S * 64,
      reinterpret_cast<const int32_t*>(base + L.pi_out_offset) + tb * (32 * RB), base + L.zero_offset,
      static_cast<const uint16_t*>(a.X), a.ldx, a.Y, a.ldy, T, L.S, a.N, n_blocks, work_per_xcd, a.relu, a.out_f32);
  return hipGetLastError();
}

// By shape.  Wide column blocks halve the re-reads of the stored values when there are enough of them
// to fill the chip.  Waves of 32 columns (twice as many waves per workgroup) hide the latency of a stage's
// copies better and cost 40 % more LDS reads per MFMA: they win wherever a compute unit holds a single
// workgroup and the layer is not large enough to be bound by LDS and L2 throughput (measured on the
// encoder, convolution and MLP shapes: 5 to 20 %; the 16384 x 16384 x 8192 layer is 2 % slower with them).
// A round of workgroups is one serial pass over the kept columns however few workgroups it holds, and a pass of
// a 512-column block costs about 1.35 passes of a 256-column block (128-row tiles, whose workgroups sit alone
// on a compute unit).  True when the 256-column blocks need fewer passes by that count (11008 x 4096 at
// N = 1280: 430 narrow blocks in two rounds, 74 us, against 258 wide blocks in two rounds, 89 us).
inline bool narrow_blocks_save_rounds(const PreparedLayout& L, int64_t wide_blocks, int64_t blocks) {
  return L.RB == 4 && (double)((blocks + 255) / 256) < ((wide_blocks + 255) / 256) * 1.35;
}

inline int choose_variant(const PreparedArgs& a) {
  const PreparedLayout L = prepared_layout(a.s);
  const int64_t wide_blocks = (int64_t)L.T * ((a.N + 511) / 512);
  // 512 columns, 64-column stages, 2 deep: sixteen 32-column waves up to a few rounds of workgroups, eight
  // 64-column waves beyond
  const int64_t blocks = (int64_t)L.T * ((a.N + 255) / 256);
  if (a.N >= 1024 && wide_blocks >= 256 && !narrow_blocks_save_rounds(L, wide_blocks, blocks))
    return (wide_blocks <= 1024 || L.RB <= 2) ? 16 : 3;  // tiles of up to 64 rows: sixteen waves measured 1-5 % ahead at any size
  // ... and wherever they save rounds of workgroups: a round is one serial pass over the kept columns however
  // few workgroups it holds, and a pass of a 512-column block costs about 1.35 passes of a 256-column block
  // (11008 x 4096 at N = 768: 258 narrow blocks, two rounds, 72 us; 172 wide blocks, one round, 47 us).  For
  // 128-row tiles only, whose workgroups sit alone on a compute unit: with 32-row tiles several share one and
  // 384 of them are no two rounds (768 x 3072, V = 32, at N = 4096: the narrow blocks stay 2 us ahead).
  if (a.N > 256 && L.RB == 4 && L.S > 8 && ((wide_blocks + 255) / 256) * 1.35 < (double)((blocks + 255) / 256)) return 16;
  // short k loops: 32-column stages, 2 deep, so that several workgroups share a compute unit and cover each
  // other's start-up and epilogue (128-row tiles with at least half as many wide blocks as units; or many
  // workgroups per unit)
  if (a.N >= 1024 && L.RB == 4 && L.S <= 8 && wide_blocks >= 128) return 17;
  if (L.S <= 8 && blocks > 512) return 17;
  // At most one workgroup per compute unit: every stage then waits one full memory round trip, and
  // 128-column stages halve the number of round trips.
  if (L.RB <= 2 && L.S % 2 == 0 && blocks <= 256) return 13;
  // 128-row tiles, more than one round of 256-column blocks but at most two, and 512-column blocks not chosen
  // above: with 32-column stages two workgroups share a compute unit and all of them run at once
  // (11008 x 4096 at N = 1280, 430 blocks: 74 -> 63 us; 16384 x 4096 with 512 kept columns at N = 768: 26 -> 22 us)
  if (L.RB == 4 && blocks > 256 && blocks <= 512) return 17;
  return 14;                                        // 256 columns, 64-column stages, 2 deep
}

// A layer whose wide blocks fill the chip a whole number of times plus a small remainder would spend a full
// round on that remainder.  The tiles of the whole rounds keep the wide configuration; the remaining tiles are
// launched behind them with 256-column blocks, twice as many workgroups of about half the duration, when
// those fit one round.  Returns false when the shape does not ask for it.
template <int DT, int RB>
bool launch_split_rounds(const PreparedArgs& a, hipStream_t stream, hipError_t* result) {
  const PreparedLayout L = prepared_layout(a.s);
  const int nbw = (a.N + 511) / 512;
  const int64_t wide_blocks = (int64_t)L.T * nbw;
  if (a.N < 1024 || wide_blocks <= 256 || wide_blocks > 1024) return false;
  if (narrow_blocks_save_rounds(L, wide_blocks, (int64_t)L.T * ((a.N + 255) / 256))) return false;
  const int rounds = (int)(wide_blocks / 256), rest = (int)(wide_blocks % 256);
  if (rest == 0 || rest > 128) return false;
  const int t_wide = 256 * rounds / nbw, t_rest = L.T - t_wide;
  if (t_wide <= 0 || (int64_t)t_rest * ((a.N + 255) / 256) > 256) return false;
  *result = launch_cfg<DT, RB, 512, 2, 2, 32>(a, stream, 0, t_wide);
  if (*result != hipSuccess) return true;
  if (RB <= 2 && L.S % 2 == 0) {
    if constexpr (RB <= 2) *result = launch_cfg<DT, RB, 256, 4, 2, 32>(a, stream, t_wide, t_rest);
  } else {
    *result = launch_cfg<DT, RB, 256, 2, 2, 32>(a, stream, t_wide, t_rest);
  }
  return true;
}

template <int DT, int RB>
hipError_t launch_rb(const PreparedArgs& a, hipStream_t stream) {
  if (a.tile_variant == 0) {
    hipError_t e;
    if (launch_split_rounds<DT, RB>(a, stream, &e)) return e;
  }
  switch (a.tile_variant ? a.tile_variant : choose_variant(a)) {
    case 1: return launch_cfg<DT, RB, 256, 2, 2>(a, stream);
    case 2: return launch_cfg<DT, RB, 256, 2, 3>(a, stream);
    case 3: return launch_cfg<DT, RB, 512, 2, 2>(a, stream);
    case 4: return launch_cfg<DT, RB, 256, 1, 3>(a, stream);
    case 5: return launch_cfg<DT, RB, 256, 1, 4>(a, stream);
    case 6: return launch_cfg<DT, RB, 512, 1, 3>(a, stream);
    case 7: return launch_cfg<DT, RB, 512, 1, 4>(a, stream);
    case 8: return launch_cfg<DT, RB, 256, 1, 2>(a, stream);
    case 9: return launch_cfg<DT, RB, 512, 1, 2>(a, stream);
    case 10:  // two 64-column steps per stage: needs an even number of steps and V <= 64 (LDS)
      if constexpr (RB <= 2) {
        if (prepared_layout(a.s).S % 2 == 0) return launch_cfg<DT, RB, 256, 4, 2>(a, stream);
      }
      break;
    case 13:  // as 10, eight waves of 32 columns each
      if constexpr (RB <= 2) {
        if (prepared_layout(a.s).S % 2 == 0) return launch_cfg<DT, RB, 256, 4, 2, 32>(a, stream);
      }
      break;
    case 14: return launch_cfg<DT, RB, 256, 2, 2, 32>(a, stream);  // as 1, eight waves of 32 columns each
    case 16: return launch_cfg<DT, RB, 512, 2, 2, 32>(a, stream);  // as 3, sixteen waves of 32 columns each
    case 17: return launch_cfg<DT, RB, 256, 1, 2, 32>(a, stream);  // as 8, eight waves of 32 columns each
    default: break;
  }
  return launch_cfg<DT, RB, 256, 2, 3>(a, stream);
}

// One part of the kernel that launch_rb would choose for this shape, for the configurations the named
// workloads use (tiles of 64 and 128 rows); anything else is refused.
template <int DT, int RB, int PART>
hipError_t launch_part_rb(const PreparedArgs& a, hipStream_t stream) {
  switch (choose_variant(a)) {
    case 3: return launch_cfg<DT, RB, 512, 2, 2, 64, PART>(a, stream);
    case 16: return launch_cfg<DT, RB, 512, 2, 2, 32, PART>(a, stream);
    case 14: return launch_cfg<DT, RB, 256, 2, 2, 32, PART>(a, stream);
    case 17: return launch_cfg<DT, RB, 256, 1, 2, 32, PART>(a, stream);
    case 13:
      if constexpr (RB <= 2) return launch_cfg<DT, RB, 256, 4, 2, 32, PART>(a, stream);
      break;
    default: break;
  }
  return hipErrorNotSupported;
}

}  // namespace

hipError_t launch_spmm_tile_prepared_part(const PreparedArgs& a, int part, hipStream_t stream) {
  if ((a.s.V != 64 && a.s.V != 128) || (part != 1 && part != 2)) return hipErrorNotSupported;
#define HINM_PART(DT)                                                                                   \
  if (a.s.V == 64) return part == 1 ? launch_part_rb<DT, 2, 1>(a, stream) : launch_part_rb<DT, 2, 2>(a, stream); \
  return part == 1 ? launch_part_rb<DT, 4, 1>(a, stream) : launch_part_rb<DT, 4, 2>(a, stream);
  if (a.s.dtype == HINM_F16) {
    HINM_PART(HINM_F16)
  } else {
    HINM_PART(HINM_BF16)
  }
#undef HINM_PART
}

hipError_t launch_spmm_tile_prepared(const PreparedArgs& a, hipStream_t stream) {
  const int RB = a.s.V / 32;
#define HINM_RB(DT)                                   \
  switch (RB) {                                       \
    case 1: return launch_rb<DT, 1>(a, stream);       \
    case 2: return launch_rb<DT, 2>(a, stream);       \
    case 3: return launch_rb<DT, 3>(a, stream);       \
    case 4: return launch_rb<DT, 4>(a, stream);       \
  }
  if (a.s.dtype == HINM_F16) {
    HINM_RB(HINM_F16)
  } else {
    HINM_RB(HINM_BF16)
  }
#undef HINM_RB
  return hipErrorInvalidValue;
}

}  // namespace hinm
