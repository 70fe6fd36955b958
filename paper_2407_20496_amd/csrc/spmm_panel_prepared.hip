// HiNM sparse GEMM with fused channel permutation for layers with few input channels (K <= 1024),
// from the device-tuned layer form (arXiv 2407.20496, Section 3.2; layout in prepared_layout.h).
//
// With one tile per workgroup every gathered input row feeds only V output rows, so the traffic
// from L2 into the compute units is T * Kv * N elements however the columns are blocked, and for
// V = 64 that traffic, not HBM, sets the time.  When a whole 64-column panel of X (all K rows) fits
// in LDS it is loaded ONCE per workgroup, in natural row order and fully coalesced, and the
// workgroup then multiplies many tiles against it: the gather by vector index (composed with the
// input-channel order) moves one level down and becomes the row address of the transposing LDS
// read that builds the B operand.  The tiles of a workgroup go round-robin to its waves, and from
// there on every wave runs on its own, with no workgroup barrier: it streams the tile's stored values
// and NM nibbles from global memory straight into the A operands (already in MFMA lane order),
// looks up the rows of the step in the gather table, and accumulates V x 64 outputs in fp32.
// Epilogue per tile and wave: optional ReLU, rounding, a private LDS staging area, then every output
// row leaves as one 128-byte segment to row pi_out[r] of Y.
#include "hinm_internal.h"
#include "mfma_types.h"
#include "prepared_layout.h"

namespace hinm {
namespace {

typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void global_void_t;

constexpr int kPanelCols = 64;
constexpr int kRowBytes = kPanelCols * 2;  // 128
constexpr int kYStride = kRowBytes + 16;   // staged output row

// Panel rows are 128 bytes = four 32-byte units; unit u of row r is stored at u ^ (r & 2).  The rows
// a transposing read touches are arbitrary (they follow the gather table), so conflicts cannot be
// excluded, but this spreads them over all four residues of r mod 4 instead of two.  The prepared
// layer carries the gather table as ready-made LDS addresses (see prepared_layout.h), padded kept
// columns pointing at an all-zero row behind the panel, so a B read costs one XOR of address math.

template <int DT, int RB, int kWaves>
__global__ __launch_bounds__(kWaves * 64) void spmm_panel_prepared_kernel(
    const uint8_t* __restrict__ prep_blocks, const uint32_t* __restrict__ panel_gather,
    const int32_t* __restrict__ out_rows, const uint16_t* __restrict__ X, int64_t ldx, void* __restrict__ Y,
    int64_t ldy, int K, int T, int S64, int N,
    int tile_groups, bool relu, bool out_f32) {
  constexpr int V = 32 * RB;
  // (tile, step) items whose global loads are in flight per wave; fewer for tall tiles (registers)
  constexpr int kDepth = (RB <= 2 && kWaves <= 8) ? 4 : 2;
  extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];  // panel, then one 32-row staging area per wave

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // Consecutive workgroup ids go to different XCDs.  The tile groups that share one column panel
  // get ids that are equal modulo 8, so the panel is fetched from HBM into one L2 only.
  const int nb = 8 * (blockIdx.x / (8 * tile_groups)) + (blockIdx.x & 7);
  const int tg = (blockIdx.x >> 3) % tile_groups;
  if (nb * kPanelCols >= N) return;
  const int n0 = nb * kPanelCols;
  const int Kp = S64 * 64;
  const int k_rows = (K + 7) / 8 * 8;  // panel rows in LDS (copies move 8 rows at a time)
  uint8_t* stage = lds + (size_t)(k_rows + 8) * kRowBytes + wave * (32 * kYStride);  // 8 zero rows behind the panel

  // ---- panel: all K rows of X, columns n0 .. n0+63, natural row order --------------------------------
  {
    const int p = lane & 7;           // 16-byte position inside the row
    const int r_in = lane >> 3;       // row inside the 8-row copy
    for (int r0 = wave * 8; r0 < k_rows; r0 += kWaves * 8) {
      const int r = min(r0 + r_in, K - 1);  // rows past K (padding to 8) re-read the last row, never used
      const int unit = (p >> 1) ^ (r0 + r_in & 2);
      const int col = (unit << 4) | ((p & 1) << 3);  // first of 8 columns
      const int n = (n0 + col < N) ? n0 + col : n0;  // columns past N are never stored: read valid memory
      __builtin_amdgcn_global_load_lds((global_void_t*)(X + (size_t)r * ldx + n), (lds_void_t*)(lds + r0 * kRowBytes), 16,
                                       0, 0);
    }
  }
  if (tid < 64) *reinterpret_cast<u32x4*>(lds + (size_t)k_rows * kRowBytes + tid * 16) = u32x4{0, 0, 0, 0};

  const int i32 = lane & 31;
  const int qh = lane >> 5;
  const int i16 = lane & 15;
  // per-lane constant of the B read address: 32-byte unit (2 cb + column half) and 8-byte piece
  uint32_t uc[2];
#pragma unroll
  for (int cb = 0; cb < 2; ++cb) uc[cb] = (uint32_t)((2 * cb + (i32 >> 4)) * 32 + (i16 & 3) * 8);

  // tiles of this workgroup: tg, tg + tile_groups, ...; wave w takes every kWaves-th of them.  The
  // wave walks the flat sequence of (tile, step) items of its tiles with the global loads of the next
  // kDepth - 1 items always in flight, across tile boundaries.
  const int t_first = tg + wave * tile_groups;
  const int t_stride = kWaves * tile_groups;
  const int my_tiles = (t_first < T) ? (T - t_first + t_stride - 1) / t_stride : 0;
  const int items = my_tiles * S64;

  struct StepRegs {
    u32x4 a_val[RB][2];
    int a_idx[RB];
    uint32_t row_entry;  // this lane's entry of the step's 64 gather-table entries (LDS address form)
  };
  auto load_item = [&](int f, StepRegs& r) {
    const int t = t_first + (f / S64) * t_stride;
    const int s = f % S64;
    const uint8_t* blk = prep_blocks + ((size_t)t * S64 + s) * RB * kPrepBlockBytes;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      r.a_val[rb][0] = *reinterpret_cast<const u32x4*>(blk + rb * kPrepBlockBytes + lane * 16);
      r.a_val[rb][1] = *reinterpret_cast<const u32x4*>(blk + rb * kPrepBlockBytes + 1024 + lane * 16);
      r.a_idx[rb] = *reinterpret_cast<const int*>(blk + rb * kPrepBlockBytes + kPrepIdxOffset + lane * 4);
    }
    // one coalesced load brings the step's 64 entries, lane l holding kept column 64 s + l
    r.row_entry = panel_gather[(size_t)t * Kp + 64 * s + lane];
  };
  // In the 8 transposing reads of a step (read q = 4 sub + 2 h + u) this lane addresses kept column
  // 32 sub + 16 h + 4 u + 8 qb + (i16 / 4) of the step; it takes that entry from the lane holding it.
  int src_lane_x4[8];
#pragma unroll
  for (int q = 0; q < 8; ++q)
    src_lane_x4[q] = 4 * (32 * (q >> 2) + 16 * ((q >> 1) & 1) + 4 * (q & 1) + 8 * qh + (i16 >> 2));

  f32x16 acc[RB][2];
  auto clear_acc = [&]() {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[rb][cb][e] = 0.f;
  };
  auto compute_item = [&](const StepRegs& r) {
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      u32x8 b[2];
#pragma unroll
      for (int hu = 0; hu < 4; ++hu) {
        const uint32_t e = (uint32_t)__builtin_amdgcn_ds_bpermute(src_lane_x4[4 * sub + hu], (int)r.row_entry);
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
          const u32x2 w = lds_read_tr16(reinterpret_cast<const uint8_t*>(lds) + (e ^ uc[cb]));
          b[cb][2 * hu] = w.x;
          b[cb][2 * hu + 1] = w.y;
        }
      }
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
          if (sub == 0) acc[rb][cb] = smfmac_32x32x32<DT, 0>(r.a_val[rb][0], b[cb], acc[rb][cb], r.a_idx[rb]);
          else acc[rb][cb] = smfmac_32x32x32<DT, 1>(r.a_val[rb][1], b[cb], acc[rb][cb], r.a_idx[rb]);
        }
    }
  };

  // output rows of the current tile for the store loop (row = lane / 8 + 8 k of every 32-row block),
  // fetched when the tile starts so that the epilogue does not wait for them
  int64_t tile_out_rows[RB][4];
  auto load_out_rows = [&](int t) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int k = 0; k < 4; ++k) tile_out_rows[rb][k] = out_rows[t * V + 32 * rb + 8 * k + (lane >> 3)];
  };
  auto epilogue = [&](int t) {
    // ---- epilogue of this tile (this wave only) ---------------------------------------------------------
    // D layout: lane holds column lane % 32, rows 8 * (reg / 4) + 4 * (lane / 32) + reg % 4.
    if (out_f32) {
      float* Yf = static_cast<float*>(Y);
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int r = t * V + 32 * rb + 8 * (e >> 2) + 4 * qh + (e & 3);
          const int64_t out_row = out_rows[r];
#pragma unroll
          for (int cb = 0; cb < 2; ++cb) {
            const int n = n0 + cb * 32 + i32;
            float v = acc[rb][cb][e];
            if (relu) v = v > 0.f ? v : 0.f;
            if (n < N) Yf[out_row * ldy + n] = v;
          }
        }
      return;
    }
    uint16_t* Yh = static_cast<uint16_t*>(Y);
    const int chunk = lane & 7;  // 8 lanes move one 128-byte row
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int row = 8 * (e >> 2) + 4 * qh + (e & 3);
          float v = acc[rb][cb][e];
          if (relu) v = v > 0.f ? v : 0.f;
          *reinterpret_cast<uint16_t*>(stage + row * kYStride + (cb * 32 + i32) * 2) = float_to_bits<DT>(v);
        }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int row = 8 * k + (lane >> 3);
        const int64_t out_row = tile_out_rows[rb][k];
        const int n = n0 + chunk * 8;
        const u32x4 v = *reinterpret_cast<const u32x4*>(stage + row * kYStride + chunk * 16);
        uint16_t* dst = Yh + out_row * ldy + n;
        if (n + 8 <= N) {
          __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(dst));
        } else if (n < N) {
          const uint32_t w[4] = {v.x, v.y, v.z, v.w};
          for (int e = 0; e < N - n; ++e) dst[e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
  };

  StepRegs ring[kDepth];
#pragma unroll
  for (int d = 0; d < kDepth - 1; ++d)
    if (d < items) load_item(d, ring[d]);
  if (items > 0) load_out_rows(t_first);
  clear_acc();
  __syncthreads();  // waits for the panel copies (and the first item loads), makes the panel visible
  int step_in_tile = 0, tile_no = 0;
  for (int f0 = 0; f0 < items; f0 += kDepth) {
#pragma unroll
    for (int d = 0; d < kDepth; ++d) {
      const int f = f0 + d;
      if (f < items) {  // wave-uniform
        if (f + kDepth - 1 < items) load_item(f + kDepth - 1, ring[(d + kDepth - 1) % kDepth]);
        compute_item(ring[d]);
        if (++step_in_tile == S64) {
          epilogue(t_first + tile_no * t_stride);
          clear_acc();
          step_in_tile = 0;
          ++tile_no;
          if (tile_no < my_tiles) load_out_rows(t_first + tile_no * t_stride);
        }
      }
    }
  }
}

inline size_t panel_lds_bytes(int K, int waves) {
  const int k_rows = (K + 7) / 8 * 8;
  return (size_t)(k_rows + 8) * kRowBytes + (size_t)waves * 32 * kYStride;
}

template <int DT, int RB, int WAVES>
hipError_t launch_waves(const PreparedArgs& a, int n_blocks, int tile_groups, hipStream_t stream) {
  const PreparedLayout L = prepared_layout(a.s);
  constexpr auto kernel = spmm_panel_prepared_kernel<DT, RB, WAVES>;
  const int nb8 = (n_blocks + 7) / 8 * 8;  // ids are laid out in groups of 8 column blocks
  if (a.plan) {
    plan_record(a.plan, "spmm_panel_prepared_kernel<DT=%d,RB=%d,WAVES=%d> grid=%d block=%d lds=%d", DT, RB, WAVES,
                nb8 * tile_groups, WAVES * 64, (int)panel_lds_bytes(a.s.K, WAVES));
    return hipSuccess;
  }
  if (hipError_t e = raise_lds_limit<kernel>(160 * 1024); e != hipSuccess) return e;
  const uint8_t* base = static_cast<const uint8_t*>(a.prepared);
  kernel<<<dim3((unsigned)(nb8 * tile_groups)), WAVES * 64, panel_lds_bytes(a.s.K, WAVES), stream>>>(
      base + L.a_offset, reinterpret_cast<const uint32_t*>(base + L.panel_offset),
      reinterpret_cast<const int32_t*>(base + L.pi_out_offset), static_cast<const uint16_t*>(a.X), a.ldx, a.Y, a.ldy,
      a.s.K, L.T, L.S, a.N, tile_groups, a.relu, a.out_f32);
  return hipGetLastError();
}

// Workgroups per column panel.  The panel fills most of a compute unit's LDS, so a unit holds one workgroup,
// and panel p runs on XCD p % 8 (32 units): the panels of the busiest XCD times the groups fit one round
// (3072 x 768 at N = 768, twelve panels: 22 groups gave that XCD 44 workgroups, 13.6 us; 16 groups: 8.9 us).
inline int panel_tile_groups(int n_blocks) {
  const int panels_per_xcd = (n_blocks + 7) / 8;
  return panels_per_xcd >= 32 ? 1 : 32 / panels_per_xcd;
}

template <int DT, int RB>
hipError_t launch_rb(const PreparedArgs& a, hipStream_t stream) {
  const PreparedLayout L = prepared_layout(a.s);
  const int n_blocks = (a.N + kPanelCols - 1) / kPanelCols;
  int tile_groups = panel_tile_groups(n_blocks);
  if (tile_groups > L.T) tile_groups = L.T;
  const int tiles_per_wg = (L.T + tile_groups - 1) / tile_groups;
  // one tile per wave when registers and LDS allow it: the waves then finish together
  if (RB <= 2 && tiles_per_wg > 8 && panel_lds_bytes(a.s.K, 12) <= 160 * 1024)
    return launch_waves<DT, RB, 12>(a, n_blocks, tile_groups, stream);
  if (tiles_per_wg <= 4) return launch_waves<DT, RB, 4>(a, n_blocks, tile_groups, stream);
  return launch_waves<DT, RB, 8>(a, n_blocks, tile_groups, stream);
}

}  // namespace

bool spmm_panel_prepared_supported(const PreparedArgs& a) {
  return panel_lds_bytes(a.s.K, 8) <= 160 * 1024 && a.N > 32 && a.ldx % 8 == 0 && a.ldy % 8 == 0;
}

// Measured on layers with K = 576 and 768: with fewer than four tiles most waves of a workgroup have
// no tile to multiply and the tile kernel is 1.3-1.9x faster; with 128-row tiles, six or more
// 64-column steps and enough 512-column blocks to occupy half the chip the wide tile kernel wins too.
bool spmm_panel_prepared_preferred(const PreparedArgs& a) {
  if (!spmm_panel_prepared_supported(a)) return false;
  const PreparedLayout L = prepared_layout(a.s);
  if (L.T < 4) return false;
  // a workgroup that stages a panel for one tile only pays the staging for nothing (3072 x 768 at N = 256:
  // 13 us against 7 us for the tile kernel; at N = 512, with two tiles per workgroup, 8 against 9)
  const int n_blocks = (a.N + kPanelCols - 1) / kPanelCols;
  if (L.T <= panel_tile_groups(n_blocks)) return false;
  // column panel p runs on XCD p % 8: fewer than eight panels leave whole XCDs idle (3072 x 768 at N = 384,
  // six panels: 13.3 us against 8.9 us)
  if (n_blocks < 8) return false;
  const int64_t wide_blocks = (int64_t)L.T * ((a.N + 511) / 512);
  if (L.RB == 4 && L.S >= 6 && a.N >= 1024 && wide_blocks >= 128) return false;
  return true;
}

hipError_t launch_spmm_panel_prepared(const PreparedArgs& a, hipStream_t stream) {
  const int RB = a.s.V / 32;
#define HINM_RB(DT)                              \
  switch (RB) {                                  \
    case 1: return launch_rb<DT, 1>(a, stream);  \
    case 2: return launch_rb<DT, 2>(a, stream);  \
    case 3: return launch_rb<DT, 3>(a, stream);  \
    case 4: return launch_rb<DT, 4>(a, stream);  \
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
