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
  // D layout: lane holds column lane % 32, rows 8 * (reg / 4) + 4 * (lane / 32) + reg % 4.
  if (out_f32) {
    float* Yf = static_cast<float*>(Y);
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int r = t * V + 32 * rb + 8 * (e >> 2) + 4 * qh + (e & 3);
        const int64_t out_row = pi_out ? pi_out[r] : r;
#pragma unroll
        for (int cb = 0; cb < kCB; ++cb) {
          const int n = n0 + wave * 64 + cb * 32 + i32;
          float v = acc[rb][cb][e];
          if (relu) v = v > 0.f ? v : 0.f;
          if (n < N) Yf[out_row * ldy + n] = v;
        }
      }
    return;
  }
  // the last loop iteration ended with a barrier: both stages are free
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int cb = 0; cb < kCB; ++cb)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int row = 32 * rb + 8 * (e >> 2) + 4 * qh + (e & 3);
        const int col = wave * 64 + cb * 32 + i32;
        float v = acc[rb][cb][e];
        if (relu) v = v > 0.f ? v : 0.f;
        *reinterpret_cast<uint16_t*>(lds + row * kYStride + col * 2) = float_to_bits<DT>(v);
      }
  __syncthreads();
  uint16_t* Yh = static_cast<uint16_t*>(Y);
  // 32 lanes move one 512-byte row; a wave moves two rows per pass
  for (int row = (tid >> 5); row < V; row += kThreads / 32) {
    const int r = t * V + row;
    const int64_t out_row = pi_out ? pi_out[r] : r;
    const int n = n0 + b_chunk * 8;
    const u32x4 v = *reinterpret_cast<const u32x4*>(lds + row * kYStride + b_chunk * 16);
    uint16_t* dst = Yh + out_row * ldy + n;
    if (n + 8 <= N) {
      *reinterpret_cast<u32x4*>(dst) = v;
    } else if (n < N) {
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
      for (int e = 0; e < N - n; ++e) dst[e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
    }
  }
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
  auto kernel = spmm_tile_kernel<DT, RB, KSUB>;
  static bool attr_set = false;  // raising the dynamic-LDS limit is idempotent; a race only repeats it
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  kernel<<<dim3((unsigned)(work_per_xcd * 8)), kThreads, lds_bytes, stream>>>(
      static_cast<const uint16_t*>(a.vals), a.nm_idx, a.vec_idx, a.pi_in, a.pi_out,
      static_cast<const uint16_t*>(a.X), a.ldx, a.Y, a.ldy, T, a.s.Kv, a.N, n_blocks, work_per_xcd, a.relu,
      a.out_f32);
  return hipGetLastError();
}

template <int DT>
hipError_t launch_dt(const SpmmArgs& a, hipStream_t stream) {
  switch (a.s.V) {
    case 32: return launch_one<DT, 1, 2>(a, stream);
    case 64: return launch_one<DT, 2, 2>(a, stream);
    case 96: return launch_one<DT, 3, 2>(a, stream);
    case 128: return launch_one<DT, 4, 2>(a, stream);
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
