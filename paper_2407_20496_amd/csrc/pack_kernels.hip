// HiNM compression on the GPU (arXiv 2407.20496, Section 1 / Figure 1 walk-through and
// Section 3.1): column-vector pruning per tile of V rows, then 2:4 on the surviving columns.
//
// Three passes over device memory:
//   score  : s[t][k] = sum_i W[tV+i][k]^2 in binary64, rows added in ascending order
//   select : per tile, the Kv largest scores (equal scores: lower column first), written as the
//            ascending vector index
//   emit   : per row and group of four surviving columns, the two largest magnitudes (equal:
//            lower position first) -> packed values + NM nibble
// plus the inverse (unpack) used by the round-trip checks.
//
// Variants of the same passes: per-weight saliency scores rho given by the caller (Section 4.1, the
// rho of Eq. 1-3) replace the squares in `score` and the magnitudes in `emit`; a caller-given
// tile-wise order of the kept columns (Section 3.2) adds an `order` pass after `select`; and the
// vector-only state of gradual pruning (Section 5.1.2) replaces `emit` by a plain gather of the
// surviving columns.
#include "hinm_internal.h"

namespace hinm {
namespace {

typedef uint32_t quad_t __attribute__((ext_vector_type(4)));  // 16 bytes for non-temporal stores

constexpr int kScoreThreads = 256;
constexpr int kSelectThreads = 1024;
constexpr int kEmitThreads = 256;

// ---------------------------------------------------------------------------------------------
// score: one thread owns VEC adjacent columns of one tile and walks down the V rows.
// The products are exact in binary64 (both factors carry at most 11 significand bits), so the
// fused multiply-add rounds exactly like a separate add would; only the add order matters and
// it is fixed to ascending rows.
// ---------------------------------------------------------------------------------------------
template <int DT, int VEC>
__global__ __launch_bounds__(kScoreThreads) void score_kernel(const uint16_t* __restrict__ W,
                                                              double* __restrict__ scores, int K, int V) {
  const int t = blockIdx.y;
  const int64_t c0 = ((int64_t)blockIdx.x * kScoreThreads + threadIdx.x) * VEC;
  if (c0 >= K) return;
  const uint16_t* p = W + (size_t)t * V * K + c0;
  double s[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) s[e] = 0.0;
  for (int i = 0; i < V; ++i) {
    uint16_t w[VEC];
    if constexpr (VEC == 8) {
      const quad_t q = __builtin_nontemporal_load(reinterpret_cast<const quad_t*>(p));  // streamed once here (C5: 110 -> 91 us)
      w[0] = q.x & 0xFFFF; w[1] = q.x >> 16; w[2] = q.y & 0xFFFF; w[3] = q.y >> 16;
      w[4] = q.z & 0xFFFF; w[5] = q.z >> 16; w[6] = q.w & 0xFFFF; w[7] = q.w >> 16;
    } else {
#pragma unroll
      for (int e = 0; e < VEC; ++e) w[e] = p[e];
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      const double a = (double)bits_to_float<DT>(w[e]);
      s[e] = __builtin_fma(a, a, s[e]);
    }
    p += K;
  }
  double* out = scores + (size_t)t * K + c0;
#pragma unroll
  for (int e = 0; e < VEC; ++e) out[e] = s[e];
}

// The same walk over caller-given scores: s[t][k] = sum_i rho[tV+i][k], binary64, ascending rows,
// starting from +0 (so a sum is never -0).
template <int VEC>
__global__ __launch_bounds__(kScoreThreads) void score_rho_kernel(const float* __restrict__ rho,
                                                                  double* __restrict__ scores, int K, int V) {
  const int t = blockIdx.y;
  const int64_t c0 = ((int64_t)blockIdx.x * kScoreThreads + threadIdx.x) * VEC;
  if (c0 >= K) return;
  const float* p = rho + (size_t)t * V * K + c0;
  double s[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) s[e] = 0.0;
  for (int i = 0; i < V; ++i) {
    float w[VEC];
    if constexpr (VEC == 4) {
      typedef float fquad_t __attribute__((ext_vector_type(4)));
      const fquad_t q = __builtin_nontemporal_load(reinterpret_cast<const fquad_t*>(p));  // streamed: nothing else wants these lines before the emit pass
      w[0] = q.x; w[1] = q.y; w[2] = q.z; w[3] = q.w;
    } else {
#pragma unroll
      for (int e = 0; e < VEC; ++e) w[e] = p[e];
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) s[e] += (double)w[e];
    p += K;
  }
  double* out = scores + (size_t)t * K + c0;
#pragma unroll
  for (int e = 0; e < VEC; ++e) out[e] = s[e];
}

// ---------------------------------------------------------------------------------------------
// select: one workgroup per tile.  A score's bit pattern is turned into a key that orders like an
// unsigned 64-bit integer (sign bit set for non-negative values, all bits flipped for negative ones;
// sums start from +0, so -0 does not occur and equal values have equal keys; NaN is not supported).
// An 8-bit-digit radix descent finds the Kv-th largest key tau and
// how many keys equal to tau still have to be taken; those are taken from the lowest columns.
// A final in-order sweep with workgroup prefix sums writes the kept columns ascending.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ unsigned long long ordered_key(unsigned long long bits) {
  return (bits >> 63) ? ~bits : (bits | (1ull << 63));
}

__device__ __forceinline__ uint32_t block_exclusive_count(bool flag, uint32_t* wave_tot, uint32_t& total) {
  const unsigned long long bal = __ballot(flag);
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const uint32_t in_wave = __popcll(bal & ((1ull << lane) - 1ull));
  __syncthreads();  // previous use of wave_tot is over
  if (lane == 0) wave_tot[wave] = __popcll(bal);
  __syncthreads();
  uint32_t before = 0, all = 0;
  for (int w = 0; w < kSelectThreads / 64; ++w) {
    const uint32_t c = wave_tot[w];
    if (w < wave) before += c;
    all += c;
  }
  total = all;
  return before + in_wave;
}

// KPT = keys per thread held in registers for the whole kernel (K <= KPT * 1024), or 0 = re-read
// the keys from memory in every pass (any K).
template <int KPT>
__global__ __launch_bounds__(kSelectThreads) void select_kernel(const double* __restrict__ scores,
                                                                int32_t* __restrict__ vec_idx, int K, int Kv) {
  __shared__ uint32_t hist[256];
  __shared__ uint32_t wave_tot[kSelectThreads / 64];
  __shared__ unsigned long long s_prefix;
  __shared__ uint32_t s_need;
  __shared__ uint32_t s_in_bin;  // keys in the bin the last pass chose
  const int t = blockIdx.x;
  const unsigned long long* key = reinterpret_cast<const unsigned long long*>(scores + (size_t)t * K);
  constexpr int kHeld = KPT > 0 ? KPT : 1;
  unsigned long long held[kHeld];
  if constexpr (KPT > 0) {
#pragma unroll
    for (int c = 0; c < KPT; ++c) {
      const int k = c * kSelectThreads + threadIdx.x;
      held[c] = (k < K) ? ordered_key(key[k]) : 0ull;
    }
  }
  const int chunks = KPT > 0 ? KPT : (K + kSelectThreads - 1) / kSelectThreads;

  unsigned long long prefix = 0, mask = 0;
  uint32_t need = (uint32_t)Kv;  // the need-th largest among keys that match prefix under mask
  for (int shift = 56; shift >= 0; shift -= 8) {
    if (threadIdx.x < 256) hist[threadIdx.x] = 0;
    __syncthreads();
#pragma unroll
    for (int c = 0; c < chunks; ++c) {
      const int k = c * kSelectThreads + threadIdx.x;
      unsigned long long u;
      if constexpr (KPT > 0) u = held[c];
      else u = (k < K) ? ordered_key(key[k]) : 0ull;
      bool pending = (k < K) && ((u & mask) == prefix);
      const uint32_t d = (uint32_t)(u >> shift) & 255u;
      // Scores of one tile share their leading bits, so in the first passes nearly every lane hits the
      // same bin: count the two most common digits of the wave with one atomic each, the rest singly.
#pragma unroll
      for (int round = 0; round < 2; ++round) {
        const unsigned long long todo = __ballot(pending);
        if (todo == 0ull) break;
        const int leader = __ffsll((long long)todo) - 1;
        const uint32_t dl = (uint32_t)__shfl((int)d, leader);
        const unsigned long long same = __ballot(pending && d == dl);
        if ((int)(threadIdx.x & 63) == leader) atomicAdd(&hist[dl], (uint32_t)__popcll(same));
        pending = pending && d != dl;
      }
      if (pending) atomicAdd(&hist[d], 1u);
    }
    __syncthreads();
    // Find the digit that holds the need-th largest key: the first wave scans the 256 bins from the
    // top, four bins per lane (lane 0 owns the highest four).
    if (threadIdx.x < 64) {
      const int lane = threadIdx.x;
      uint32_t h[4];
      uint32_t mine = 0;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        h[q] = hist[255 - (4 * lane + q)];
        mine += h[q];
      }
      uint32_t incl = mine;  // inclusive prefix over lanes = keys in this lane's bins or higher ones
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const uint32_t v = (uint32_t)__shfl_up((int)incl, off);
        if (lane >= off) incl += v;
      }
      uint32_t above = incl - mine;  // keys in strictly higher lanes' bins
      const bool here = (above < need) && (incl >= need);
      const bool nowhere = (__ballot(here) == 0ull);  // fewer keys than asked for: cannot happen for Kv <= K
      if (here || (nowhere && lane == 63)) {
        int pick = 3;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          if (above + h[q] >= need) {
            pick = q;
            break;
          }
          above += h[q];
        }
        s_prefix = prefix | ((unsigned long long)(255 - (4 * lane + pick)) << shift);
        s_need = need - above;
        s_in_bin = h[pick];
      }
    }
    __syncthreads();
    prefix = s_prefix;
    need = s_need;
    mask |= 0xFFull << shift;
    // Every key of the chosen bin is wanted: the lower digits decide nothing any more.  (With distinct scores
    // this happens after three or four of the eight passes.)
    if (s_in_bin == need) break;
  }
  // tau = the Kv-th largest key, or, after an early exit, its leading digits with zeros behind them: in both
  // cases keys above tau survive, and of the keys equal to tau (only possible without an early exit) the
  // take_equal lowest columns do.
  const unsigned long long tau = prefix;
  const uint32_t take_equal = need;
  const bool ties_cut = s_in_bin != need;  // some keys equal to tau are dropped: their order matters

  int32_t* out = vec_idx + (size_t)t * Kv;
  if constexpr (KPT > 0) {
    // Keys in registers: one count per (chunk, wave), one scan of those <= 256 counts by the first wave, and
    // every thread knows where its kept columns go -- two barriers per ranking instead of four per chunk.
    constexpr int kWaves = kSelectThreads / 64;
    __shared__ uint32_t cnt[KPT * kWaves];  // counts in (chunk, wave) order, then their exclusive prefix sums
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const unsigned long long below = (1ull << lane) - 1ull;
    auto scan_counts = [&]() {
      __syncthreads();
      if (threadIdx.x < 64) {
        constexpr int kPer = (KPT * kWaves + 63) / 64;
        uint32_t v[kPer], mine = 0;
#pragma unroll
        for (int q = 0; q < kPer; ++q) {
          const int idx = kPer * lane + q;
          v[q] = idx < KPT * kWaves ? cnt[idx] : 0u;
          mine += v[q];
        }
        uint32_t incl = mine;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
          const uint32_t o = (uint32_t)__shfl_up((int)incl, off);
          if (lane >= off) incl += o;
        }
        uint32_t run = incl - mine;
#pragma unroll
        for (int q = 0; q < kPer; ++q) {
          const int idx = kPer * lane + q;
          if (idx < KPT * kWaves) cnt[idx] = run;
          run += v[q];
        }
      }
      __syncthreads();
    };
    uint32_t keep_bits = 0;  // bit c: this thread's key of chunk c survives
    if (ties_cut) {          // uniform: rank the keys equal to tau by column
#pragma unroll
      for (int c = 0; c < KPT; ++c) {
        const bool eq = (c * kSelectThreads + (int)threadIdx.x < K) && held[c] == tau;
        const unsigned long long bal = __ballot(eq);
        if (lane == 0) cnt[c * kWaves + wave] = (uint32_t)__popcll(bal);
      }
      scan_counts();
#pragma unroll
      for (int c = 0; c < KPT; ++c) {
        const bool in = c * kSelectThreads + (int)threadIdx.x < K;
        const bool eq = in && held[c] == tau;
        const unsigned long long bal = __ballot(eq);
        const uint32_t rank = cnt[c * kWaves + wave] + (uint32_t)__popcll(bal & below);
        if (in && (held[c] > tau || (eq && rank < take_equal))) keep_bits |= 1u << c;
      }
      __syncthreads();  // cnt is rewritten below
    } else {
#pragma unroll
      for (int c = 0; c < KPT; ++c)
        if (c * kSelectThreads + (int)threadIdx.x < K && held[c] >= tau) keep_bits |= 1u << c;
    }
#pragma unroll
    for (int c = 0; c < KPT; ++c) {
      const unsigned long long bal = __ballot((keep_bits >> c) & 1u);
      if (lane == 0) cnt[c * kWaves + wave] = (uint32_t)__popcll(bal);
    }
    scan_counts();
#pragma unroll
    for (int c = 0; c < KPT; ++c) {
      const bool keep = (keep_bits >> c) & 1u;
      const unsigned long long bal = __ballot(keep);
      const uint32_t pos = cnt[c * kWaves + wave] + (uint32_t)__popcll(bal & below);
      if (keep && pos < (uint32_t)Kv) out[pos] = c * kSelectThreads + (int)threadIdx.x;
    }
  } else {
    uint32_t eq_base = 0, kept_base = 0;
    for (int c = 0; c < chunks; ++c) {
      const int k = c * kSelectThreads + threadIdx.x;
      const bool in = k < K;
      const unsigned long long u = in ? ordered_key(key[k]) : 0ull;
      const bool gt = in && u > tau;
      const bool eq = in && u == tau;
      uint32_t eq_total, kept_total;
      const uint32_t eq_rank = eq_base + block_exclusive_count(eq, wave_tot, eq_total);
      const bool keep = gt || (eq && (!ties_cut || eq_rank < take_equal));
      const uint32_t pos = kept_base + block_exclusive_count(keep, wave_tot, kept_total);
      if (keep && pos < (uint32_t)Kv) out[pos] = k;
      eq_base += eq_total;
      kept_base += kept_total;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// emit: one thread per (row, NM byte) = two groups of four surviving columns.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void top2_of_4(const uint16_t w[4], uint32_t& p0, uint32_t& p1) {
  uint32_t m[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) m[q] = w[q] & 0x7FFFu;
  uint32_t kept_mask = 0;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    uint32_t rank = 0;
#pragma unroll
    for (int o = 0; o < 4; ++o) {
      if (o == q) continue;
      rank += (m[o] > m[q] || (m[o] == m[q] && o < q)) ? 1u : 0u;
    }
    if (rank < 2) kept_mask |= 1u << q;
  }
  p0 = __builtin_ctz(kept_mask);
  p1 = 31 - __builtin_clz(kept_mask);
}

// The same choice on caller-given scores, compared as signed numbers (-0 equals +0).
__device__ __forceinline__ void top2_of_4_scores(const float sc[4], uint32_t& p0, uint32_t& p1) {
  uint32_t kept_mask = 0;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    uint32_t rank = 0;
#pragma unroll
    for (int o = 0; o < 4; ++o) {
      if (o == q) continue;
      rank += (sc[o] > sc[q] || (sc[o] == sc[q] && o < q)) ? 1u : 0u;
    }
    if (rank < 2) kept_mask |= 1u << q;
  }
  p0 = __builtin_ctz(kept_mask);
  p1 = 31 - __builtin_clz(kept_mask);
}

// One NM byte = two groups of four surviving columns of one row: picks the eight entries through
// `w_at` (and their scores through `rho_at` when SCORED), stores four values and the byte.
template <bool SCORED, typename WAt, typename RhoAt>
__device__ __forceinline__ void emit_byte(const int32_t* __restrict__ vi, WAt w_at, RhoAt rho_at,
                                          uint16_t* __restrict__ vals_out, uint8_t* __restrict__ nm_out) {
  uint16_t out[4];
  uint32_t byte = 0;
#pragma unroll
  for (int g = 0; g < 2; ++g) {
    uint16_t w[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) w[q] = w_at(vi[4 * g + q]);
    uint32_t p0, p1;
    if constexpr (SCORED) {
      float sc[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) sc[q] = rho_at(vi[4 * g + q]);
      top2_of_4_scores(sc, p0, p1);
    } else {
      top2_of_4(w, p0, p1);
    }
    out[2 * g] = w[p0];
    out[2 * g + 1] = w[p1];
    byte |= (p0 | (p1 << 2)) << (4 * g);
  }
  uint2 packed;
  packed.x = (uint32_t)out[0] | ((uint32_t)out[1] << 16);
  packed.y = (uint32_t)out[2] | ((uint32_t)out[3] << 16);
  // written once and read by a later kernel: kept from displacing the rows of W in the caches
  typedef uint32_t pair_t __attribute__((ext_vector_type(2)));
  __builtin_nontemporal_store(pair_t{packed.x, packed.y}, reinterpret_cast<pair_t*>(vals_out));
  __builtin_nontemporal_store((uint8_t)byte, nm_out);
}

template <bool SCORED>
__global__ __launch_bounds__(kEmitThreads) void emit_kernel(const uint16_t* __restrict__ W,
                                                            const float* __restrict__ rho,
                                                            const int32_t* __restrict__ vec_idx,
                                                            uint16_t* __restrict__ vals, uint8_t* __restrict__ nm_idx,
                                                            int M, int K, int V, int Kv) {
  const int bytes_per_row = Kv / 8;
  const int64_t id = (int64_t)blockIdx.x * kEmitThreads + threadIdx.x;
  if (id >= (int64_t)M * bytes_per_row) return;
  const int r = (int)(id / bytes_per_row);
  const int b = (int)(id % bytes_per_row);
  const int t = r / V;
  const uint16_t* wr = W + (size_t)r * K;
  const float* rr = SCORED ? rho + (size_t)r * K : nullptr;
  emit_byte<SCORED>(
      vec_idx + (size_t)t * Kv + 8 * b, [&](int c) { return wr[c]; }, [&](int c) { return rr[c]; },
      vals + (size_t)r * (Kv / 2) + 4 * b, nm_idx + (size_t)r * bytes_per_row + b);
}

// Vector pruning alone: vals_v[r][j] = W[r][vec_idx[t][j]], eight outputs per thread.
__global__ __launch_bounds__(kEmitThreads) void gather_kernel(const uint16_t* __restrict__ W,
                                                              const int32_t* __restrict__ vec_idx,
                                                              uint16_t* __restrict__ vals_v, int M, int K, int V,
                                                              int Kv) {
  const int pieces_per_row = Kv / 8;
  const int64_t id = (int64_t)blockIdx.x * kEmitThreads + threadIdx.x;
  if (id >= (int64_t)M * pieces_per_row) return;
  const int r = (int)(id / pieces_per_row);
  const int b = (int)(id % pieces_per_row);
  const int32_t* vi = vec_idx + (size_t)(r / V) * Kv + 8 * b;
  const uint16_t* wr = W + (size_t)r * K;
  uint32_t o[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) o[q] = (uint32_t)wr[vi[2 * q]] | ((uint32_t)wr[vi[2 * q + 1]] << 16);
  __builtin_nontemporal_store(quad_t{o[0], o[1], o[2], o[3]}, reinterpret_cast<quad_t*>(vals_v + (size_t)r * Kv + 8 * b));
}

// ---------------------------------------------------------------------------------------------
// unpack: zero fill, then scatter the two survivors of every group.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void zero_kernel(uint16_t* __restrict__ p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0;
}

__global__ __launch_bounds__(256) void scatter_kernel(const uint16_t* __restrict__ vals,
                                                      const uint8_t* __restrict__ nm_idx,
                                                      const int32_t* __restrict__ vec_idx,
                                                      uint16_t* __restrict__ W, int M, int K, int V, int Kv) {
  const int groups = Kv / 4;
  const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (id >= (int64_t)M * groups) return;
  const int r = (int)(id / groups);
  const int g = (int)(id % groups);
  const int t = r / V;
  const uint32_t nib = (nm_idx[(size_t)r * (Kv / 8) + (g >> 1)] >> (4 * (g & 1))) & 0xFu;
  const int32_t* vi = vec_idx + (size_t)t * Kv + 4 * g;
  uint16_t* wr = W + (size_t)r * K;
  wr[vi[nib & 3u]] = vals[(size_t)r * (Kv / 2) + 2 * g];
  wr[vi[(nib >> 2) & 3u]] = vals[(size_t)r * (Kv / 2) + 2 * g + 1];
}

// The same emission with the row of W (and of rho) staged in LDS: one workgroup per row reads the
// row once, fully coalesced, and picks the kept columns from LDS.  The picks of emit_kernel go to
// global memory, which costs one address-unit cycle per lane and is slow as soon as the vector
// index is not ascending (a caller-given tile order).  Needs 2 K bytes of LDS, 6 K with scores.
constexpr int kEmitRowMaxK = 32 * 1024;
constexpr int kEmitRowScoredMaxK = 16 * 1024;

template <int THREADS>
__device__ __forceinline__ void stage_row(uint16_t* row, const uint16_t* __restrict__ wr, int K, bool vec8) {
  if (vec8) {  // K % 8 == 0 and the source 16-byte aligned
    for (int i = threadIdx.x; i < K / 8; i += THREADS)
      reinterpret_cast<uint4*>(row)[i] = reinterpret_cast<const uint4*>(wr)[i];
  } else {
    for (int i = threadIdx.x; i < K; i += THREADS) row[i] = wr[i];
  }
}

// 512 threads per row measured best without scores (C5: 300 -> 278 us for the whole pack against 256
// threads, 283 us with 1024).  With scores a row needs three times the LDS, so fewer workgroups fit a
// compute unit: they are made of 1024 threads then, to keep the unit's memory pipeline full.
template <bool SCORED>
constexpr int kEmitRowThreads = SCORED ? 1024 : 512;

template <bool SCORED>
__global__ __launch_bounds__(kEmitRowThreads<SCORED>) void emit_rows_kernel(const uint16_t* __restrict__ W,
                                                                 const float* __restrict__ rho,
                                                                 const int32_t* __restrict__ vec_idx,
                                                                 uint16_t* __restrict__ vals,
                                                                 uint8_t* __restrict__ nm_idx, int K, int V, int Kv,
                                                                 bool vec8, bool rho_vec4) {
  extern __shared__ __attribute__((aligned(16))) uint8_t emit_lds[];
  const int K8 = (K + 7) / 8 * 8;
  float* score_row = reinterpret_cast<float*>(emit_lds);                     // K floats, only when SCORED
  uint16_t* row = reinterpret_cast<uint16_t*>(emit_lds + (SCORED ? (size_t)K8 * 4 : 0));  // K elements
  constexpr int THREADS = kEmitRowThreads<SCORED>;
  // Rows are taken last to first: the score pass has just read the layer first to last, so its tail
  // is the part that the memory-side cache still holds.
  const int r = (int)gridDim.x - 1 - (int)blockIdx.x;
  const int t = r / V;
  stage_row<THREADS>(row, W + (size_t)r * K, K, vec8);
  if constexpr (SCORED) {
    const float* rr = rho + (size_t)r * K;
    if (rho_vec4) {  // K % 4 == 0 and rho 16-byte aligned
      for (int i = threadIdx.x; i < K / 4; i += THREADS)
        reinterpret_cast<float4*>(score_row)[i] = reinterpret_cast<const float4*>(rr)[i];
    } else {
      for (int i = threadIdx.x; i < K; i += THREADS) score_row[i] = rr[i];
    }
  }
  __syncthreads();
  const int bytes_per_row = Kv / 8;
  for (int b = threadIdx.x; b < bytes_per_row; b += THREADS)
    emit_byte<SCORED>(
        vec_idx + (size_t)t * Kv + 8 * b, [&](int c) { return row[c]; }, [&](int c) { return score_row[c]; },
        vals + (size_t)r * (Kv / 2) + 4 * b, nm_idx + (size_t)r * bytes_per_row + b);
}

__global__ __launch_bounds__(kEmitRowThreads<false>) void gather_rows_kernel(const uint16_t* __restrict__ W,
                                                                   const int32_t* __restrict__ vec_idx,
                                                                   uint16_t* __restrict__ vals_v, int K, int V, int Kv,
                                                                   bool vec8) {
  extern __shared__ __attribute__((aligned(16))) uint8_t emit_lds[];
  uint16_t* row = reinterpret_cast<uint16_t*>(emit_lds);
  const int r = (int)gridDim.x - 1 - (int)blockIdx.x;  // last to first, as in emit_rows_kernel
  stage_row<kEmitRowThreads<false>>(row, W + (size_t)r * K, K, vec8);
  __syncthreads();
  const int32_t* vt = vec_idx + (size_t)(r / V) * Kv;
  for (int b = threadIdx.x; b < Kv / 8; b += kEmitRowThreads<false>) {
    const int32_t* vi = vt + 8 * b;
    uint32_t o[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) o[q] = (uint32_t)row[vi[2 * q]] | ((uint32_t)row[vi[2 * q + 1]] << 16);
    __builtin_nontemporal_store(quad_t{o[0], o[1], o[2], o[3]}, reinterpret_cast<quad_t*>(vals_v + (size_t)r * Kv + 8 * b));
  }
}

// Tile-wise input-channel order (Section 3.2, "tile-wise input channel permutation"): the kept
// columns of tile t, so far ascending, are rewritten in the order in which they appear in
// sigma[t][0..K), a permutation of the input channels.  One workgroup per tile, in place: a bitmap of
// the kept columns is built in LDS first, then sigma is swept in order with workgroup prefix sums.
// Entries of sigma outside [0, K) are skipped and nothing is written past slot Kv - 1, so a sigma that
// is not a permutation leaves an unspecified but in-range vector index.
constexpr int kOrderThreads = 1024;

__global__ __launch_bounds__(kOrderThreads) void order_kernel(const int32_t* __restrict__ sigma,
                                                              int32_t* __restrict__ vec_idx, int K, int Kv) {
  extern __shared__ uint32_t kept_bits[];  // ceil(K / 32) words
  __shared__ uint32_t wave_count[kOrderThreads / 64];
  const int t = blockIdx.x;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  int32_t* vi = vec_idx + (size_t)t * Kv;
  const int32_t* sg = sigma + (size_t)t * K;
  for (int w = tid; w < (K + 31) / 32; w += kOrderThreads) kept_bits[w] = 0;
  __syncthreads();
  for (int j = tid; j < Kv; j += kOrderThreads) {
    const int c = vi[j];
    atomicOr(&kept_bits[c >> 5], 1u << (c & 31));
  }
  __syncthreads();
  int done = 0;  // kept columns written so far (same value in every thread)
  for (int base = 0; base < K; base += kOrderThreads) {
    const int i = base + tid;
    const int c = (i < K) ? sg[i] : -1;
    const bool take = c >= 0 && c < K && ((kept_bits[c >> 5] >> (c & 31)) & 1u);
    const uint64_t votes = __ballot(take);
    const int before_in_wave = __popcll(votes & ((1ull << lane) - 1));
    if (lane == 0) wave_count[wave] = (uint32_t)__popcll(votes);
    __syncthreads();
    int before_waves = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kOrderThreads / 64; ++w) {
      const int n = (int)wave_count[w];
      if (w < wave) before_waves += n;
      total += n;
    }
    const int pos = done + before_waves + before_in_wave;
    if (take && pos < Kv) vi[pos] = c;
    done += total;
    __syncthreads();  // wave_count is rewritten by the next sweep
  }
}

// The inverse bookkeeping (Section 3.2: any arrangement of a tile's kept vectors is a valid layer): from an
// arrangement vec_idx[t][0..Kv) to a full order of the K input channels that reproduces it when given to
// order_kernel: the kept channels in their arrangement, then the pruned ones ascending.  One workgroup per
// tile: bitmap of the kept channels in LDS, then one ordered sweep over the channels with workgroup prefix sums.
// Entries of vec_idx outside [0, K) are copied but mark nothing; nothing is written past slot K - 1.
__global__ __launch_bounds__(kOrderThreads) void tile_order_kernel(const int32_t* __restrict__ vec_idx,
                                                                   int32_t* __restrict__ sigma, int K, int Kv) {
  extern __shared__ uint32_t kept_bits[];  // ceil(K / 32) words
  __shared__ uint32_t wave_count[kOrderThreads / 64];
  const int t = blockIdx.x;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int32_t* vi = vec_idx + (size_t)t * Kv;
  int32_t* sg = sigma + (size_t)t * K;
  for (int w = tid; w < (K + 31) / 32; w += kOrderThreads) kept_bits[w] = 0;
  __syncthreads();
  for (int j = tid; j < Kv; j += kOrderThreads) {
    const int c = vi[j];
    sg[j] = c;
    if (c >= 0 && c < K) atomicOr(&kept_bits[c >> 5], 1u << (c & 31));
  }
  __syncthreads();
  int done = Kv;  // slots written so far (same value in every thread)
  for (int base = 0; base < K; base += kOrderThreads) {
    const int c = base + tid;
    const bool take = c < K && !((kept_bits[c >> 5] >> (c & 31)) & 1u);
    const uint64_t votes = __ballot(take);
    const int before_in_wave = __popcll(votes & ((1ull << lane) - 1));
    if (lane == 0) wave_count[wave] = (uint32_t)__popcll(votes);
    __syncthreads();
    int before_waves = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kOrderThreads / 64; ++w) {
      const int n = (int)wave_count[w];
      if (w < wave) before_waves += n;
      total += n;
    }
    const int pos = done + before_waves + before_in_wave;
    if (take && pos < K) sg[pos] = c;
    done += total;
    __syncthreads();  // wave_count is rewritten by the next sweep
  }
}

// dst row r = src row row_order[r]; rows of row_bytes bytes (a multiple of 4), one workgroup per row.  Rows named
// outside [0, rows) are left unwritten.
__global__ __launch_bounds__(256) void gather_rows_by_order_kernel(const uint32_t* __restrict__ src, uint32_t* __restrict__ dst,
                                                                   const int32_t* __restrict__ row_order, int rows,
                                                                   size_t row_words) {
  const int r = blockIdx.x;
  const int from = row_order[r];
  if (from < 0 || from >= rows) return;
  const uint32_t* in = src + (size_t)from * row_words;
  uint32_t* out = dst + (size_t)r * row_words;
  for (size_t i = threadIdx.x; i < row_words; i += 256) out[i] = in[i];
}

}  // namespace

hipError_t launch_gather_rows(const void* src, void* dst, const int32_t* row_order, int rows, size_t row_bytes,
                              hipStream_t stream) {
  gather_rows_by_order_kernel<<<rows, 256, 0, stream>>>(static_cast<const uint32_t*>(src), static_cast<uint32_t*>(dst),
                                                         row_order, rows, row_bytes / 4);
  return hipGetLastError();
}

hipError_t launch_tile_order(const hinm_shape& s, const int32_t* vec_idx, int32_t* tile_order, hipStream_t stream) {
  tile_order_kernel<<<s.M / s.V, kOrderThreads, (size_t)((s.K + 31) / 32) * 4, stream>>>(vec_idx, tile_order, s.K, s.Kv);
  return hipGetLastError();
}

hipError_t launch_pack(const PackArgs& a, hipStream_t stream) {
  const hinm_shape& s = a.s;
  const int T = s.M / s.V;
  const uint16_t* Wb = static_cast<const uint16_t*>(a.W);
  uint16_t* vals = static_cast<uint16_t*>(a.vals);
  const bool vec8 = (s.K % 8 == 0) && ((reinterpret_cast<uintptr_t>(a.W) & 15u) == 0);
  const bool rho_vec4 = a.rho && (s.K % 4 == 0) && ((reinterpret_cast<uintptr_t>(a.rho) & 15u) == 0);
  // ---- score
  const int cols_per_thread = a.rho ? (rho_vec4 ? 4 : 1) : (vec8 ? 8 : 1);
  const int threads_needed = (s.K + cols_per_thread - 1) / cols_per_thread;
  dim3 grid((threads_needed + kScoreThreads - 1) / kScoreThreads, T);
  if (a.rho) {
    if (rho_vec4) score_rho_kernel<4><<<grid, kScoreThreads, 0, stream>>>(a.rho, a.scores, s.K, s.V);
    else score_rho_kernel<1><<<grid, kScoreThreads, 0, stream>>>(a.rho, a.scores, s.K, s.V);
  } else if (s.dtype == HINM_F16) {
    if (vec8) score_kernel<HINM_F16, 8><<<grid, kScoreThreads, 0, stream>>>(Wb, a.scores, s.K, s.V);
    else score_kernel<HINM_F16, 1><<<grid, kScoreThreads, 0, stream>>>(Wb, a.scores, s.K, s.V);
  } else {
    if (vec8) score_kernel<HINM_BF16, 8><<<grid, kScoreThreads, 0, stream>>>(Wb, a.scores, s.K, s.V);
    else score_kernel<HINM_BF16, 1><<<grid, kScoreThreads, 0, stream>>>(Wb, a.scores, s.K, s.V);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  // ---- select
  if (s.K <= 4 * kSelectThreads) select_kernel<4><<<T, kSelectThreads, 0, stream>>>(a.scores, a.vec_idx, s.K, s.Kv);
  else if (s.K <= 16 * kSelectThreads) select_kernel<16><<<T, kSelectThreads, 0, stream>>>(a.scores, a.vec_idx, s.K, s.Kv);
  else select_kernel<0><<<T, kSelectThreads, 0, stream>>>(a.scores, a.vec_idx, s.K, s.Kv);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  // ---- order
  if (a.tile_order) {
    order_kernel<<<T, kOrderThreads, (size_t)((s.K + 31) / 32) * 4, stream>>>(a.tile_order, a.vec_idx, s.K, s.Kv);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  // ---- emit (or gather): rows long enough to fill a workgroup go through LDS, short rows keep the
  // flat kernels
  const size_t row_bytes = (size_t)((s.K + 7) / 8 * 8) * 2;
  const bool long_rows = s.Kv >= 8 * kEmitThreads;
  const int64_t flat_threads = (int64_t)s.M * (s.Kv / 8);
  const unsigned flat_blocks = (unsigned)((flat_threads + kEmitThreads - 1) / kEmitThreads);
  if (!a.nm_idx) {
    if (long_rows && s.K <= kEmitRowMaxK)
      gather_rows_kernel<<<(unsigned)s.M, kEmitRowThreads<false>, row_bytes, stream>>>(Wb, a.vec_idx, vals, s.K, s.V, s.Kv, vec8);
    else
      gather_kernel<<<flat_blocks, kEmitThreads, 0, stream>>>(Wb, a.vec_idx, vals, s.M, s.K, s.V, s.Kv);
  } else if (a.rho) {
    if (long_rows && s.K <= kEmitRowScoredMaxK) {
      const size_t lds_bytes = 3 * row_bytes;
      // a row of W and its float32 saliencies: up to 96 KB, beyond a workgroup's default 64 KB
      e = raise_lds_limit<emit_rows_kernel<true>>(3 * kEmitRowScoredMaxK * 2);
      if (e != hipSuccess) return e;
      emit_rows_kernel<true><<<(unsigned)s.M, kEmitRowThreads<true>, lds_bytes, stream>>>(Wb, a.rho, a.vec_idx, vals, a.nm_idx,
                                                                                 s.K, s.V, s.Kv, vec8, rho_vec4);
    } else {
      emit_kernel<true><<<flat_blocks, kEmitThreads, 0, stream>>>(Wb, a.rho, a.vec_idx, vals, a.nm_idx, s.M, s.K, s.V,
                                                                  s.Kv);
    }
  } else {
    if (long_rows && s.K <= kEmitRowMaxK)
      emit_rows_kernel<false><<<(unsigned)s.M, kEmitRowThreads<false>, row_bytes, stream>>>(Wb, nullptr, a.vec_idx, vals,
                                                                                  a.nm_idx, s.K, s.V, s.Kv, vec8, false);
    else
      emit_kernel<false><<<flat_blocks, kEmitThreads, 0, stream>>>(Wb, nullptr, a.vec_idx, vals, a.nm_idx, s.M, s.K,
                                                                   s.V, s.Kv);
  }
  return hipGetLastError();
}

hipError_t launch_unpack(const hinm_shape& s, const void* vals, const uint8_t* nm_idx, const int32_t* vec_idx,
                         void* W_out, hipStream_t stream) {
  const int64_t n = (int64_t)s.M * s.K;
  zero_kernel<<<(unsigned)((n + 255) / 256), 256, 0, stream>>>(static_cast<uint16_t*>(W_out), n);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int64_t groups = (int64_t)s.M * (s.Kv / 4);
  scatter_kernel<<<(unsigned)((groups + 255) / 256), 256, 0, stream>>>(
      static_cast<const uint16_t*>(vals), nm_idx, vec_idx, static_cast<uint16_t*>(W_out), s.M, s.K, s.V, s.Kv);
  return hipGetLastError();
}

}  // namespace hinm
