// hinm_prepare: canonical packed arrays + channel orders -> device-tuned form (see prepared_layout.h).
// A pure re-ordering: arXiv 2407.20496, Section 3.2 has the channel orders settled offline and the
// vector indices rewritten to match; this is that offline step, done on the GPU.
#include "hinm_internal.h"
#include "prepared_layout.h"

namespace hinm {
namespace {

__global__ __launch_bounds__(256) void prepare_blocks_kernel(const uint16_t* __restrict__ vals,
                                                             const uint8_t* __restrict__ nm_idx,
                                                             uint8_t* __restrict__ out, int V, int Kv, int RB, int S,
                                                             int64_t n_blocks) {
  const int64_t id = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);  // block (t, s, rb)
  if (id >= n_blocks) return;
  const int lane = threadIdx.x & 63;
  const int rb = (int)(id % RB);
  const int s = (int)((id / RB) % S);
  const int t = (int)(id / ((int64_t)RB * S));
  const int row = t * V + 32 * rb + (lane & 31);
  const int qa = lane >> 5;
  const int groups = Kv / 4;
  const uint16_t* vr = vals + (size_t)row * (Kv / 2);
  const uint8_t* nr = nm_idx + (size_t)row * (Kv / 8);
  uint8_t* blk = out + id * kPrepBlockBytes;
  uint32_t idx_word = 0;
#pragma unroll
  for (int sub = 0; sub < 2; ++sub) {
    uint32_t w[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int g = 16 * s + 8 * sub + 4 * qa + k;
      uint32_t pair = 0, nib = 0x4;
      if (g < groups) {
        pair = (uint32_t)vr[2 * g] | ((uint32_t)vr[2 * g + 1] << 16);
        nib = (nr[g >> 1] >> (4 * (g & 1))) & 0xFu;
      }
      w[k] = pair;
      idx_word |= nib << (16 * sub + 4 * k);
    }
    uint4 v;
    v.x = w[0]; v.y = w[1]; v.z = w[2]; v.w = w[3];
    *reinterpret_cast<uint4*>(blk + sub * 1024 + lane * 16) = v;
  }
  *reinterpret_cast<uint32_t*>(blk + kPrepIdxOffset + lane * 4) = idx_word;
}

__global__ __launch_bounds__(256) void prepare_tables_kernel(const int32_t* __restrict__ vec_idx,
                                                             const int32_t* __restrict__ pi_in,
                                                             const int32_t* __restrict__ pi_out,
                                                             int32_t* __restrict__ gather, int32_t* __restrict__ out_rows,
                                                             uint32_t* __restrict__ zeros, uint32_t* __restrict__ panel,
                                                             int T, int Kv, int Kp, int M, int K) {
  const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t n_gather = (int64_t)T * Kp;
  if (id < n_gather) {
    const int t = (int)(id / Kp), j = (int)(id % Kp);
    int g = -1;
    if (j < Kv) {
      g = vec_idx[(size_t)t * Kv + j];
      if (pi_in) g = pi_in[g];
    }
    gather[id] = g;
    panel[id] = panel_entry_of_row(g, K);
  }
  if (id < M) out_rows[id] = pi_out ? pi_out[id] : (int32_t)id;
  if (id < kPrepZeroBytes / 4) zeros[id] = 0;
}

}  // namespace

hipError_t launch_prepare(const hinm_shape& s, const void* vals, const uint8_t* nm_idx, const int32_t* vec_idx,
                          const int32_t* pi_in, const int32_t* pi_out, void* prepared, hipStream_t stream) {
  const PreparedLayout L = prepared_layout(s);
  uint8_t* base = static_cast<uint8_t*>(prepared);
  const int64_t n_blocks = (int64_t)L.T * L.S * L.RB;
  prepare_blocks_kernel<<<(unsigned)((n_blocks + 3) / 4), 256, 0, stream>>>(
      static_cast<const uint16_t*>(vals), nm_idx, base + L.a_offset, s.V, s.Kv, L.RB, L.S, n_blocks);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  int64_t n = (int64_t)L.T * L.Kp;
  if (n < s.M) n = s.M;
  if (n < kPrepZeroBytes / 4) n = kPrepZeroBytes / 4;
  prepare_tables_kernel<<<(unsigned)((n + 255) / 256), 256, 0, stream>>>(
      vec_idx, pi_in, pi_out, reinterpret_cast<int32_t*>(base + L.gather_offset),
      reinterpret_cast<int32_t*>(base + L.pi_out_offset), reinterpret_cast<uint32_t*>(base + L.zero_offset),
      reinterpret_cast<uint32_t*>(base + L.panel_offset), L.T, s.Kv, L.Kp, s.M, s.K);
  return hipGetLastError();
}

}  // namespace hinm
