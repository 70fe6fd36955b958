// Plain HiNM product, one thread per output element (arXiv 2407.20496, Section 3.2):
//   Y[pi_out[r]][n] = sum over groups g of row r of
//                     vals[r][2g]   * X[pi_in[vec_idx[t][4g+p0]]][n]
//                   + vals[r][2g+1] * X[pi_in[vec_idx[t][4g+p1]]][n]
// fp32 fused multiply-adds in ascending group order.  Reads the canonical packed arrays
// directly; works for every legal shape and serves as the on-GPU cross-check of the fast kernels.
#include "hinm_internal.h"

namespace hinm {
namespace {

template <int DT>
__global__ __launch_bounds__(256) void spmm_reference_kernel(
    const uint16_t* __restrict__ vals, const uint8_t* __restrict__ nm_idx, const int32_t* __restrict__ vec_idx,
    const int32_t* __restrict__ pi_in, const int32_t* __restrict__ pi_out, const uint16_t* __restrict__ X,
    int64_t ldx, void* __restrict__ Y, int64_t ldy, int M, int V, int Kv, int N, bool relu, bool out_f32) {
  const int n = blockIdx.x * 64 + (threadIdx.x & 63);
  const int r = blockIdx.y * 4 + (threadIdx.x >> 6);
  if (n >= N || r >= M) return;
  const int t = r / V;
  const int groups = Kv / 4;
  const uint16_t* vr = vals + (size_t)r * (Kv / 2);
  const uint8_t* nr = nm_idx + (size_t)r * (Kv / 8);
  const int32_t* vi = vec_idx + (size_t)t * Kv;
  float acc = 0.f;
  for (int g = 0; g < groups; ++g) {
    const uint32_t nib = (nr[g >> 1] >> (4 * (g & 1))) & 0xFu;
    int c0 = vi[4 * g + (nib & 3u)];
    int c1 = vi[4 * g + ((nib >> 2) & 3u)];
    if (pi_in) {
      c0 = pi_in[c0];
      c1 = pi_in[c1];
    }
    acc = __builtin_fmaf(bits_to_float<DT>(vr[2 * g]), bits_to_float<DT>(X[(size_t)c0 * ldx + n]), acc);
    acc = __builtin_fmaf(bits_to_float<DT>(vr[2 * g + 1]), bits_to_float<DT>(X[(size_t)c1 * ldx + n]), acc);
  }
  if (relu) acc = acc > 0.f ? acc : 0.f;
  const int64_t row = pi_out ? pi_out[r] : r;
  if (out_f32) static_cast<float*>(Y)[row * ldy + n] = acc;
  else static_cast<uint16_t*>(Y)[row * ldy + n] = float_to_bits<DT>(acc);
}

}  // namespace

hipError_t launch_spmm_reference(const SpmmArgs& a, hipStream_t stream) {
  dim3 grid((a.N + 63) / 64, (a.s.M + 3) / 4);
  if (grid.y > 65535u) return hipErrorInvalidConfiguration;
  auto v = static_cast<const uint16_t*>(a.vals);
  auto x = static_cast<const uint16_t*>(a.X);
  if (a.s.dtype == HINM_F16)
    spmm_reference_kernel<HINM_F16><<<grid, 256, 0, stream>>>(v, a.nm_idx, a.vec_idx, a.pi_in, a.pi_out, x, a.ldx, a.Y,
                                                              a.ldy, a.s.M, a.s.V, a.s.Kv, a.N, a.relu, a.out_f32);
  else
    spmm_reference_kernel<HINM_BF16><<<grid, 256, 0, stream>>>(v, a.nm_idx, a.vec_idx, a.pi_in, a.pi_out, x, a.ldx,
                                                               a.Y, a.ldy, a.s.M, a.s.V, a.s.Kv, a.N, a.relu, a.out_f32);
  return hipGetLastError();
}

}  // namespace hinm
