// Measurement aids (hinm_calib.h): plain kernels of known work.  None is part of the HiNM path.
#include "hinm_calib.h"
#include "hinm_internal.h"
#include "mfma_types.h"
#include "direct_lds.h"

namespace hinm {
namespace {

constexpr int kCalibThreads = 256;
constexpr int kCalibGrid = 2048;  // eight workgroups per compute unit

template <bool NT>
__global__ __launch_bounds__(kCalibThreads) void calib_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst,
                                                                   size_t n16) {
  const size_t stride = (size_t)gridDim.x * kCalibThreads;
  size_t i = (size_t)blockIdx.x * kCalibThreads + threadIdx.x;
  // four independent loads in flight per lane before the first store
  for (; i + 3 * stride < n16; i += 4 * stride) {
    u32x4 v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] = NT ? __builtin_nontemporal_load(src + i + k * stride) : src[i + k * stride];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if constexpr (NT) __builtin_nontemporal_store(v[k], dst + i + k * stride);
      else dst[i + k * stride] = v[k];
    }
  }
  for (; i < n16; i += stride) {
    const u32x4 v = NT ? __builtin_nontemporal_load(src + i) : src[i];
    if constexpr (NT) __builtin_nontemporal_store(v, dst + i);
    else dst[i] = v;
  }
}

template <bool NT>
__global__ __launch_bounds__(kCalibThreads) void calib_fill_kernel(u32x4* __restrict__ dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * kCalibThreads;
  const u32x4 v{0x3c003c00u, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u};
  for (size_t i = (size_t)blockIdx.x * kCalibThreads + threadIdx.x; i < n16; i += stride) {
    if constexpr (NT) __builtin_nontemporal_store(v, dst + i);
    else dst[i] = v;
  }
}

template <bool NT>
__global__ __launch_bounds__(kCalibThreads) void calib_read_kernel(const u32x4* __restrict__ src, size_t n16,
                                                                   uint32_t* __restrict__ sink) {
  const size_t stride = (size_t)gridDim.x * kCalibThreads;
  uint32_t fold = 0;
  size_t i = (size_t)blockIdx.x * kCalibThreads + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    u32x4 v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] = NT ? __builtin_nontemporal_load(src + i + k * stride) : src[i + k * stride];
#pragma unroll
    for (int k = 0; k < 4; ++k) fold ^= v[k].x ^ v[k].y ^ v[k].z ^ v[k].w;
  }
  for (; i < n16; i += stride) {
    const u32x4 v = NT ? __builtin_nontemporal_load(src + i) : src[i];
    fold ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  if (fold == 0x9E3779B9u) *sink = fold;
}

// One lane writes 16 bytes; a piece of PIECE bytes is written by PIECE / 16 neighbouring lanes.
__global__ __launch_bounds__(kCalibThreads) void calib_scatter_rows_kernel(uint16_t* __restrict__ dst, int M, int N,
                                                                           int64_t ld, const int32_t* __restrict__ rows,
                                                                           int lanes_per_piece) {
  const int pieces_per_row = (N * 2) / (lanes_per_piece * 16);
  const int64_t pieces = (int64_t)M * pieces_per_row;
  const int pieces_per_block = kCalibThreads / lanes_per_piece;
  const int sub = threadIdx.x / lanes_per_piece, lane = threadIdx.x % lanes_per_piece;
  const u32x4 v{0x3c003c00u, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u};
  for (int64_t p = (int64_t)blockIdx.x * pieces_per_block + sub; p < pieces; p += (int64_t)gridDim.x * pieces_per_block) {
    // consecutive pieces belong to consecutive rows of one column block, as the tiles of a product do
    const int r = (int)(p % M), c = (int)(p / M);
    const int64_t out_row = rows ? rows[r] : r;
    uint16_t* at = dst + out_row * ld + (int64_t)c * lanes_per_piece * 8 + lane * 8;
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(at));
  }
}

template <int DT>
__global__ __launch_bounds__(kCalibThreads) void calib_smfmac_kernel(int iterations, float* __restrict__ sink) {
  const int lane = threadIdx.x & 63;
  // operands of ordinary magnitude (weights around 0.02, activations around 1): all-zero operands would
  // let the matrix unit run cooler and faster than it does on real data
  const uint32_t w = (DT == HINM_F16) ? 0x25002500u + 0x00010001u * (uint32_t)lane   // ~0.02 in binary16
                                      : 0x3ca03ca0u + 0x00010001u * (uint32_t)lane;  // ~0.02 in bfloat16
  const uint32_t x = (DT == HINM_F16) ? 0x3c003c00u + 0x00030003u * (uint32_t)lane   // ~1
                                      : 0x3f803f80u + 0x00010001u * (uint32_t)lane;
  u32x4 a{w, w ^ 0x80000000u, w + 0x00020000u, w ^ 0x00008000u};
  u32x8 b{x, x ^ 0x80000000u, x + 0x00010000u, x ^ 0x00008000u, x, x ^ 0x80008000u, x + 2u, x ^ 0x80000000u};
  const int idx = 0x94e4;  // four valid nibbles (p0 < p1): 0x4, 0xe, 0x4, 0x9
  f32x16 acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
  for (int i = 0; i < iterations; ++i) {
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[j] = smfmac_32x32x32<DT, 0>(a, b, acc[j], idx);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += acc[j][e];
  sink[(size_t)blockIdx.x * kCalibThreads + threadIdx.x] = s;
}

__global__ void calib_empty_kernel() {}

constexpr int kStreamThreads = 512;
constexpr int kStreamChunk = 8192;       // bytes one wave-round of the workgroup copies (512 lanes x 16 bytes)
constexpr int kStreamLdsBytes = 65536;   // LDS ring the copies land in
__global__ __launch_bounds__(kStreamThreads) void calib_lds_stream_kernel(const uint8_t* __restrict__ region,
                                                                          uint32_t chunks, uint32_t start_stride_chunks,
                                                                          int64_t total) {
  __shared__ __attribute__((aligned(1024))) uint8_t lds[kStreamLdsBytes];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  uint32_t chunk = (uint32_t)(((uint64_t)blockIdx.x * start_stride_chunks) % chunks);
  for (int64_t it = 0; it < total; ++it) {
    const uint8_t* src = region + (size_t)chunk * kStreamChunk + wave * 1024 + lane * 16;
    uint8_t* to = lds + ((it * kStreamChunk) % kStreamLdsBytes) + wave * 1024;
    copy16_to_lds(src, to);
    chunk = (chunk + 1 == chunks) ? 0 : chunk + 1;
    // at most eight copies of this wave in flight: the ring holds eight chunks
    wait_copies_outstanding<7>();
  }
  wait_copies_outstanding<0>();
}

// Gathered rows: the first `waves` waves of every workgroup each copy `copies` row segments of 1 KB into their own
// ring of eight LDS slots, OUT copies in flight per wave; the rows are taken at a fixed stride through [0, rows) from
// a start that depends on workgroup and wave, the segment's column offset on the workgroup (eight different ones).
// This is the request pattern of the tile kernels' gathered input rows without their stages and barriers.
template <int OUT>
__global__ __launch_bounds__(kStreamThreads) void calib_gather_stream_kernel(const uint8_t* __restrict__ region,
                                                                             int64_t pitch, uint32_t rows, int waves,
                                                                             int copies) {
  __shared__ __attribute__((aligned(1024))) uint8_t lds[kStreamLdsBytes];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if (wave >= waves) return;
  uint32_t r = (blockIdx.x * 2654435761u + (uint32_t)wave * 40503u) % rows;
  const uint32_t step = 7919u % rows;
  const uint8_t* col = region + (size_t)((blockIdx.x & 7) * 1024) + lane * 16;
  for (int it = 0; it < copies; ++it) {
    copy16_to_lds(col + (size_t)r * pitch, lds + (wave * 8 + (it & 7)) * 1024);
    r += step;
    if (r >= rows) r -= rows;
    wait_copies_outstanding<OUT - 1>();
  }
  wait_copies_outstanding<0>();
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace
}  // namespace hinm

using namespace hinm;

extern "C" {

hinm_status hinm_calib_copy(const void* src, void* dst, size_t bytes, int32_t nontemporal, void* stream) {
  if (!src || !dst) return HINM_ERR_NULL;
  if (bytes == 0 || bytes % 16 != 0 || !aligned16(src) || !aligned16(dst)) return HINM_ERR_SHAPE;
  auto s = static_cast<hipStream_t>(stream);
  if (nontemporal)
    calib_copy_kernel<true><<<kCalibGrid, kCalibThreads, 0, s>>>(static_cast<const u32x4*>(src), static_cast<u32x4*>(dst), bytes / 16);
  else
    calib_copy_kernel<false><<<kCalibGrid, kCalibThreads, 0, s>>>(static_cast<const u32x4*>(src), static_cast<u32x4*>(dst), bytes / 16);
  return hipGetLastError() == hipSuccess ? HINM_OK : HINM_ERR_DEVICE;
}

hinm_status hinm_calib_fill(void* dst, size_t bytes, int32_t nontemporal, void* stream) {
  if (!dst) return HINM_ERR_NULL;
  if (bytes == 0 || bytes % 16 != 0 || !aligned16(dst)) return HINM_ERR_SHAPE;
  auto s = static_cast<hipStream_t>(stream);
  if (nontemporal) calib_fill_kernel<true><<<kCalibGrid, kCalibThreads, 0, s>>>(static_cast<u32x4*>(dst), bytes / 16);
  else calib_fill_kernel<false><<<kCalibGrid, kCalibThreads, 0, s>>>(static_cast<u32x4*>(dst), bytes / 16);
  return hipGetLastError() == hipSuccess ? HINM_OK : HINM_ERR_DEVICE;
}

hinm_status hinm_calib_read(const void* src, size_t bytes, int32_t nontemporal, uint32_t* sink, void* stream) {
  if (!src || !sink) return HINM_ERR_NULL;
  if (bytes == 0 || bytes % 16 != 0 || !aligned16(src)) return HINM_ERR_SHAPE;
  auto s = static_cast<hipStream_t>(stream);
  if (nontemporal) calib_read_kernel<true><<<kCalibGrid, kCalibThreads, 0, s>>>(static_cast<const u32x4*>(src), bytes / 16, sink);
  else calib_read_kernel<false><<<kCalibGrid, kCalibThreads, 0, s>>>(static_cast<const u32x4*>(src), bytes / 16, sink);
  return hipGetLastError() == hipSuccess ? HINM_OK : HINM_ERR_DEVICE;
}

hinm_status hinm_calib_scatter_rows(void* dst, int32_t M, int32_t N, int64_t ld, const int32_t* rows,
                                    int32_t piece_bytes, void* stream) {
  if (!dst) return HINM_ERR_NULL;
  if (M <= 0 || N <= 0 || ld < N || ld % 8 != 0 || !aligned16(dst)) return HINM_ERR_SHAPE;
  if (piece_bytes != 64 && piece_bytes != 128 && piece_bytes != 256 && piece_bytes != 512 && piece_bytes != 1024)
    return HINM_ERR_SHAPE;
  if (((int64_t)N * 2) % piece_bytes != 0) return HINM_ERR_SHAPE;
  calib_scatter_rows_kernel<<<kCalibGrid, kCalibThreads, 0, static_cast<hipStream_t>(stream)>>>(
      static_cast<uint16_t*>(dst), M, N, ld, rows, piece_bytes / 16);
  return hipGetLastError() == hipSuccess ? HINM_OK : HINM_ERR_DEVICE;
}

hinm_status hinm_calib_smfmac(int32_t dtype, int32_t iterations, float* sink, double* stored_value_flops,
                              void* stream) {
  if (!sink) return HINM_ERR_NULL;
  if (dtype != HINM_F16 && dtype != HINM_BF16) return HINM_ERR_DTYPE;
  if (iterations <= 0) return HINM_ERR_SHAPE;
  if (stored_value_flops)
    *stored_value_flops = (double)kCalibGrid * (kCalibThreads / 64) * (double)iterations * 4.0 * (2.0 * 32 * 16 * 32);
  auto s = static_cast<hipStream_t>(stream);
  if (dtype == HINM_F16) calib_smfmac_kernel<HINM_F16><<<kCalibGrid, kCalibThreads, 0, s>>>(iterations, sink);
  else calib_smfmac_kernel<HINM_BF16><<<kCalibGrid, kCalibThreads, 0, s>>>(iterations, sink);
  return hipGetLastError() == hipSuccess ? HINM_OK : HINM_ERR_DEVICE;
}

hinm_status hinm_calib_empty(void* stream) {
  calib_empty_kernel<<<1, 64, 0, static_cast<hipStream_t>(stream)>>>();
  return hipGetLastError() == hipSuccess ? HINM_OK : HINM_ERR_DEVICE;
}

hinm_status hinm_calib_lds_stream(const void* region, size_t region_bytes, size_t start_stride_bytes,
                                  int64_t chunks_per_workgroup, int32_t workgroups, void* stream) {
  if (!region) return HINM_ERR_NULL;
  if (region_bytes == 0 || region_bytes % kStreamChunk != 0 || region_bytes > ((size_t)1 << 40) || !aligned16(region) ||
      start_stride_bytes % kStreamChunk != 0 || chunks_per_workgroup <= 0 || workgroups <= 0)
    return HINM_ERR_SHAPE;
  calib_lds_stream_kernel<<<(unsigned)workgroups, kStreamThreads, 0, static_cast<hipStream_t>(stream)>>>(
      static_cast<const uint8_t*>(region), (uint32_t)(region_bytes / kStreamChunk),
      (uint32_t)((start_stride_bytes / kStreamChunk) % (region_bytes / kStreamChunk)), chunks_per_workgroup);
  return hipGetLastError() == hipSuccess ? HINM_OK : HINM_ERR_DEVICE;
}

hinm_status hinm_calib_gather_stream(const void* region, size_t region_bytes, int64_t row_pitch_bytes, int32_t rows,
                                     int32_t waves, int32_t outstanding, int32_t copies_per_wave, int32_t workgroups,
                                     void* stream) {
  if (!region) return HINM_ERR_NULL;
  if (rows <= 0 || row_pitch_bytes < 8192 || row_pitch_bytes % 16 != 0 || !aligned16(region) ||
      (size_t)rows * (size_t)row_pitch_bytes > region_bytes || waves < 1 || waves > kStreamThreads / 64 ||
      copies_per_wave <= 0 || workgroups <= 0)
    return HINM_ERR_SHAPE;
  auto s = static_cast<hipStream_t>(stream);
  const uint8_t* x = static_cast<const uint8_t*>(region);
  const unsigned g = (unsigned)workgroups;
  switch (outstanding) {
    case 4: calib_gather_stream_kernel<4><<<g, kStreamThreads, 0, s>>>(x, row_pitch_bytes, (uint32_t)rows, waves, copies_per_wave); break;
    case 8: calib_gather_stream_kernel<8><<<g, kStreamThreads, 0, s>>>(x, row_pitch_bytes, (uint32_t)rows, waves, copies_per_wave); break;
    case 16: calib_gather_stream_kernel<16><<<g, kStreamThreads, 0, s>>>(x, row_pitch_bytes, (uint32_t)rows, waves, copies_per_wave); break;
    default: return HINM_ERR_UNSUPPORTED;
  }
  return hipGetLastError() == hipSuccess ? HINM_OK : HINM_ERR_DEVICE;
}

}  // extern "C"
