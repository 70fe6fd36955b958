// Internal declarations shared by the translation units of libhinm (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <cstdarg>
#include <cstdio>

#include "hinm.h"

namespace hinm {

// ---- host: dynamic LDS beyond the default 64 KB of a workgroup -----------------------------------

// Raises the dynamic-LDS limit of one kernel to `bytes`, once per device: the attribute belongs to
// the device's copy of the code object, so a process that drives several GPUs needs it on each.
// One flag word per kernel (the template argument is the kernel itself, not its type); setting the
// attribute twice is harmless, so a race between two first calls only repeats it.
template <auto Kernel>
inline hipError_t raise_lds_limit(int bytes) {
  static std::atomic<uint64_t> done{0};  // bit d: set on device d (devices >= 64 set it on every call)
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 64 && ((done.load(std::memory_order_relaxed) >> dev) & 1u)) return hipSuccess;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(Kernel), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess && dev < 64) done.fetch_or(uint64_t{1} << dev, std::memory_order_relaxed);
  return e;
}

// ---- host: dry run of a launcher ------------------------------------------------------------------
// With a plan attached to its arguments a launcher records which kernel it would launch, with which
// template configuration and launch shape, and launches nothing (hinm_spmm_prepared_plan).
struct LaunchPlan {
  char* text;       // caller's buffer, always NUL-terminated
  size_t capacity;
  size_t length = 0;
  int launches = 0;
};
inline void plan_record(LaunchPlan* p, const char* fmt, ...) {
  if (p->launches > 0 && p->length + 2 < p->capacity) {
    p->text[p->length++] = ';';
    p->text[p->length++] = ' ';
    p->text[p->length] = 0;
  }
  ++p->launches;
  if (p->length + 1 >= p->capacity) return;
  va_list ap;
  va_start(ap, fmt);
  const int n = vsnprintf(p->text + p->length, p->capacity - p->length, fmt, ap);
  va_end(ap);
  if (n > 0) p->length = (p->length + (size_t)n < p->capacity) ? p->length + (size_t)n : p->capacity - 1;
}

// ---- 16-bit storage helpers (device) ---------------------------------------------------------

// Exact widening of a stored 16-bit pattern to float.
template <int DT>
__device__ __forceinline__ float bits_to_float(uint16_t b) {
  if constexpr (DT == HINM_F16) {
    return (float)__builtin_bit_cast(_Float16, b);
  } else {
    return __builtin_bit_cast(float, (uint32_t)b << 16);
  }
}

// float -> storage type, round-to-nearest-even.
template <int DT>
__device__ __forceinline__ uint16_t float_to_bits(float f) {
  if constexpr (DT == HINM_F16) {
    return __builtin_bit_cast(uint16_t, (_Float16)f);
  } else {
    return __builtin_bit_cast(uint16_t, (__bf16)f);
  }
}

// ---- launchers implemented in the kernel translation units -------------------------------------
// All return hipSuccess or the launch error; all are asynchronous on `stream`.

struct PackArgs {
  hinm_shape s;
  const void* W;
  const float* rho;           // NULL: the weights' own squares / magnitudes; else float32 [M][K] scores
  const int32_t* tile_order;  // NULL: kept columns ascending; else int32 [T][K], see hinm_pack_ordered
  void* vals;                 // [M][Kv/2] after 2:4, or [M][Kv] when nm_idx is NULL
  uint8_t* nm_idx;            // NULL: column-vector pruning only, no 2:4 step
  int32_t* vec_idx;
  double* scores;             // workspace, [T][K]
};
hipError_t launch_pack(const PackArgs& a, hipStream_t stream);
// dst row r = src row row_order[r] (rows of row_bytes bytes, a multiple of 4)
hipError_t launch_gather_rows(const void* src, void* dst, const int32_t* row_order, int rows, size_t row_bytes,
                              hipStream_t stream);
// vec_idx [T][Kv] (an arrangement of every tile's kept channels) -> tile_order [T][K] that reproduces it
hipError_t launch_tile_order(const hinm_shape& s, const int32_t* vec_idx, int32_t* tile_order, hipStream_t stream);
constexpr int kPackOrderMaxK = 32 * 12 * 1024;  // the bitmap of kept columns must fit 48 KB of LDS
hipError_t launch_unpack(const hinm_shape& s, const void* vals, const uint8_t* nm_idx, const int32_t* vec_idx,
                         void* W_out, hipStream_t stream);

struct SpmmArgs {
  hinm_shape s;
  int32_t N;
  const void* vals;
  const uint8_t* nm_idx;
  const int32_t* vec_idx;
  const int32_t* pi_in;
  const int32_t* pi_out;
  const void* X;
  int64_t ldx;
  void* Y;
  int64_t ldy;
  bool relu;
  bool out_f32;
};

hipError_t launch_spmm_reference(const SpmmArgs& a, hipStream_t stream);
// Sparse-MFMA tile kernel (32x32x32 form): V in {32, 64, 96, 128}, N >= 1, ldx % 8 == 0, ldy % 8 == 0.
bool spmm_tile_supported(const SpmmArgs& a);
hipError_t launch_spmm_tile(const SpmmArgs& a, hipStream_t stream);
// Sparse-MFMA skinny kernel (16x16x64 form, 16-column blocks, k split over the waves of a workgroup):
// V % 16 == 0.
bool spmm_skinny_supported(const SpmmArgs& a);
hipError_t launch_spmm_skinny(const SpmmArgs& a, hipStream_t stream);

// ---- layer with the column-vector mask alone (all Kv surviving entries of a row stored) ---------
struct VectorsArgs {
  hinm_shape s;
  int32_t N;
  const void* vals_v;  // [M][Kv]
  const int32_t* vec_idx;
  const int32_t* pi_in;
  const int32_t* pi_out;
  const void* X;
  int64_t ldx;
  void* Y;
  int64_t ldy;
  bool relu;
  bool out_f32;
  int variant;  // 0 = choose by shape; 1 = register-staged, 2 / 3 = direct-to-LDS with 256 / 512 columns
};
// Dense-MFMA tile kernels: V in {32, 64, 96, 128}, ldx % 8 == 0, ldy % 8 == 0; the direct-to-LDS ones
// also need Kv % 64 == 0.
bool spmm_vectors_mfma_supported(const VectorsArgs& a);
int spmm_vectors_variant(const VectorsArgs& a);
hipError_t launch_spmm_vectors_mfma(const VectorsArgs& a, hipStream_t stream);
hipError_t launch_spmm_vectors_plain(const VectorsArgs& a, hipStream_t stream);

// ---- tile-wise input-channel permutation search ------------------------------------------------------
constexpr int kIcpMaxPartitions = 1024;  // partitions (groups of four kept vectors) per tile: Kv <= 4096
struct IcpWorkspace {  // byte offsets into the caller's workspace, each 256-byte aligned
  size_t gathered, order, sample, min1, min2, cost, assign, total_bytes;
};
IcpWorkspace icp_workspace_layout(const hinm_shape& s);
struct IcpArgs {
  hinm_shape s;
  const void* W;           // used when rho is NULL: saliency = |w|
  const float* rho;        // float32 [M][K] or NULL
  int32_t* vec_idx;        // [T][Kv], re-arranged in place
  const uint8_t* samples;  // [iters][T][Kv/4], member 0..3 of every partition
  int32_t iters;
  double* objective;       // [iters][T] or NULL
  void* workspace;
};
hipError_t launch_icp_search(const IcpArgs& a, hipStream_t stream);
// `problems` independent n x n linear assignment problems (cost row-major, binary64), n <= kIcpMaxPartitions:
// assign[q][i] = the column given to row i at minimal total cost
hipError_t launch_assignment(const double* cost, int32_t* assign, int problems, int n, hipStream_t stream);

// ---- output-channel permutation search ---------------------------------------------------------------
constexpr int kOcpMaxK = 16384;   // columns one workgroup of the cost kernel holds in registers
constexpr int kOcpMaxV = 4096;    // positions of a tile (flags in LDS)
struct OcpWorkspace {
  size_t base, cluster, cost, assign, moved, total_bytes;
};
OcpWorkspace ocp_workspace_layout(const hinm_shape& s, int n_samples);
struct OcpArgs {
  hinm_shape s;
  const void* W;            // used when rho is NULL: saliency = |w|
  const float* rho;         // float32 [M][K] or NULL
  int32_t* row_order;       // [M], row_order[t V + p] = the channel at position p of tile t; updated in place
  const int32_t* samples;   // [iters][T][n] positions 0..V-1
  const int32_t* clusters;  // [iters][T][n] items 0..T n - 1 grouped into clusters, or NULL
  int32_t n_samples;
  int32_t iters;
  double* objective;        // [iters] or NULL
  void* workspace;
};
hipError_t launch_ocp_search(const OcpArgs& a, hipStream_t stream);

// clustering phase of the output-channel search: balanced K-means over the sampled channels
struct KmeansWorkspace {
  size_t features, dist, cost, assign, total_bytes;
};
KmeansWorkspace kmeans_workspace_layout(const hinm_shape& s, int n_samples);
struct KmeansArgs {
  hinm_shape s;
  const void* W;
  const float* rho;
  const int32_t* row_order;  // [M]
  const int32_t* samples;    // [T][n] positions of one iteration
  int32_t n_samples;
  int32_t rounds;            // >= 1
  double* centroids;         // [T][K], in/out
  bool init_centroids;       // start from the first sample of every tile instead of the given centroids
  int32_t* clusters;         // out [T][n]
  double* objective;         // [rounds] or NULL
  void* workspace;
};
hipError_t launch_ocp_cluster(const KmeansArgs& a, hipStream_t stream);

// ---- device-tuned ("prepared") layer form -------------------------------------------------------------
hipError_t launch_prepare(const hinm_shape& s, const void* vals, const uint8_t* nm_idx, const int32_t* vec_idx,
                          const int32_t* pi_in, const int32_t* pi_out, void* prepared, hipStream_t stream);

struct PreparedArgs {
  hinm_shape s;
  int32_t N;
  const void* prepared;
  const void* X;
  int64_t ldx;
  void* Y;
  int64_t ldy;
  bool relu;
  bool out_f32;
  int tile_variant;  // 0 = choose by shape; 1.. = a fixed (column block, stage size, depth) choice
  void* workspace;
  size_t workspace_bytes;
  LaunchPlan* plan = nullptr;  // non-NULL: record the launches instead of making them
};

hipError_t launch_spmm_tile_prepared(const PreparedArgs& a, hipStream_t stream);
// measurement aid: part 1 = only the copy stream of the tile kernel chosen for the shape, part 2 = only its LDS
// reads and MFMAs; stores nothing; hipErrorNotSupported for shapes outside the named workloads' configurations
hipError_t launch_spmm_tile_prepared_part(const PreparedArgs& a, int part, hipStream_t stream);
// few input channels (a 64-column panel of X with all K rows fits in LDS): many tiles per workgroup
bool spmm_panel_prepared_supported(const PreparedArgs& a);
bool spmm_panel_prepared_preferred(const PreparedArgs& a);  // supported and faster than the tile kernel
hipError_t launch_spmm_panel_prepared(const PreparedArgs& a, hipStream_t stream);
// few columns (N <= 32): whole-tile workgroups, kept columns split over workgroups
size_t skinny_prepared_workspace_bytes(const hinm_shape& s, int N);
hipError_t launch_spmm_skinny_prepared(const PreparedArgs& a, hipStream_t stream);
// few columns and few tiles: 16-row workgroups on the 16x16x64 form, reading the same prepared blocks
hipError_t launch_spmm_rows16_prepared(const PreparedArgs& a, hipStream_t stream);
// ... with all input rows resident in LDS (16 columns, K rows of 32 bytes beside the waves' slabs)
bool spmm_rows16_resident_supported(const PreparedArgs& a);
int spmm_rows16_prepared_blocks_per_wg(const PreparedArgs& a);  // 16-column blocks per workgroup chosen for this call (1, 2, 4)

}  // namespace hinm
