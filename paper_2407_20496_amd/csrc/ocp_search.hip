// Output-channel permutation search of gyro-permutation (arXiv 2407.20496, Section 4.1 Eq. 2 and
// Section 4.2): the output channels are re-distributed over the tiles of V channels so that
// column-vector pruning removes as little saliency as possible.  One iteration:
//   sampling   : the same number n of channels leaves every tile (positions given by the caller);
//   clustering : the T n sampled channels are grouped into T clusters of n (given by the caller; by
//                default every tile's own samples -- the balanced K-means of the paper is not part
//                of this file);
//   cost       : Eq. 4, cost[i][j] = saliency vector pruning removes from tile i's remaining channels
//                plus cluster j = the sum of the K - Kv smallest column scores, a score being
//                (sum over the remaining channels) + (sum over the cluster's channels) in binary64;
//   assignment : clusters -> tiles at minimal total cost (the solver of the tile-wise search);
//   apply      : the channels of cluster assign[i] fill the positions tile i vacated, in order.
// Indices read from the caller's arrays (positions, cluster items, channels) are clamped into range
// before use, so malformed input gives a meaningless order but no access out of bounds.
#include "hinm_internal.h"
#include "wave_reduce.h"

namespace hinm {
namespace {

constexpr int kThreads = 256;

template <int DT>
__device__ __forceinline__ double saliency_at(const uint16_t* W, const float* rho, size_t idx) {
  return rho ? (double)rho[idx] : (double)__builtin_fabsf(bits_to_float<DT>(W[idx]));
}

__device__ __forceinline__ int clamp_index(int x, int n) { return x < 0 ? 0 : (x >= n ? n - 1 : x); }

// base[t][k] = sum over the positions of tile t that stay (ascending position) of the saliency in
// column k; cluster[t][k] = the same over the channels of cluster t (cluster order).
template <int DT>
__global__ __launch_bounds__(kThreads) void ocp_sums_kernel(const uint16_t* __restrict__ W,
                                                            const float* __restrict__ rho,
                                                            const int32_t* __restrict__ row_order,
                                                            const int32_t* __restrict__ samples,
                                                            const int32_t* __restrict__ clusters,
                                                            double* __restrict__ base, double* __restrict__ cluster,
                                                            int T, int K, int V, int n) {
  __shared__ uint8_t leaves[kOcpMaxV];
  const int t = blockIdx.x;
  for (int p = threadIdx.x; p < V; p += kThreads) leaves[p] = 0;
  __syncthreads();
  for (int e = threadIdx.x; e < n; e += kThreads) leaves[clamp_index(samples[(size_t)t * n + e], V)] = 1;
  __syncthreads();
  const int k = blockIdx.y * kThreads + threadIdx.x;
  if (k >= K) return;
  double stay = 0.0;
  for (int p = 0; p < V; ++p) {
    if (leaves[p]) continue;
    const size_t row = (size_t)clamp_index(row_order[(size_t)t * V + p], T * V);
    stay += saliency_at<DT>(W, rho, row * K + k);
  }
  double come = 0.0;
  for (int e = 0; e < n; ++e) {
    const int q = clusters ? clamp_index(clusters[(size_t)t * n + e], T * n) : t * n + e;
    const int tq = q / n, eq = q % n;
    const size_t row = (size_t)clamp_index(row_order[(size_t)tq * V + clamp_index(samples[(size_t)tq * n + eq], V)], T * V);
    come += saliency_at<DT>(W, rho, row * K + k);
  }
  base[(size_t)t * K + k] = stay;
  cluster[(size_t)t * K + k] = come;
}

__device__ __forceinline__ unsigned long long ordered_key(double x) {
  const unsigned long long bits = (unsigned long long)__double_as_longlong(x);
  return (bits >> 63) ? ~bits : (bits | (1ull << 63));
}
__device__ __forceinline__ double key_value(unsigned long long key) {
  const unsigned long long bits = (key >> 63) ? (key & ~(1ull << 63)) : ~key;
  return __longlong_as_double((long long)bits);
}

// Workgroup-wide sum of one int per thread.  Three counters are used in rotation: every call clears
// the counter of the next call before its own barrier, when every thread has long left the call
// that read it last.
__device__ __forceinline__ int block_count(int local, int* counters, int call) {
  local = wave_sum(local);
  if (threadIdx.x == 0) counters[(call + 1) % 3] = 0;
  if ((threadIdx.x & 63) == 0) atomicAdd(&counters[call % 3], local);
  __syncthreads();
  return counters[call % 3];
}

// One workgroup per (tile i, cluster j): the K column scores live in registers (KPT per thread) as
// order-preserving 64-bit keys, split into two 32-bit words.  The Kv-th largest key is found bit by
// bit with 64 workgroup-wide counting passes -- 32 on the high words, then 32 on the low words of
// the keys whose high word equals the threshold's (the others have their low word cleared, and a
// candidate always has a bit set) -- so every pass is one full-rate 32-bit compare and one add per
// key.  Then everything below the threshold, plus the surplus of scores equal to it, is summed.
template <int KPT>
__global__ __launch_bounds__(kThreads) void ocp_cost_kernel(const double* __restrict__ base,
                                                            const double* __restrict__ cluster,
                                                            double* __restrict__ cost, int T, int K, int Kv) {
  __shared__ int counters[3];
  __shared__ double wave_sum_f64[kThreads / 64];
  const int j = blockIdx.x, i = blockIdx.y;
  const double* b = base + (size_t)i * K;
  const double* c = cluster + (size_t)j * K;
  uint32_t hi[KPT], lo[KPT];
#pragma unroll
  for (int q = 0; q < KPT; ++q) {
    const int k = q * kThreads + threadIdx.x;
    const unsigned long long key = (k < K) ? ordered_key(b[k] + c[k]) : 0ull;  // key 0: never counted below
    hi[q] = (uint32_t)(key >> 32);
    lo[q] = (uint32_t)key;
  }
  if (threadIdx.x < 3) counters[threadIdx.x] = 0;
  __syncthreads();
  int call = 0;
  uint32_t tau_hi = 0;
  for (int bit = 31; bit >= 0; --bit) {
    const uint32_t cand = tau_hi | (1u << bit);
    int local = 0;
#pragma unroll
    for (int q = 0; q < KPT; ++q) local += (hi[q] >= cand) ? 1 : 0;
    if (block_count(local, counters, call++) >= Kv) tau_hi = cand;
  }
  // keys above the threshold's high word always count; those below never do
  int above_hi = 0;
#pragma unroll
  for (int q = 0; q < KPT; ++q) {
    above_hi += (hi[q] > tau_hi) ? 1 : 0;
    lo[q] = (hi[q] == tau_hi) ? lo[q] : 0u;  // in place: the last pass reads the scores again
  }
  const int need = Kv - block_count(above_hi, counters, call++);  // >= 1 by the choice of tau_hi
  uint32_t tau_lo = 0;
  for (int bit = 31; bit >= 0; --bit) {
    const uint32_t cand = tau_lo | (1u << bit);
    int local = 0;
#pragma unroll
    for (int q = 0; q < KPT; ++q) local += (lo[q] >= cand) ? 1 : 0;
    if (block_count(local, counters, call++) >= need) tau_lo = cand;
  }
  const unsigned long long tau = ((unsigned long long)tau_hi << 32) | tau_lo;  // the Kv-th largest key
  int above = 0, equal = 0;
  double below = 0.0;
#pragma unroll
  for (int q = 0; q < KPT; ++q) {
    const int k = q * kThreads + threadIdx.x;
    if (k < K) {
      const unsigned long long key = ordered_key(b[k] + c[k]);
      above += key > tau ? 1 : 0;
      equal += key == tau ? 1 : 0;
      if (key < tau) below += key_value(key);
    }
  }
  const int n_above = block_count(above, counters, call++);
  const int n_equal = block_count(equal, counters, call++);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) below += __shfl_xor(below, off);
  if ((threadIdx.x & 63) == 0) wave_sum_f64[threadIdx.x >> 6] = below;
  __syncthreads();
  if (threadIdx.x == 0) {
    double total = 0.0;
    for (int w = 0; w < kThreads / 64; ++w) total += wave_sum_f64[w];
    const int pruned_equal = n_equal - (Kv - n_above);  // scores equal to the threshold that do not survive
    if (pruned_equal > 0) total += (double)pruned_equal * key_value(tau);
    cost[(size_t)i * T + j] = total;
  }
}

// The same with whole 64-bit keys and 64 passes of 64-bit compares (a quarter of the 32-bit rate): with
// 64 keys per thread the split form needs more registers than it saves time (measured 2.5 ms against
// 1.8 ms on a 16384-column layer), so the widest configuration keeps this form.
template <int KPT>
__global__ __launch_bounds__(kThreads) void ocp_cost_wide_kernel(const double* __restrict__ base,
                                                            const double* __restrict__ cluster,
                                                            double* __restrict__ cost, int T, int K, int Kv) {
  __shared__ int counters[3];
  __shared__ double wave_sum_f64[kThreads / 64];
  const int j = blockIdx.x, i = blockIdx.y;
  const double* b = base + (size_t)i * K;
  const double* c = cluster + (size_t)j * K;
  unsigned long long key[KPT];
#pragma unroll
  for (int q = 0; q < KPT; ++q) {
    const int k = q * kThreads + threadIdx.x;
    key[q] = (k < K) ? ordered_key(b[k] + c[k]) : 0ull;  // key 0 is below every real score's key
  }
  if (threadIdx.x < 3) counters[threadIdx.x] = 0;
  __syncthreads();
  int call = 0;
  unsigned long long tau = 0ull;  // becomes the Kv-th largest key
  for (int bit = 63; bit >= 0; --bit) {
    const unsigned long long cand = tau | (1ull << bit);
    int local = 0;
#pragma unroll
    for (int q = 0; q < KPT; ++q) local += (key[q] >= cand) ? 1 : 0;
    if (block_count(local, counters, call++) >= Kv) tau = cand;
  }
  int above = 0, equal = 0;
  double below = 0.0;
#pragma unroll
  for (int q = 0; q < KPT; ++q) {
    const int k = q * kThreads + threadIdx.x;
    if (k < K) {
      above += key[q] > tau ? 1 : 0;
      equal += key[q] == tau ? 1 : 0;
      if (key[q] < tau) below += key_value(key[q]);
    }
  }
  const int n_above = block_count(above, counters, call++);
  const int n_equal = block_count(equal, counters, call++);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) below += __shfl_xor(below, off);
  if ((threadIdx.x & 63) == 0) wave_sum_f64[threadIdx.x >> 6] = below;
  __syncthreads();
  if (threadIdx.x == 0) {
    double total = 0.0;
    for (int w = 0; w < kThreads / 64; ++w) total += wave_sum_f64[w];
    const int pruned_equal = n_equal - (Kv - n_above);  // scores equal to the threshold that do not survive
    if (pruned_equal > 0) total += (double)pruned_equal * key_value(tau);
    cost[(size_t)i * T + j] = total;
  }
}

// moved[i][e] = the channel of cluster assign[i], item e; block 0 also reports the total cost.
__global__ __launch_bounds__(kThreads) void ocp_moved_kernel(const double* __restrict__ cost,
                                                             const int32_t* __restrict__ assign,
                                                             const int32_t* __restrict__ row_order,
                                                             const int32_t* __restrict__ samples,
                                                             const int32_t* __restrict__ clusters,
                                                             int32_t* __restrict__ moved, double* __restrict__ objective,
                                                             int T, int V, int n) {
  const int i = blockIdx.x;
  const int j = clamp_index(assign[i], T);
  for (int e = threadIdx.x; e < n; e += kThreads) {
    const int q = clusters ? clamp_index(clusters[(size_t)j * n + e], T * n) : j * n + e;
    const int tq = q / n, eq = q % n;
    moved[(size_t)i * n + e] = row_order[(size_t)tq * V + clamp_index(samples[(size_t)tq * n + eq], V)];
  }
  if (objective && i == 0 && threadIdx.x == 0) {
    double total = 0.0;
    for (int r = 0; r < T; ++r) total += cost[(size_t)r * T + clamp_index(assign[r], T)];
    *objective = total;
  }
}

__global__ __launch_bounds__(kThreads) void ocp_write_kernel(const int32_t* __restrict__ moved,
                                                             const int32_t* __restrict__ samples,
                                                             int32_t* __restrict__ row_order, int V, int n) {
  const int i = blockIdx.x;
  for (int e = threadIdx.x; e < n; e += kThreads)
    row_order[(size_t)i * V + clamp_index(samples[(size_t)i * n + e], V)] = moved[(size_t)i * n + e];
}

// ---------------------------------------------------------------------------------------------
// Clustering phase (Section 4.2 names balanced K-means without detail; this is one reading): the
// T n sampled channels are the points, their saliency rows the features; T clusters of exactly n
// points.  A round = squared Euclidean distances in binary64 (columns in ascending order, separate
// multiply and add), a minimal-cost assignment of the points to the T n (cluster, slot) pairs, and
// centroids = sum of the members in ascending item order, divided by n.
// ---------------------------------------------------------------------------------------------
template <int DT>
__global__ __launch_bounds__(kThreads) void km_features_kernel(const uint16_t* __restrict__ W,
                                                               const float* __restrict__ rho,
                                                               const int32_t* __restrict__ row_order,
                                                               const int32_t* __restrict__ samples,
                                                               float* __restrict__ F, int T, int K, int V, int n) {
  const int q = blockIdx.x;
  const int k = blockIdx.y * kThreads + threadIdx.x;
  if (k >= K) return;
  const int t = q / n, e = q % n;
  const size_t row = (size_t)clamp_index(row_order[(size_t)t * V + clamp_index(samples[(size_t)t * n + e], V)], T * V);
  F[(size_t)q * K + k] = (float)saliency_at<DT>(W, rho, row * K + k);
}

__global__ __launch_bounds__(kThreads) void km_init_kernel(const float* __restrict__ F, double* __restrict__ C, int K,
                                                           int n) {
  const int c = blockIdx.x;
  const int k = blockIdx.y * kThreads + threadIdx.x;
  if (k < K) C[(size_t)c * K + k] = (double)F[(size_t)c * n * K + k];
}

// d[q][c], also written n times into the square matrix the assignment solver works on
__global__ __launch_bounds__(kThreads) void km_distance_kernel(const float* __restrict__ F,
                                                               const double* __restrict__ C,
                                                               double* __restrict__ dist, double* __restrict__ cost,
                                                               int T, int K, int n) {
#pragma clang fp contract(off)  // product and sum are rounded separately: that rounding is part of the definition
  const int q = blockIdx.x;
  const int c = blockIdx.y * kThreads + threadIdx.x;
  if (c >= T) return;
  const float* f = F + (size_t)q * K;
  const double* cen = C + (size_t)c * K;
  double acc = 0.0;
  for (int k = 0; k < K; ++k) {
    const double diff = (double)f[k] - cen[k];
    const double sq = diff * diff;
    acc = acc + sq;
  }
  dist[(size_t)q * T + c] = acc;
  double* out = cost + (size_t)q * T * n + (size_t)c * n;
  for (int s = 0; s < n; ++s) out[s] = acc;
}

// new centroids from the assignment (point q belongs to cluster assign[q] / n); block (0, 0) also
// reports the sum of the distances of the points to the centroids they were assigned to
__global__ __launch_bounds__(kThreads) void km_update_kernel(const float* __restrict__ F,
                                                             const int32_t* __restrict__ assign,
                                                             const double* __restrict__ dist, double* __restrict__ C,
                                                             double* __restrict__ objective, int T, int K, int n) {
  const int c = blockIdx.x;
  const int k = blockIdx.y * kThreads + threadIdx.x;
  const int points = T * n;
  if (k < K) {
    double acc = 0.0;
    for (int q = 0; q < points; ++q)
      if (clamp_index(assign[q], points) / n == c) acc += (double)F[(size_t)q * K + k];
    C[(size_t)c * K + k] = acc / (double)n;
  }
  if (objective && c == 0 && blockIdx.y == 0 && threadIdx.x == 0) {
    double total = 0.0;
    for (int q = 0; q < points; ++q) total += dist[(size_t)q * T + clamp_index(assign[q], points) / n];
    *objective = total;
  }
}

// clusters[c] = its items in ascending order
__global__ __launch_bounds__(kThreads) void km_clusters_kernel(const int32_t* __restrict__ assign,
                                                               int32_t* __restrict__ clusters, int T, int n) {
  const int c = blockIdx.x * kThreads + threadIdx.x;
  if (c >= T) return;
  const int points = T * n;
  int filled = 0;
  for (int q = 0; q < points && filled < n; ++q)
    if (clamp_index(assign[q], points) / n == c) clusters[(size_t)c * n + filled++] = q;
  for (; filled < n; ++filled) clusters[(size_t)c * n + filled] = c * n + filled;  // only after a malformed assignment
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

}  // namespace

KmeansWorkspace kmeans_workspace_layout(const hinm_shape& s, int n_samples) {
  const size_t T = s.M / s.V, points = T * (size_t)n_samples;
  KmeansWorkspace w;
  size_t off = 0;
  w.features = off; off += align256(points * s.K * sizeof(float));
  w.dist = off;     off += align256(points * T * sizeof(double));
  w.cost = off;     off += align256(points * points * sizeof(double));
  w.assign = off;   off += align256(points * sizeof(int32_t));
  w.total_bytes = off;
  return w;
}

hipError_t launch_ocp_cluster(const KmeansArgs& a, hipStream_t stream) {
  const hinm_shape& s = a.s;
  const int T = s.M / s.V, n = a.n_samples, points = T * n;
  const KmeansWorkspace w = kmeans_workspace_layout(s, n);
  uint8_t* ws = static_cast<uint8_t*>(a.workspace);
  float* F = reinterpret_cast<float*>(ws + w.features);
  double* dist = reinterpret_cast<double*>(ws + w.dist);
  double* cost = reinterpret_cast<double*>(ws + w.cost);
  int32_t* assign = reinterpret_cast<int32_t*>(ws + w.assign);
  const uint16_t* Wb = static_cast<const uint16_t*>(a.W);
  const int k_blocks = (s.K + kThreads - 1) / kThreads;
  if (s.dtype == HINM_F16)
    km_features_kernel<HINM_F16><<<dim3(points, k_blocks), kThreads, 0, stream>>>(Wb, a.rho, a.row_order, a.samples, F, T,
                                                                                   s.K, s.V, n);
  else
    km_features_kernel<HINM_BF16><<<dim3(points, k_blocks), kThreads, 0, stream>>>(Wb, a.rho, a.row_order, a.samples, F,
                                                                                    T, s.K, s.V, n);
  if (a.init_centroids) km_init_kernel<<<dim3(T, k_blocks), kThreads, 0, stream>>>(F, a.centroids, s.K, n);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  for (int r = 0; r < a.rounds; ++r) {
    km_distance_kernel<<<dim3(points, (T + kThreads - 1) / kThreads), kThreads, 0, stream>>>(F, a.centroids, dist, cost,
                                                                                             T, s.K, n);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    e = launch_assignment(cost, assign, 1, points, stream);
    if (e != hipSuccess) return e;
    km_update_kernel<<<dim3(T, k_blocks), kThreads, 0, stream>>>(F, assign, dist, a.centroids,
                                                                 a.objective ? a.objective + r : nullptr, T, s.K, n);
  }
  km_clusters_kernel<<<(T + kThreads - 1) / kThreads, kThreads, 0, stream>>>(assign, a.clusters, T, n);
  return hipGetLastError();
}

OcpWorkspace ocp_workspace_layout(const hinm_shape& s, int n_samples) {
  const size_t T = s.M / s.V;
  OcpWorkspace w;
  size_t off = 0;
  w.base = off;    off += align256(T * s.K * sizeof(double));
  w.cluster = off; off += align256(T * s.K * sizeof(double));
  w.cost = off;    off += align256(T * T * sizeof(double));
  w.assign = off;  off += align256(T * sizeof(int32_t));
  w.moved = off;   off += align256(T * (size_t)n_samples * sizeof(int32_t));
  w.total_bytes = off;
  return w;
}

hipError_t launch_ocp_search(const OcpArgs& a, hipStream_t stream) {
  const hinm_shape& s = a.s;
  const int T = s.M / s.V, n = a.n_samples;
  const OcpWorkspace w = ocp_workspace_layout(s, n);
  uint8_t* ws = static_cast<uint8_t*>(a.workspace);
  double* base = reinterpret_cast<double*>(ws + w.base);
  double* cluster = reinterpret_cast<double*>(ws + w.cluster);
  double* cost = reinterpret_cast<double*>(ws + w.cost);
  int32_t* assign = reinterpret_cast<int32_t*>(ws + w.assign);
  int32_t* moved = reinterpret_cast<int32_t*>(ws + w.moved);
  const uint16_t* Wb = static_cast<const uint16_t*>(a.W);
  const dim3 sums_grid(T, (s.K + kThreads - 1) / kThreads);
  const dim3 cost_grid(T, T);
  for (int it = 0; it < a.iters; ++it) {
    const int32_t* smp = a.samples + (size_t)it * T * n;
    const int32_t* cl = a.clusters ? a.clusters + (size_t)it * T * n : nullptr;
    if (s.dtype == HINM_F16)
      ocp_sums_kernel<HINM_F16><<<sums_grid, kThreads, 0, stream>>>(Wb, a.rho, a.row_order, smp, cl, base, cluster, T,
                                                                     s.K, s.V, n);
    else
      ocp_sums_kernel<HINM_BF16><<<sums_grid, kThreads, 0, stream>>>(Wb, a.rho, a.row_order, smp, cl, base, cluster, T,
                                                                      s.K, s.V, n);
    if (s.K <= 4 * kThreads) ocp_cost_kernel<4><<<cost_grid, kThreads, 0, stream>>>(base, cluster, cost, T, s.K, s.Kv);
    else if (s.K <= 16 * kThreads) ocp_cost_kernel<16><<<cost_grid, kThreads, 0, stream>>>(base, cluster, cost, T, s.K, s.Kv);
    else ocp_cost_wide_kernel<64><<<cost_grid, kThreads, 0, stream>>>(base, cluster, cost, T, s.K, s.Kv);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    e = launch_assignment(cost, assign, 1, T, stream);
    if (e != hipSuccess) return e;
    ocp_moved_kernel<<<T, kThreads, 0, stream>>>(cost, assign, a.row_order, smp, cl, moved,
                                                 a.objective ? a.objective + it : nullptr, T, s.V, n);
    ocp_write_kernel<<<T, kThreads, 0, stream>>>(moved, smp, a.row_order, s.V, n);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace hinm
