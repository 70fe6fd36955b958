// Tile-wise input-channel permutation search of gyro-permutation (arXiv 2407.20496, Section 4.1
// Eq. 3 and Section 4.2): the kept column vectors of every tile are re-arranged so that the 2:4 step
// prunes as little saliency as possible.  Every four consecutive kept vectors form one partition.
// One iteration, per tile:
//   sampling   : one vector per partition, chosen by the caller (`samples`);
//   cost       : Eq. 4, cost[i][j] = saliency the 2:4 step prunes in partition i when the slot it
//                vacated holds sample j = sum over rows of the two smallest of four values, added in
//                binary64 in ascending row order.  With (m1, m2) the two smallest of partition i's
//                three remaining values this is sum_r m1 + min(sample_j, m2): a (min, +) contraction
//                over the V rows, the data-parallel part of the search;
//   assignment : samples -> partitions minimising the total cost (shortest augmenting paths with row
//                and column potentials, one workgroup per tile);
//   apply      : every sample moves into the slot its partition vacated.
// The arrangement is tracked as a permutation of the slots of the incoming vector index, so the
// saliencies are gathered from W (or rho) only once.
#include "hinm_internal.h"
#include "wave_reduce.h"

namespace hinm {
namespace {

constexpr int kThreads = 256;
constexpr int kMaxP = kIcpMaxPartitions;
constexpr int kSmallP = 128;  // up to here a tile's cost matrix fits in LDS
constexpr int kCostRowsPerThread = 8;
constexpr double kInf = 1e300;

// G[t][r][slot] = saliency of W[tV + r][vec_idx[t][slot]]: the caller's rho, or |w|; order = identity
template <int DT>
__global__ __launch_bounds__(kThreads) void icp_gather_kernel(const uint16_t* __restrict__ W,
                                                              const float* __restrict__ rho,
                                                              const int32_t* __restrict__ vec_idx,
                                                              float* __restrict__ G, int32_t* __restrict__ order,
                                                              int K, int V, int Kv) {
  const int t = blockIdx.x, r = blockIdx.y;
  const size_t row = (size_t)t * V + r;
  const int32_t* vi = vec_idx + (size_t)t * Kv;
  float* g = G + row * Kv;
  for (int s = threadIdx.x; s < Kv; s += kThreads) {
    const int c = vi[s];
    g[s] = rho ? rho[row * K + c] : __builtin_fabsf(bits_to_float<DT>(W[row * K + c]));
    if (r == 0) order[(size_t)t * Kv + s] = s;
  }
}

// Per row and partition: the sampled value, and the two smallest of the three remaining ones.
__global__ __launch_bounds__(kThreads) void icp_split_kernel(const float* __restrict__ G,
                                                             const int32_t* __restrict__ order,
                                                             const uint8_t* __restrict__ samples,
                                                             float* __restrict__ S, float* __restrict__ M1,
                                                             float* __restrict__ M2, int V, int Kv) {
  const int t = blockIdx.x, r = blockIdx.y;
  const int P = Kv / 4;
  const size_t row = (size_t)t * V + r;
  const float* g = G + row * Kv;
  const int32_t* ord = order + (size_t)t * Kv;
  const uint8_t* smp = samples + (size_t)t * P;
  for (int i = threadIdx.x; i < P; i += kThreads) {
    const int pick = smp[i] & 3;
    float v[4];
#pragma unroll
    for (int m = 0; m < 4; ++m) v[m] = g[ord[4 * i + m]];
    const float s = pick == 0 ? v[0] : pick == 1 ? v[1] : pick == 2 ? v[2] : v[3];
    // the two smallest of the three that stay: the sampled one is lifted out of the way
#pragma unroll
    for (int m = 0; m < 4; ++m) v[m] = (m == pick) ? __builtin_inff() : v[m];
    const float lo01 = __builtin_fminf(v[0], v[1]), hi01 = __builtin_fmaxf(v[0], v[1]);
    const float lo23 = __builtin_fminf(v[2], v[3]), hi23 = __builtin_fmaxf(v[2], v[3]);
    const float m1 = __builtin_fminf(lo01, lo23);
    const float m2 = __builtin_fminf(__builtin_fmaxf(lo01, lo23), __builtin_fminf(hi01, hi23));
    S[row * P + i] = s;
    M1[row * P + i] = m1;
    M2[row * P + i] = m2;
  }
}

// cost[t][i][j] = sum_r (double) m1[r][i] + (double) min(s[r][j], m2[r][i]), rows ascending.
// One thread owns one sample j and kCostRowsPerThread consecutive partitions i; the (m1, m2) pairs
// are the same for the whole workgroup.
__global__ __launch_bounds__(kThreads) void icp_cost_kernel(const float* __restrict__ S, const float* __restrict__ M1,
                                                            const float* __restrict__ M2, double* __restrict__ cost,
                                                            int V, int P) {
  const int t = blockIdx.z;
  const int i0 = blockIdx.y * kCostRowsPerThread;
  const int j = blockIdx.x * kThreads + threadIdx.x;
  const float* s_t = S + (size_t)t * V * P;
  const float* m1_t = M1 + (size_t)t * V * P;
  const float* m2_t = M2 + (size_t)t * V * P;
  double acc[kCostRowsPerThread];
#pragma unroll
  for (int e = 0; e < kCostRowsPerThread; ++e) acc[e] = 0.0;
  const int jj = j < P ? j : P - 1;  // lanes beyond P repeat the last sample and store nothing
  for (int r = 0; r < V; ++r) {
    const float s = s_t[(size_t)r * P + jj];
#pragma unroll
    for (int e = 0; e < kCostRowsPerThread; ++e) {
      const int i = (i0 + e < P) ? i0 + e : P - 1;  // workgroup-uniform
      const float m1 = m1_t[(size_t)r * P + i];
      const float m2 = m2_t[(size_t)r * P + i];
      acc[e] += (double)m1 + (double)__builtin_fminf(s, m2);
    }
  }
  if (j < P) {
#pragma unroll
    for (int e = 0; e < kCostRowsPerThread; ++e)
      if (i0 + e < P) cost[((size_t)t * P + i0 + e) * P + j] = acc[e];
  }
}

// Linear assignment by shortest augmenting paths (rows = partitions, columns = samples), one
// workgroup per tile.  Index 0 is the virtual start column; rows and columns are 1-based inside.
// Every loop is bounded by the problem size, so the kernel ends for any input; if the costs are not
// finite no augmenting path is found and the tile keeps its arrangement (identity assignment).
// Each of the up to n^2 inner steps reads one row of the cost matrix and is one dependent chain of
// memory latency, reduction and barriers: for n <= MAXN = 128 the matrix is held in LDS (IN_LDS) and
// the workgroup has two waves, which makes a step about three times shorter.
template <int MAXN, int THREADS, bool IN_LDS>
__global__ __launch_bounds__(THREADS) void icp_assign_kernel(const double* __restrict__ cost,
                                                             int32_t* __restrict__ assign, int n) {
  __shared__ double u[MAXN + 1], v[MAXN + 1], minv[MAXN + 1];
  __shared__ int p[MAXN + 1], way[MAXN + 1];
  __shared__ uint8_t used[MAXN + 1];
  __shared__ double red_val[THREADS / 64];
  __shared__ int red_idx[THREADS / 64];
  extern __shared__ __attribute__((aligned(16))) double cost_lds[];  // n * n doubles when IN_LDS
  const int t = blockIdx.x;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const double* a = cost + (size_t)t * n * n;
  if constexpr (IN_LDS) {
    for (int e = tid; e < n * n; e += THREADS) cost_lds[e] = a[e];
  }
  for (int j = tid; j <= n; j += THREADS) {
    u[j] = 0.0;
    v[j] = 0.0;
    p[j] = 0;
    way[j] = 0;
    used[j] = 0;  // until the main loop: "row j is matched"
  }
  __syncthreads();
  // Start from feasible potentials and a greedy partial matching instead of from nothing: v[j] = the
  // smallest cost in column j, u[i] = the smallest reduced cost in row i, and row i takes the column
  // where that minimum sits (the lowest one) if it is still free.  Most rows are matched here, with n
  // reductions; only the others need an augmenting path (up to n reductions each).
  {
    const double* m = IN_LDS ? cost_lds : a;
    for (int j = 1 + tid; j <= n; j += THREADS) {
      double lo = kInf;
      for (int i = 0; i < n; ++i) {
        const double x = m[(size_t)i * n + (j - 1)];
        lo = x < lo ? x : lo;
      }
      v[j] = lo < kInf ? lo : 0.0;
    }
    __syncthreads();
    for (int i = 1; i <= n; ++i) {
      const double* arow = m + (size_t)(i - 1) * n;
      double best = kInf;
      int best_j = n + 1;
      for (int j = 1 + tid; j <= n; j += THREADS) {
        const double x = arow[j - 1] - v[j];
        if (x < best) {
          best = x;
          best_j = j;
        }
      }
      wave_argmin(best, best_j, n + 1);
      if (lane == 0) {
        red_val[wave] = best;
        red_idx[wave] = best_j;
      }
      __syncthreads();
      if (tid == 0) {
        double lo = red_val[0];
        int at = red_idx[0];
        for (int w = 1; w < THREADS / 64; ++w)
          if (red_val[w] < lo || (red_val[w] == lo && red_idx[w] < at)) {
            lo = red_val[w];
            at = red_idx[w];
          }
        if (lo < kInf && at <= n) {
          u[i] = lo;
          if (p[at] == 0) {
            p[at] = i;
            used[i] = 1;
          }
        }
      }
      __syncthreads();
    }
  }
  // rows still to be matched, in ascending order
  __shared__ int free_list[MAXN];
  __shared__ int n_free;
  if (tid == 0) {
    int count = 0;
    for (int i = 1; i <= n; ++i)
      if (!used[i]) free_list[count++] = i;
    n_free = count;
  }
  __syncthreads();
  const int free_rows = n_free;
  bool failed = false;
  for (int f = 0; f < free_rows && !failed; ++f) {
    const int i = free_list[f];
    if (tid == 0) p[0] = i;
    for (int j = tid; j <= n; j += THREADS) {
      minv[j] = kInf;
      used[j] = 0;
    }
    int j0 = 0;
    __syncthreads();
    for (int step = 0; step <= n; ++step) {  // every pass marks one more column used
      if (tid == 0) used[j0] = 1;
      __syncthreads();
      const int i0 = p[j0];
      const double ui0 = u[i0];
      const double* arow = (IN_LDS ? cost_lds : a) + (size_t)(i0 - 1) * n;
      double best = kInf;
      int best_j = n + 1;
      for (int j = 1 + tid; j <= n; j += THREADS) {
        if (used[j]) continue;
        const double cur = arow[j - 1] - ui0 - v[j];
        double m = minv[j];
        if (cur < m) {
          m = cur;
          minv[j] = cur;
          way[j] = j0;
        }
        if (m < best) {  // j ascends inside a thread: the first minimum is the lowest column
          best = m;
          best_j = j;
        }
      }
      wave_argmin(best, best_j, n + 1);
      if (lane == 0) {
        red_val[wave] = best;
        red_idx[wave] = best_j;
      }
      __syncthreads();
      double delta = red_val[0];
      int j1 = red_idx[0];
#pragma unroll
      for (int w = 1; w < THREADS / 64; ++w) {
        const double ob = red_val[w];
        const int oj = red_idx[w];
        if (ob < delta || (ob == delta && oj < j1)) {
          delta = ob;
          j1 = oj;
        }
      }
      if (!(delta < kInf) || j1 > n) {  // same value in every thread
        failed = true;
        break;
      }
      for (int j = tid; j <= n; j += THREADS) {
        if (used[j]) {
          u[p[j]] += delta;  // the rows matched to used columns are distinct
          v[j] -= delta;
        } else {
          minv[j] -= delta;
        }
      }
      j0 = j1;
      __syncthreads();
      if (p[j0] == 0) break;  // a free column: the path is complete
    }
    if (failed) break;
    if (tid == 0) {
      int jj = j0;
      for (int guard = 0; jj != 0 && guard <= n; ++guard) {
        const int j1 = way[jj];
        p[jj] = p[j1];
        jj = j1;
      }
    }
    __syncthreads();
  }
  int32_t* out = assign + (size_t)t * n;
  if (failed) {
    for (int i = tid; i < n; i += THREADS) out[i] = i;
  } else {
    for (int j = 1 + tid; j <= n; j += THREADS) {
      const int row = p[j];
      if (row >= 1) out[row - 1] = j - 1;
    }
  }
}

// Moves sample assign[i] into the slot partition i vacated, and reports the total cost of the
// assignment (partitions added in ascending order).
__global__ __launch_bounds__(kThreads) void icp_apply_kernel(const double* __restrict__ cost,
                                                             const int32_t* __restrict__ assign,
                                                             const uint8_t* __restrict__ samples,
                                                             int32_t* __restrict__ order,
                                                             double* __restrict__ objective, int Kv) {
  __shared__ int32_t moved[kMaxP];
  __shared__ double picked[kMaxP];
  const int t = blockIdx.x;
  const int P = Kv / 4;
  const int32_t* asg = assign + (size_t)t * P;
  const uint8_t* smp = samples + (size_t)t * P;
  int32_t* ord = order + (size_t)t * Kv;
  for (int i = threadIdx.x; i < P; i += kThreads) {
    int j = asg[i];
    j = (j >= 0 && j < P) ? j : i;
    moved[i] = ord[4 * j + (smp[j] & 3)];
    picked[i] = cost[((size_t)t * P + i) * P + j];
  }
  __syncthreads();
  for (int i = threadIdx.x; i < P; i += kThreads) ord[4 * i + (smp[i] & 3)] = moved[i];
  if (objective && threadIdx.x == 0) {
    double total = 0.0;
    for (int i = 0; i < P; ++i) total += picked[i];
    objective[t] = total;
  }
}

// vec_idx[t][pos] = (incoming vec_idx)[t][order[t][pos]], in place through LDS.
__global__ __launch_bounds__(kThreads) void icp_finish_kernel(const int32_t* __restrict__ order,
                                                              int32_t* __restrict__ vec_idx, int Kv) {
  __shared__ int32_t cols[4 * kMaxP];
  const int t = blockIdx.x;
  int32_t* vi = vec_idx + (size_t)t * Kv;
  const int32_t* ord = order + (size_t)t * Kv;
  for (int s = threadIdx.x; s < Kv; s += kThreads) cols[s] = vi[s];
  __syncthreads();
  for (int s = threadIdx.x; s < Kv; s += kThreads) {
    const int o = ord[s];
    vi[s] = cols[(o >= 0 && o < Kv) ? o : s];
  }
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

}  // namespace

hipError_t launch_assignment(const double* cost, int32_t* assign, int problems, int n, hipStream_t stream) {
  if (n <= kSmallP) {  // the cost matrix in LDS: up to 128 KB beside the solver's own arrays
    constexpr auto kernel = icp_assign_kernel<kSmallP, 128, true>;
    if (hipError_t e = raise_lds_limit<kernel>(kSmallP * kSmallP * (int)sizeof(double)); e != hipSuccess) return e;
    kernel<<<problems, 128, (size_t)n * n * sizeof(double), stream>>>(cost, assign, n);
  } else {
    icp_assign_kernel<kMaxP, kThreads, false><<<problems, kThreads, 0, stream>>>(cost, assign, n);
  }
  return hipGetLastError();
}

IcpWorkspace icp_workspace_layout(const hinm_shape& s) {
  const size_t T = s.M / s.V, P = s.Kv / 4;
  IcpWorkspace w;
  size_t off = 0;
  w.gathered = off; off += align256((size_t)s.M * s.Kv * sizeof(float));
  w.order = off;    off += align256(T * s.Kv * sizeof(int32_t));
  w.sample = off;   off += align256((size_t)s.M * P * sizeof(float));
  w.min1 = off;     off += align256((size_t)s.M * P * sizeof(float));
  w.min2 = off;     off += align256((size_t)s.M * P * sizeof(float));
  w.cost = off;     off += align256(T * P * P * sizeof(double));
  w.assign = off;   off += align256(T * P * sizeof(int32_t));
  w.total_bytes = off;
  return w;
}

hipError_t launch_icp_search(const IcpArgs& a, hipStream_t stream) {
  const hinm_shape& s = a.s;
  const int T = s.M / s.V, P = s.Kv / 4;
  const IcpWorkspace w = icp_workspace_layout(s);
  uint8_t* base = static_cast<uint8_t*>(a.workspace);
  float* G = reinterpret_cast<float*>(base + w.gathered);
  int32_t* order = reinterpret_cast<int32_t*>(base + w.order);
  float* S = reinterpret_cast<float*>(base + w.sample);
  float* M1 = reinterpret_cast<float*>(base + w.min1);
  float* M2 = reinterpret_cast<float*>(base + w.min2);
  double* cost = reinterpret_cast<double*>(base + w.cost);
  int32_t* assign = reinterpret_cast<int32_t*>(base + w.assign);
  const uint16_t* Wb = static_cast<const uint16_t*>(a.W);
  const dim3 rows_grid(T, s.V);
  if (s.dtype == HINM_F16)
    icp_gather_kernel<HINM_F16><<<rows_grid, kThreads, 0, stream>>>(Wb, a.rho, a.vec_idx, G, order, s.K, s.V, s.Kv);
  else
    icp_gather_kernel<HINM_BF16><<<rows_grid, kThreads, 0, stream>>>(Wb, a.rho, a.vec_idx, G, order, s.K, s.V, s.Kv);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const dim3 cost_grid((P + kThreads - 1) / kThreads, (P + kCostRowsPerThread - 1) / kCostRowsPerThread, T);
  for (int it = 0; it < a.iters; ++it) {
    const uint8_t* smp = a.samples + (size_t)it * T * P;
    icp_split_kernel<<<rows_grid, kThreads, 0, stream>>>(G, order, smp, S, M1, M2, s.V, s.Kv);
    icp_cost_kernel<<<cost_grid, kThreads, 0, stream>>>(S, M1, M2, cost, s.V, P);
    e = launch_assignment(cost, assign, T, P, stream);
    if (e != hipSuccess) return e;
    icp_apply_kernel<<<T, kThreads, 0, stream>>>(cost, assign, smp, order,
                                                 a.objective ? a.objective + (size_t)it * T : nullptr, s.Kv);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  icp_finish_kernel<<<T, kThreads, 0, stream>>>(order, a.vec_idx, s.Kv);
  return hipGetLastError();
}

}  // namespace hinm
