// C-ABI entry points of libhinm: host-side argument validation and kernel dispatch.
// Every check here runs before anything is launched, so the error paths need no GPU.
#include "hinm_internal.h"
#include "prepared_layout.h"
#include "hinm_calib.h"


namespace {

using namespace hinm;

hinm_status check_shape(const hinm_shape* s) {
  if (!s) return HINM_ERR_NULL;
  if (s->dtype != HINM_F16 && s->dtype != HINM_BF16) return HINM_ERR_DTYPE;
  if (s->M <= 0 || s->K <= 0 || s->V <= 0 || s->Kv <= 0) return HINM_ERR_SHAPE;
  if (s->M % s->V != 0) return HINM_ERR_SHAPE;
  if (s->Kv > s->K || s->Kv % 8 != 0) return HINM_ERR_SHAPE;
  return HINM_OK;
}

bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

hinm_status check_spmm(const hinm_shape* s, int32_t N, const void* vals, const uint8_t* nm_idx,
                       const int32_t* vec_idx, const void* X, int64_t ldx, const void* Y, int64_t ldy,
                       uint32_t flags) {
  hinm_status st = check_shape(s);
  if (st != HINM_OK) return st;
  if (!vals || !nm_idx || !vec_idx || !X || !Y) return HINM_ERR_NULL;
  if (N <= 0 || ldx < N || ldy < N) return HINM_ERR_SHAPE;
  if (N > 1 && (ldx % 8 != 0 || ldy % 8 != 0)) return HINM_ERR_SHAPE;
  if (!aligned(vals, 16) || !aligned(X, 16) || !aligned(Y, 16)) return HINM_ERR_SHAPE;
  const uint32_t known = HINM_EPI_RELU | HINM_OUT_F32 | HINM_KERNEL_REFERENCE | HINM_KERNEL_SMFMAC | HINM_KERNEL_GEMV;
  if (flags & ~known) return HINM_ERR_UNSUPPORTED;
  const uint32_t forced = flags & (HINM_KERNEL_REFERENCE | HINM_KERNEL_SMFMAC | HINM_KERNEL_GEMV);
  if (forced & (forced - 1)) return HINM_ERR_UNSUPPORTED;  // at most one kernel may be forced
  return HINM_OK;
}

hinm_status run_spmm(const SpmmArgs& a, uint32_t flags, hipStream_t stream) {
  hipError_t e;
  if (flags & HINM_KERNEL_REFERENCE) {
    e = launch_spmm_reference(a, stream);
  } else if (flags & HINM_KERNEL_SMFMAC) {
    if (spmm_tile_supported(a)) e = launch_spmm_tile(a, stream);
    else if (spmm_skinny_supported(a)) e = launch_spmm_skinny(a, stream);
    else return HINM_ERR_UNSUPPORTED;
  } else if (flags & HINM_KERNEL_GEMV) {
    if (a.N > 16 || !spmm_skinny_supported(a)) return HINM_ERR_UNSUPPORTED;
    e = launch_spmm_skinny(a, stream);
  } else {
    // by shape: few columns -> k-split skinny kernel (bandwidth-bound on the packed weights);
    // otherwise the tile kernel; shapes neither covers fall back to the plain kernel.
    if (a.N <= 16 && spmm_skinny_supported(a)) e = launch_spmm_skinny(a, stream);
    else if (spmm_tile_supported(a)) e = launch_spmm_tile(a, stream);
    else if (spmm_skinny_supported(a)) e = launch_spmm_skinny(a, stream);
    else e = launch_spmm_reference(a, stream);
  }
  return e == hipSuccess ? HINM_OK : HINM_ERR_DEVICE;
}

size_t elem_bytes_out(uint32_t flags) { return (flags & HINM_OUT_F32) ? 4 : 2; }

// ---- hinm_pack_static: the score workspace of the pack kernels in a file-scope device array -------------
// One binary64 score per tile and column, at most kStaticScoreCount of them (4 MiB).  Every GPU the library runs
// on holds its own copy of the array at its own address until the process ends.
constexpr size_t kStaticScoreCount = (size_t)HINM_PACK_STATIC_MAX_SCORES;
static __device__ __align__(256) double scratch[kStaticScoreCount];

// In host code `scratch` is only a stand-in for the symbol: the device address comes from
// hipGetSymbolAddress, once per device with that device current, and is kept per device.
constexpr int kStaticMaxDevices = 64;
hipError_t static_scores(double** out) {
  static std::atomic<double*> per_device[kStaticMaxDevices];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kStaticMaxDevices) return hipErrorInvalidDevice;
  double* p = per_device[dev].load(std::memory_order_acquire);
  if (!p) {
    void* addr = nullptr;
    e = hipGetSymbolAddress(&addr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!addr) return hipErrorInvalidSymbol;
    p = static_cast<double*>(addr);
    per_device[dev].store(p, std::memory_order_release);  // two first calls racing store the same address
  }
  *out = p;
  return hipSuccess;
}

}  // namespace

extern "C" {

hinm_status hinm_pack_sizes(const hinm_shape* shape, size_t* vals_bytes, size_t* nm_bytes, size_t* vec_bytes,
                            size_t* workspace_bytes) {
  hinm_status st = check_shape(shape);
  if (st != HINM_OK) return st;
  const size_t M = shape->M, K = shape->K, Kv = shape->Kv, T = shape->M / shape->V;
  if (vals_bytes) *vals_bytes = M * (Kv / 2) * 2;
  if (nm_bytes) *nm_bytes = M * (Kv / 8);
  if (vec_bytes) *vec_bytes = T * Kv * sizeof(int32_t);
  if (workspace_bytes) *workspace_bytes = T * K * sizeof(double);
  return HINM_OK;
}

static hinm_status run_pack(const hinm_shape* shape, const void* W, const float* rho, bool with_rho,
                            const int32_t* tile_order, void* vals, uint8_t* nm_idx, bool with_nm, int32_t* vec_idx,
                            void* workspace, size_t workspace_bytes, void* stream) {
  hinm_status st = check_shape(shape);
  if (st != HINM_OK) return st;
  if (!W || !vals || !vec_idx || (with_nm && !nm_idx) || (with_rho && !rho)) return HINM_ERR_NULL;
  size_t need = 0;
  hinm_pack_sizes(shape, nullptr, nullptr, nullptr, &need);
  if (!workspace || workspace_bytes < need || !aligned(workspace, 8)) return HINM_ERR_WORKSPACE;
  if (!aligned(vals, with_nm ? 8 : 16) || !aligned(vec_idx, 4) || !aligned(W, 2)) return HINM_ERR_SHAPE;
  if (with_rho && !aligned(rho, 4)) return HINM_ERR_SHAPE;
  if (tile_order && (!aligned(tile_order, 4) || shape->K > kPackOrderMaxK)) return HINM_ERR_UNSUPPORTED;
  const PackArgs a{*shape, W, rho, tile_order, vals, with_nm ? nm_idx : nullptr, vec_idx,
                   static_cast<double*>(workspace)};
  hipError_t e = launch_pack(a, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? HINM_OK : HINM_ERR_DEVICE;
}

hinm_status hinm_pack(const hinm_shape* shape, const void* W, void* vals, uint8_t* nm_idx, int32_t* vec_idx,
                      void* workspace, size_t workspace_bytes, void* stream) {
  return run_pack(shape, W, nullptr, false, nullptr, vals, nm_idx, true, vec_idx, workspace, workspace_bytes, stream);
}

hinm_status hinm_pack_static(const hinm_shape* shape, const void* W, void* vals, uint8_t* nm_idx, int32_t* vec_idx,
                             void* stream) {
  hinm_status st = check_shape(shape);
  if (st != HINM_OK) return st;
  if (!W || !vals || !nm_idx || !vec_idx) return HINM_ERR_NULL;
  // the size limit comes before anything touches the device
  if ((size_t)(shape->M / shape->V) * (size_t)shape->K > kStaticScoreCount) return HINM_ERR_WORKSPACE;
  if (!aligned(vals, 8) || !aligned(vec_idx, 4) || !aligned(W, 2)) return HINM_ERR_SHAPE;
  double* scores = nullptr;
  if (static_scores(&scores) != hipSuccess) return HINM_ERR_DEVICE;
  // every score the select step reads is written by the score step of the same call: nothing to clear
  const PackArgs a{*shape, W, nullptr, nullptr, vals, nm_idx, vec_idx, scores};
  hipError_t e = launch_pack(a, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? HINM_OK : HINM_ERR_DEVICE;
}

hinm_status hinm_pack_ordered(const hinm_shape* shape, const void* W, const int32_t* tile_order, void* vals,
                              uint8_t* nm_idx, int32_t* vec_idx, void* workspace, size_t workspace_bytes,
                              void* stream) {
  return run_pack(shape, W, nullptr, false, tile_order, vals, nm_idx, true, vec_idx, workspace, workspace_bytes,
                  stream);
}

hinm_status hinm_pack_scored(const hinm_shape* shape, const void* W, const float* rho, const int32_t* tile_order,
                             void* vals, uint8_t* nm_idx, int32_t* vec_idx, void* workspace, size_t workspace_bytes,
                             void* stream) {
  return run_pack(shape, W, rho, true, tile_order, vals, nm_idx, true, vec_idx, workspace, workspace_bytes, stream);
}

hinm_status hinm_pack_vectors(const hinm_shape* shape, const void* W, const float* rho, const int32_t* tile_order,
                              void* vals_v, int32_t* vec_idx, void* workspace, size_t workspace_bytes, void* stream) {
  return run_pack(shape, W, rho, rho != nullptr, tile_order, vals_v, nullptr, false, vec_idx, workspace,
                  workspace_bytes, stream);
}

hinm_status hinm_apply_row_order(const void* src, void* dst, const int32_t* row_order, int32_t rows, size_t row_bytes,
                                 void* stream) {
  if (!src || !dst || !row_order) return HINM_ERR_NULL;
  if (rows <= 0 || row_bytes == 0 || row_bytes % 4 != 0 || !aligned(src, 4) || !aligned(dst, 4) || !aligned(row_order, 4) ||
      src == dst)
    return HINM_ERR_SHAPE;
  return launch_gather_rows(src, dst, row_order, rows, row_bytes, static_cast<hipStream_t>(stream)) == hipSuccess
             ? HINM_OK
             : HINM_ERR_DEVICE;
}

hinm_status hinm_tile_order(const hinm_shape* shape, const int32_t* vec_idx, int32_t* tile_order, void* stream) {
  hinm_status st = check_shape(shape);
  if (st != HINM_OK) return st;
  if (!vec_idx || !tile_order) return HINM_ERR_NULL;
  if (!aligned(vec_idx, 4) || !aligned(tile_order, 4)) return HINM_ERR_SHAPE;
  if (shape->K > kPackOrderMaxK) return HINM_ERR_UNSUPPORTED;
  return launch_tile_order(*shape, vec_idx, tile_order, static_cast<hipStream_t>(stream)) == hipSuccess ? HINM_OK
                                                                                                          : HINM_ERR_DEVICE;
}

static hinm_status check_icp_shape(const hinm_shape* shape) {
  hinm_status st = check_shape(shape);
  if (st != HINM_OK) return st;
  if (shape->Kv / 4 > kIcpMaxPartitions || shape->M / shape->V > 65535 || shape->V > 65535) return HINM_ERR_UNSUPPORTED;
  return HINM_OK;
}

hinm_status hinm_icp_sizes(const hinm_shape* shape, size_t* workspace_bytes) {
  hinm_status st = check_icp_shape(shape);
  if (st != HINM_OK) return st;
  if (!workspace_bytes) return HINM_ERR_NULL;
  *workspace_bytes = icp_workspace_layout(*shape).total_bytes;
  return HINM_OK;
}

hinm_status hinm_icp_search(const hinm_shape* shape, const void* W, const float* rho, int32_t* vec_idx,
                            const uint8_t* samples, int32_t iters, double* objective, void* workspace,
                            size_t workspace_bytes, void* stream) {
  hinm_status st = check_icp_shape(shape);
  if (st != HINM_OK) return st;
  if ((!W && !rho) || !vec_idx || (iters > 0 && !samples)) return HINM_ERR_NULL;
  if (iters < 0) return HINM_ERR_SHAPE;
  if (!aligned(vec_idx, 4) || (rho && !aligned(rho, 4)) || (!rho && !aligned(W, 2)) ||
      (objective && !aligned(objective, 8)))
    return HINM_ERR_SHAPE;
  const size_t need = icp_workspace_layout(*shape).total_bytes;
  if (!workspace || workspace_bytes < need || !aligned(workspace, 256)) return HINM_ERR_WORKSPACE;
  if (iters == 0) return HINM_OK;
  const IcpArgs a{*shape, W, rho, vec_idx, samples, iters, objective, workspace};
  hipError_t e = launch_icp_search(a, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? HINM_OK : HINM_ERR_DEVICE;
}

static hinm_status check_ocp_shape(const hinm_shape* shape, int32_t n_samples) {
  hinm_status st = check_shape(shape);
  if (st != HINM_OK) return st;
  if (n_samples < 1 || n_samples > shape->V) return HINM_ERR_SHAPE;
  if (shape->M / shape->V > kIcpMaxPartitions || shape->K > kOcpMaxK || shape->V > kOcpMaxV) return HINM_ERR_UNSUPPORTED;
  return HINM_OK;
}

hinm_status hinm_ocp_sizes(const hinm_shape* shape, int32_t n_samples, size_t* workspace_bytes) {
  hinm_status st = check_ocp_shape(shape, n_samples);
  if (st != HINM_OK) return st;
  if (!workspace_bytes) return HINM_ERR_NULL;
  *workspace_bytes = ocp_workspace_layout(*shape, n_samples).total_bytes;
  return HINM_OK;
}

hinm_status hinm_ocp_search(const hinm_shape* shape, const void* W, const float* rho, int32_t* row_order,
                            const int32_t* samples, const int32_t* clusters, int32_t n_samples, int32_t iters,
                            double* objective, void* workspace, size_t workspace_bytes, void* stream) {
  hinm_status st = check_ocp_shape(shape, n_samples);
  if (st != HINM_OK) return st;
  if ((!W && !rho) || !row_order || (iters > 0 && !samples)) return HINM_ERR_NULL;
  if (iters < 0) return HINM_ERR_SHAPE;
  if (!aligned(row_order, 4) || !aligned(samples, 4) || !aligned(clusters, 4) || (rho && !aligned(rho, 4)) ||
      (!rho && !aligned(W, 2)) || (objective && !aligned(objective, 8)))
    return HINM_ERR_SHAPE;
  const size_t need = ocp_workspace_layout(*shape, n_samples).total_bytes;
  if (!workspace || workspace_bytes < need || !aligned(workspace, 256)) return HINM_ERR_WORKSPACE;
  if (iters == 0) return HINM_OK;
  const OcpArgs a{*shape, W, rho, row_order, samples, clusters, n_samples, iters, objective, workspace};
  hipError_t e = launch_ocp_search(a, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? HINM_OK : HINM_ERR_DEVICE;
}

static hinm_status check_cluster_shape(const hinm_shape* shape, int32_t n_samples) {
  hinm_status st = check_ocp_shape(shape, n_samples);
  if (st != HINM_OK) return st;
  if ((int64_t)(shape->M / shape->V) * n_samples > kIcpMaxPartitions) return HINM_ERR_UNSUPPORTED;
  return HINM_OK;
}

hinm_status hinm_ocp_cluster_sizes(const hinm_shape* shape, int32_t n_samples, size_t* workspace_bytes) {
  hinm_status st = check_cluster_shape(shape, n_samples);
  if (st != HINM_OK) return st;
  if (!workspace_bytes) return HINM_ERR_NULL;
  *workspace_bytes = kmeans_workspace_layout(*shape, n_samples).total_bytes;
  return HINM_OK;
}

hinm_status hinm_ocp_cluster(const hinm_shape* shape, const void* W, const float* rho, const int32_t* row_order,
                             const int32_t* samples, int32_t n_samples, int32_t rounds, double* centroids,
                             int32_t init_centroids, int32_t* clusters, double* objective, void* workspace,
                             size_t workspace_bytes, void* stream) {
  hinm_status st = check_cluster_shape(shape, n_samples);
  if (st != HINM_OK) return st;
  if ((!W && !rho) || !row_order || !samples || !centroids || !clusters) return HINM_ERR_NULL;
  if (rounds < 1) return HINM_ERR_SHAPE;
  if (!aligned(row_order, 4) || !aligned(samples, 4) || !aligned(clusters, 4) || !aligned(centroids, 8) ||
      (rho && !aligned(rho, 4)) || (!rho && !aligned(W, 2)) || (objective && !aligned(objective, 8)))
    return HINM_ERR_SHAPE;
  const size_t need = kmeans_workspace_layout(*shape, n_samples).total_bytes;
  if (!workspace || workspace_bytes < need || !aligned(workspace, 256)) return HINM_ERR_WORKSPACE;
  const KmeansArgs a{*shape, W, rho, row_order, samples, n_samples, rounds, centroids, init_centroids != 0,
                     clusters, objective, workspace};
  hipError_t e = launch_ocp_cluster(a, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? HINM_OK : HINM_ERR_DEVICE;
}

hinm_status hinm_unpack(const hinm_shape* shape, const void* vals, const uint8_t* nm_idx, const int32_t* vec_idx,
                        void* W_out, void* stream) {
  hinm_status st = check_shape(shape);
  if (st != HINM_OK) return st;
  if (!vals || !nm_idx || !vec_idx || !W_out) return HINM_ERR_NULL;
  hipError_t e = launch_unpack(*shape, vals, nm_idx, vec_idx, W_out, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? HINM_OK : HINM_ERR_DEVICE;
}

hinm_status hinm_spmm(const hinm_shape* shape, int32_t N, const void* vals, const uint8_t* nm_idx,
                      const int32_t* vec_idx, const int32_t* pi_in, const int32_t* pi_out, const void* X, int64_t ldx,
                      void* Y, int64_t ldy, uint32_t flags, void* workspace, size_t workspace_bytes, void* stream) {
  (void)workspace;
  (void)workspace_bytes;
  hinm_status st = check_spmm(shape, N, vals, nm_idx, vec_idx, X, ldx, Y, ldy, flags);
  if (st != HINM_OK) return st;
  SpmmArgs a{*shape, N, vals, nm_idx, vec_idx, pi_in, pi_out, X, ldx, Y, ldy,
             (flags & HINM_EPI_RELU) != 0, (flags & HINM_OUT_F32) != 0};
  return run_spmm(a, flags, static_cast<hipStream_t>(stream));
}

hinm_status hinm_spmm_vectors(const hinm_shape* shape, int32_t N, const void* vals_v, const int32_t* vec_idx,
                              const int32_t* pi_in, const int32_t* pi_out, const void* X, int64_t ldx, void* Y,
                              int64_t ldy, uint32_t flags, void* stream) {
  hinm_status st = check_shape(shape);
  if (st != HINM_OK) return st;
  if (!vals_v || !vec_idx || !X || !Y) return HINM_ERR_NULL;
  if (N <= 0 || ldx < N || ldy < N) return HINM_ERR_SHAPE;
  if (N > 1 && (ldx % 8 != 0 || ldy % 8 != 0)) return HINM_ERR_SHAPE;
  if (!aligned(vals_v, 16) || !aligned(X, 16) || !aligned(Y, 16)) return HINM_ERR_SHAPE;
  if (flags & ~(uint32_t)(HINM_EPI_RELU | HINM_OUT_F32 | HINM_KERNEL_REFERENCE | HINM_VARIANT_MASK))
    return HINM_ERR_UNSUPPORTED;
  const int variant = (int)((flags & HINM_VARIANT_MASK) >> HINM_VARIANT_SHIFT);
  if (variant && (flags & HINM_KERNEL_REFERENCE)) return HINM_ERR_UNSUPPORTED;
  const VectorsArgs a{*shape, N, vals_v, vec_idx, pi_in, pi_out, X, ldx, Y, ldy,
                      (flags & HINM_EPI_RELU) != 0, (flags & HINM_OUT_F32) != 0, variant};
  hipError_t e;
  if (variant && !spmm_vectors_mfma_supported(a)) return HINM_ERR_UNSUPPORTED;  // a pinned kernel must fit the shape
  if (!(flags & HINM_KERNEL_REFERENCE) && spmm_vectors_mfma_supported(a))
    e = launch_spmm_vectors_mfma(a, static_cast<hipStream_t>(stream));
  else
    e = launch_spmm_vectors_plain(a, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? HINM_OK : HINM_ERR_DEVICE;
}

static hinm_status check_prepared_call(const hinm_shape* shape, int32_t N, const void* prepared, const void* X,
                                       int64_t ldx, const void* Y, int64_t ldy, uint32_t flags, void* workspace,
                                       size_t workspace_bytes);
static hinm_status run_prepared(const hinm_shape* shape, int32_t N, const void* prepared, const void* X, int64_t ldx,
                                void* Y, int64_t ldy, uint32_t flags, void* workspace, size_t workspace_bytes,
                                hipStream_t stream, LaunchPlan* plan);

static hinm_status check_chain(int32_t L, const hinm_layer* layers, int32_t N, size_t* bytes_per_buffer) {
  if (!layers) return HINM_ERR_NULL;
  if (L <= 0 || N <= 0) return HINM_ERR_SHAPE;
  size_t widest = 0;
  for (int l = 0; l < L; ++l) {
    hinm_status st = check_shape(&layers[l].shape);
    if (st != HINM_OK) return st;
    if (!layers[l].prepared && (!layers[l].vals || !layers[l].nm_idx || !layers[l].vec_idx)) return HINM_ERR_NULL;
    if (layers[l].shape.dtype != layers[0].shape.dtype) return HINM_ERR_DTYPE;
    if (l > 0 && layers[l].shape.K != layers[l - 1].shape.M) return HINM_ERR_SHAPE;
    if (l + 1 < L && (layers[l].flags & HINM_OUT_F32)) return HINM_ERR_UNSUPPORTED;
    if (l + 1 < L) {
      const size_t b = (size_t)layers[l].shape.M * (size_t)((N + 7) / 8 * 8) * 2;
      widest = b > widest ? b : widest;
    }
  }
  *bytes_per_buffer = (widest + 255) / 256 * 256;
  return HINM_OK;
}

hinm_status hinm_chain_sizes(int32_t L, const hinm_layer* layers, int32_t N, size_t* scratch_bytes) {
  if (!scratch_bytes) return HINM_ERR_NULL;
  size_t per = 0;
  hinm_status st = check_chain(L, layers, N, &per);
  if (st != HINM_OK) return st;
  *scratch_bytes = (L <= 1) ? 0 : (L == 2 ? per : 2 * per);
  return HINM_OK;
}

hinm_status hinm_chain(int32_t L, const hinm_layer* layers, int32_t N, const void* X, int64_t ldx, void* Y,
                       int64_t ldy, void* scratch, size_t scratch_bytes, void* stream) {
  size_t per = 0;
  hinm_status st = check_chain(L, layers, N, &per);
  if (st != HINM_OK) return st;
  if (!X || !Y) return HINM_ERR_NULL;
  const size_t need = (L <= 1) ? 0 : (L == 2 ? per : 2 * per);
  if (need > 0 && (!scratch || scratch_bytes < need || !aligned(scratch, 256))) return HINM_ERR_WORKSPACE;
  const int64_t ldh = (N + 7) / 8 * 8;
  // validate every layer's call before launching the first one
  for (int l = 0; l < L; ++l) {
    const void* in = (l == 0) ? X : scratch;
    void* out = (l == L - 1) ? Y : scratch;
    if (layers[l].prepared)
      st = check_prepared_call(&layers[l].shape, N, layers[l].prepared, in, l == 0 ? ldx : ldh, out,
                               l == L - 1 ? ldy : ldh, layers[l].flags, nullptr, 0);
    else
      st = check_spmm(&layers[l].shape, N, layers[l].vals, layers[l].nm_idx, layers[l].vec_idx, in,
                      l == 0 ? ldx : ldh, out, l == L - 1 ? ldy : ldh, layers[l].flags);
    if (st != HINM_OK) return st;
  }
  char* buf[2] = {static_cast<char*>(scratch), static_cast<char*>(scratch) + per};
  const void* in = X;
  int64_t ld_in = ldx;
  for (int l = 0; l < L; ++l) {
    const bool last = (l == L - 1);
    void* out = last ? Y : static_cast<void*>(buf[l & 1]);
    const int64_t ld_out = last ? ldy : ldh;
    const hinm_layer& ly = layers[l];
    if (ly.prepared) {
      st = run_prepared(&ly.shape, N, ly.prepared, in, ld_in, out, ld_out, ly.flags, nullptr, 0,
                        static_cast<hipStream_t>(stream), nullptr);
    } else {
      SpmmArgs a{ly.shape, N, ly.vals, ly.nm_idx, ly.vec_idx, ly.pi_in, ly.pi_out, in, ld_in, out, ld_out,
                 (ly.flags & HINM_EPI_RELU) != 0, (ly.flags & HINM_OUT_F32) != 0};
      st = run_spmm(a, ly.flags, static_cast<hipStream_t>(stream));
    }
    if (st != HINM_OK) return st;
    in = out;
    ld_in = ld_out;
  }
  return HINM_OK;
}


hinm_status hinm_prepare_sizes(const hinm_shape* shape, size_t* prepared_bytes) {
  hinm_status st = check_shape(shape);
  if (st != HINM_OK) return st;
  if (!prepared_bytes) return HINM_ERR_NULL;
  if (shape->V % 32 != 0 || shape->V > 128) return HINM_ERR_UNSUPPORTED;
  *prepared_bytes = prepared_layout(*shape).total_bytes;
  return HINM_OK;
}

hinm_status hinm_prepare(const hinm_shape* shape, const void* vals, const uint8_t* nm_idx, const int32_t* vec_idx,
                         const int32_t* pi_in, const int32_t* pi_out, void* prepared, size_t prepared_bytes,
                         void* stream) {
  size_t need = 0;
  hinm_status st = hinm_prepare_sizes(shape, &need);
  if (st != HINM_OK) return st;
  if (!vals || !nm_idx || !vec_idx || !prepared) return HINM_ERR_NULL;
  if (prepared_bytes < need || !aligned(prepared, 256)) return HINM_ERR_WORKSPACE;
  hipError_t e = launch_prepare(*shape, vals, nm_idx, vec_idx, pi_in, pi_out, prepared,
                                static_cast<hipStream_t>(stream));
  return e == hipSuccess ? HINM_OK : HINM_ERR_DEVICE;
}

hinm_status hinm_spmm_prepared_workspace(const hinm_shape* shape, int32_t N, size_t* workspace_bytes) {
  size_t need = 0;
  hinm_status st = hinm_prepare_sizes(shape, &need);
  if (st != HINM_OK) return st;
  if (!workspace_bytes) return HINM_ERR_NULL;
  if (N <= 0) return HINM_ERR_SHAPE;
  *workspace_bytes = (N <= 32) ? skinny_prepared_workspace_bytes(*shape, N) : 0;
  return HINM_OK;
}

// Which kernel family a prepared call runs on; everything that can make the call fail is decided here, on the
// host, before anything is launched (hinm_chain validates every layer with it before its first launch).
enum class PreparedRoute { Rows16, Skinny, Panel, Tile };

static PreparedArgs prepared_args(const hinm_shape* shape, int32_t N, const void* prepared, const void* X, int64_t ldx,
                                  void* Y, int64_t ldy, uint32_t flags, void* workspace, size_t workspace_bytes) {
  return PreparedArgs{*shape, N, prepared, X, ldx, Y, ldy, (flags & HINM_EPI_RELU) != 0, (flags & HINM_OUT_F32) != 0,
                      (int)((flags & HINM_VARIANT_MASK) >> HINM_VARIANT_SHIFT), workspace, workspace_bytes};
}

static hinm_status route_prepared(const PreparedArgs& a, PreparedRoute* route) {
  const hinm_shape* shape = &a.s;
  const int32_t N = a.N;
  // up to 16 columns: 16-row workgroups on the 16x16x64 form (measured faster than the 32-row kernel on every
  // decode shape tried, by 8-10 % with 344 row blocks of 32 and by 15-37 % with 128); variant 11 pins it for any N, 19 its form with
  // the input rows resident in LDS (16 columns only)
  if (a.tile_variant == 19 && !spmm_rows16_resident_supported(a)) return HINM_ERR_UNSUPPORTED;
  // ... and for up to 64 columns on every layer tried (one workgroup per 16..64 rows and 16 columns re-reads
  // the weights for every column block and still wins: 11008 x 4096 at N = 64 23 vs 40 us, 1024 x 4096 6 vs
  // 33 us), and up to 2048 columns while its cost, which grows with M * Kv * ceil(N / 16), stays under the tile
  // kernels' floor of one serial pass over the kept columns (about 15 us per 1024 of them, a little more per
  // column on short passes): layers whose tiles cannot fill the chip.  The constants are fitted to timings of
  // 42 (layer, N) pairs between 512 x 4608 and 8192 x 8192 and checked on some 250 more at other N.
  bool few_columns = N <= 64;
  if (!few_columns && N <= 2048) {
    const double units = (double)shape->M * ((N + 15) / 16);
    // the tile kernels' pass: 15 us per 1024 kept columns (12 with tiles of up to 64 rows: smaller stages,
    // 128-column stages where the step count is even), and on short passes 2 us more, 4 with 128-row tiles
    const double tile_floor_us =
        shape->V >= 96 ? 1.0 + 15.0 * shape->Kv / 1024.0 + (shape->Kv <= 1024 ? (shape->V >= 128 ? 4.0 : 2.0) : 0.0)
                       : 2.0 + 12.0 * shape->Kv / 1024.0 + (shape->Kv <= 1024 ? 2.0 : 0.0);
    // with two column blocks per workgroup the 16-row kernel measured 19-34 % faster, with four as much again
    const int blocks_per_wg = spmm_rows16_prepared_blocks_per_wg(a);
    const double pair_factor = blocks_per_wg == 4 ? 0.58 : blocks_per_wg == 2 ? 0.78 : 1.0;
    // beyond 512 columns X (K x N) often outgrows one L2 and the gathers slow down, those that use a quarter
    // or half of each cache line first (measured on small layers up to N = 4096: the kernel still wins to
    // 1024..2048 columns on layers of a few hundred rows)
    const bool x_beyond_l2 = (double)shape->K * N * 2 > 3.5e6;
    const double l2_factor = !x_beyond_l2 ? 1.0 : N > 1024 ? 2.0 : (N > 512 && blocks_per_wg < 4) ? 1.5 : 1.0;
    few_columns = 2.5 + units * (0.14 * shape->Kv + 40.0) * 1e-6 * l2_factor * pair_factor < tile_floor_us;
  }
  if (a.tile_variant == 11 || a.tile_variant == 19 || (a.tile_variant == 0 && few_columns)) {
    if ((N + 15) / 16 > 65535) return HINM_ERR_UNSUPPORTED;
    *route = PreparedRoute::Rows16;
  } else if (N <= 32 && (a.tile_variant == 0 || a.tile_variant == 12)) {  // variant 12 pins the 32-row skinny kernel
    const size_t need = skinny_prepared_workspace_bytes(*shape, N);
    if (need > 0 && (!a.workspace || a.workspace_bytes < need || !aligned(a.workspace, 256)))
      return HINM_ERR_WORKSPACE;
    *route = PreparedRoute::Skinny;
  } else {
    if (N == 1 || a.ldx % 8 != 0 || a.ldy % 8 != 0 || a.tile_variant == 12) return HINM_ERR_UNSUPPORTED;
    const bool panel = (a.tile_variant == 15) || (a.tile_variant == 0 && spmm_panel_prepared_preferred(a));
    if (panel && !spmm_panel_prepared_supported(a)) return HINM_ERR_UNSUPPORTED;
    *route = panel ? PreparedRoute::Panel : PreparedRoute::Tile;
  }
  return HINM_OK;
}

static hinm_status check_prepared_call(const hinm_shape* shape, int32_t N, const void* prepared, const void* X,
                                       int64_t ldx, const void* Y, int64_t ldy, uint32_t flags, void* workspace,
                                       size_t workspace_bytes) {
  size_t need = 0;
  hinm_status st = hinm_prepare_sizes(shape, &need);
  if (st != HINM_OK) return st;
  if (!prepared || !X || !Y) return HINM_ERR_NULL;
  if (N <= 0 || ldx < N || ldy < N) return HINM_ERR_SHAPE;
  if (N > 1 && (ldx % 8 != 0 || ldy % 8 != 0)) return HINM_ERR_SHAPE;
  if (!aligned(prepared, 256) || !aligned(X, 16) || !aligned(Y, 16)) return HINM_ERR_SHAPE;
  if (flags & ~(uint32_t)(HINM_EPI_RELU | HINM_OUT_F32 | HINM_VARIANT_MASK)) return HINM_ERR_UNSUPPORTED;
  PreparedRoute route;
  return route_prepared(prepared_args(shape, N, prepared, X, ldx, const_cast<void*>(Y), ldy, flags, workspace,
                                      workspace_bytes), &route);
}

// The call has passed check_prepared_call.
static hinm_status run_prepared(const hinm_shape* shape, int32_t N, const void* prepared, const void* X, int64_t ldx,
                                void* Y, int64_t ldy, uint32_t flags, void* workspace, size_t workspace_bytes,
                                hipStream_t stream, LaunchPlan* plan) {
  PreparedArgs a = prepared_args(shape, N, prepared, X, ldx, Y, ldy, flags, workspace, workspace_bytes);
  a.plan = plan;
  PreparedRoute route;
  hinm_status st = route_prepared(a, &route);
  if (st != HINM_OK) return st;
  hipError_t e = hipSuccess;
  switch (route) {
    case PreparedRoute::Rows16: e = launch_spmm_rows16_prepared(a, stream); break;
    case PreparedRoute::Skinny: e = launch_spmm_skinny_prepared(a, stream); break;
    case PreparedRoute::Panel: e = launch_spmm_panel_prepared(a, stream); break;
    case PreparedRoute::Tile: e = launch_spmm_tile_prepared(a, stream); break;
  }
  return e == hipSuccess ? HINM_OK : HINM_ERR_DEVICE;
}

hinm_status hinm_spmm_prepared(const hinm_shape* shape, int32_t N, const void* prepared, const void* X, int64_t ldx,
                               void* Y, int64_t ldy, uint32_t flags, void* workspace, size_t workspace_bytes,
                               void* stream) {
  hinm_status st = check_prepared_call(shape, N, prepared, X, ldx, Y, ldy, flags, workspace, workspace_bytes);
  if (st != HINM_OK) return st;
  return run_prepared(shape, N, prepared, X, ldx, Y, ldy, flags, workspace, workspace_bytes,
                      static_cast<hipStream_t>(stream), nullptr);
}

hinm_status hinm_spmm_prepared_plan(const hinm_shape* shape, int32_t N, int64_t ldx, int64_t ldy, uint32_t flags,
                                    char* text, size_t text_bytes, int32_t* launches) {
  if (!text || text_bytes == 0) return HINM_ERR_NULL;
  text[0] = 0;
  // stand-ins with the alignment of real buffers: a dry run dereferences nothing
  void* const fake = reinterpret_cast<void*>(uintptr_t{1} << 20);
  hinm_status st = check_prepared_call(shape, N, fake, fake, ldx, fake, ldy, flags, fake, ~size_t{0});
  if (st != HINM_OK) return st;
  LaunchPlan plan{text, text_bytes};
  st = run_prepared(shape, N, fake, fake, ldx, fake, ldy, flags, fake, ~size_t{0}, nullptr, &plan);
  if (launches) *launches = plan.launches;
  return st;
}

hinm_status hinm_calib_tile_part(const hinm_shape* shape, int32_t N, const void* prepared, const void* X, int64_t ldx,
                                 int32_t part, void* stream) {
  // Y is never written: any aligned non-NULL stand-in passes the checks
  void* const no_y = reinterpret_cast<void*>(uintptr_t{1} << 20);
  hinm_status st = check_prepared_call(shape, N, prepared, X, ldx, no_y, (N + 7) / 8 * 8, 0, nullptr, 0);
  if (st != HINM_OK) return st;
  if (part != 1 && part != 2) return HINM_ERR_UNSUPPORTED;
  PreparedArgs a = prepared_args(shape, N, prepared, X, ldx, no_y, (N + 7) / 8 * 8, 0, nullptr, 0);
  PreparedRoute route;
  st = route_prepared(a, &route);
  if (st != HINM_OK) return st;
  if (route != PreparedRoute::Tile) return HINM_ERR_UNSUPPORTED;
  hipError_t e = launch_spmm_tile_prepared_part(a, part, static_cast<hipStream_t>(stream));
  if (e == hipErrorNotSupported) return HINM_ERR_UNSUPPORTED;
  return e == hipSuccess ? HINM_OK : HINM_ERR_DEVICE;
}

const char* hinm_status_str(hinm_status s) {
  switch (s) {
    case HINM_OK: return "ok";
    case HINM_ERR_NULL: return "null pointer argument";
    case HINM_ERR_SHAPE: return "invalid shape, leading dimension or alignment";
    case HINM_ERR_DTYPE: return "unsupported dtype";
    case HINM_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case HINM_ERR_UNSUPPORTED: return "request not supported by this build";
    case HINM_ERR_DEVICE: return "HIP launch failed";
  }
  return "unknown status";
}

int32_t hinm_version(void) { return 1000 * 0 + 1; }

}  // extern "C"
