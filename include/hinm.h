/*
 * hinm.h -- C ABI of the HiNM sparse-GEMM library for AMD MI355X (gfx950).
 *
 * Hierarchical N:M (HiNM) sparsity, arXiv 2407.20496:
 *   Section 1 (Figure 1): a dense weight matrix W (M output channels x K input
 *   channels) is pruned in two levels.  Inside every tile of V consecutive
 *   output channels whole V x 1 column vectors are removed until Kv of the K
 *   columns survive; the surviving columns are listed in the tile's *vector
 *   index*.  Then every row of the tile is pruned 2:4 over consecutive groups
 *   of four surviving columns; the two kept positions of each group form the
 *   *NM index*, and the kept values are stored densely.
 *   Section 3.2 / Section 5.3: at run time the product reads only the input
 *   rows named by the vector index, and channel re-ordering is absorbed into
 *   that indexing, so each layer may use its own input- and output-channel
 *   order with no separate permute pass:
 *         Y = P_out ( W_HiNM ( P_in X ) ).
 *
 * Conventions shared by all entry points
 *   - Row-major matrices.  W is M x K, X is K x N (leading dimension ldx
 *     elements), Y is M x N (leading dimension ldy elements).
 *   - T = M / V tiles.  Kv kept columns per tile; Kv/2 stored values per row.
 *   - Canonical packed form (what parity is judged on):
 *       vals    16-bit values  [M][Kv/2]  for group g of row r: the two kept
 *                                         values in ascending position order
 *                                         at [r][2g], [r][2g+1] (bit copies of W)
 *       nm_idx  uint8          [M][Kv/8]  nibble of group g = p0 | (p1 << 2),
 *                                         p0 < p1 the kept positions (0..3);
 *                                         group g sits in byte g/2, bits
 *                                         4*(g&1) .. 4*(g&1)+3
 *       vec_idx int32          [T][Kv]    surviving columns of tile t, ascending
 *                                         (hinm_pack) or in a caller-given order
 *                                         (hinm_pack_ordered); group g covers
 *                                         entries 4g .. 4g+3
 *   - Channel orders: pi_in is int32[K], row k of (P_in X) is row pi_in[k] of X
 *     (gather); pi_out is int32[M], row r of W_HiNM(P_in X) is written to row
 *     pi_out[r] of Y (scatter).  NULL means identity.  They are not checked
 *     for being bijections; entries must lie in [0,K) resp. [0,M).
 *   - Selection rules of hinm_pack: vector saliency = sum of squares of the V
 *     entries, accumulated in IEEE binary64 in ascending row order; the Kv
 *     largest survive, equal scores -> lower column.  2:4 saliency = |w|
 *     (compared on the 15 magnitude bits), equal -> lower position; always
 *     exactly two survivors per group, explicit zeros included.
 *   - Pointers: `hinm_shape` / `hinm_layer` arguments are HOST memory, read
 *     during the call only.  Every other pointer is DEVICE memory owned by the
 *     caller; the library allocates nothing, keeps no reference after the
 *     work is enqueued, and the caller keeps buffers alive until `stream`
 *     (a hipStream_t, NULL = the default stream) has passed that work.
 *     All work is asynchronous on `stream`; no entry point synchronises.
 *   - Errors: a status code is returned; argument errors are detected on the
 *     host before anything is launched (so they can be tested without a GPU).
 *     HINM_ERR_DEVICE reports a failed launch.  W must be finite.
 *   - Alignment: vals, X and Y base pointers 16-byte aligned; ldx, ldy
 *     multiples of 8 elements unless N == 1 (then any ld >= 1).
 *   - Readable extent of X: the kernels load X in 16-byte pieces, so for N > 1 every row is read up to
 *     column 8 * ceil(N / 8) - 1, the last row included: X must be readable for
 *     (K - 1) * ldx + 8 * ceil(N / 8) elements (ldx >= that rounded N guarantees it for an allocation of
 *     K * ldx elements).  What those extra columns hold never reaches a result.
 *   - HIP stream capture: the library records kernel launches only (no memset, copy, allocation or
 *     synchronisation).  The first launch of a kernel on a device may raise that kernel's dynamic-LDS
 *     limit (a function attribute, set once per device): make one un-captured call of the same entry
 *     point with the same shape on that device before capturing it.
 */
#ifndef HINM_H
#define HINM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  HINM_OK = 0,
  HINM_ERR_NULL = 1,        /* a required pointer is NULL */
  HINM_ERR_SHAPE = 2,       /* M % V != 0, Kv % 8 != 0, Kv > K, non-positive size, bad ld / alignment */
  HINM_ERR_DTYPE = 3,       /* dtype is neither HINM_F16 nor HINM_BF16 */
  HINM_ERR_WORKSPACE = 4,   /* workspace / scratch missing or too small */
  HINM_ERR_UNSUPPORTED = 5, /* valid request this build has no kernel for (e.g. forced kernel vs. shape) */
  HINM_ERR_DEVICE = 6       /* HIP reported an error at launch */
} hinm_status;

typedef enum { HINM_F16 = 0, HINM_BF16 = 1 } hinm_dtype;

/* flags of hinm_spmm / hinm_layer (bit-or) */
enum {
  HINM_EPI_RELU = 1u,         /* y = max(y, 0) before rounding (used between chained layers) */
  HINM_OUT_F32 = 2u,          /* Y is float32 [M][N]: the un-rounded accumulators (verification mode) */
  /* kernel choice; default (none set) picks by shape */
  HINM_KERNEL_REFERENCE = 0x100u, /* one thread per output element, plain FMA; any V */
  HINM_KERNEL_SMFMAC = 0x200u,    /* a sparse-MFMA kernel: 32x32 tiles (V in {32,64,96,128}, Kv % 32 == 0,
                                     ld % 8 == 0) or else the 16-column form (V % 16 == 0) */
  HINM_KERNEL_GEMV = 0x400u,      /* 16-column sparse-MFMA form with k split over the waves; N <= 16, V % 16 == 0 */
  /* hinm_spmm_prepared and hinm_spmm_vectors only, tuning aid: bits 16..21 pin one kernel configuration
   * (0 = by shape); a configuration that does not fit the shape returns HINM_ERR_UNSUPPORTED */
  HINM_VARIANT_SHIFT = 16,
  HINM_VARIANT_MASK = 0x3F0000u
};

typedef struct {
  int32_t M;     /* output channels (rows of W) */
  int32_t K;     /* input channels (columns of W) */
  int32_t V;     /* vector height = rows per tile; M % V == 0 */
  int32_t Kv;    /* surviving columns per tile; 0 < Kv <= K, Kv % 8 == 0 */
  int32_t dtype; /* hinm_dtype of W, vals, X and (unless HINM_OUT_F32) Y */
} hinm_shape;

/* Size in bytes of the three packed arrays and of hinm_pack's workspace
 * (one binary64 score per tile and column).  Any output pointer may be NULL. */
hinm_status hinm_pack_sizes(const hinm_shape* shape, size_t* vals_bytes, size_t* nm_bytes,
                            size_t* vec_bytes, size_t* workspace_bytes);

/* Section 1 / Section 3.1: dense W [M][K] -> canonical packed arrays, on the
 * GPU, following the selection rules above.  `workspace` needs
 * workspace_bytes from hinm_pack_sizes and 8-byte alignment. */
hinm_status hinm_pack(const hinm_shape* shape, const void* W,
                      void* vals, uint8_t* nm_idx, int32_t* vec_idx,
                      void* workspace, size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory or pass a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): hinm_pack with its score workspace in a
 * device array that is part of the library image.  Same inputs, outputs, selection rules and
 * results (bit for bit) as hinm_pack.  Limit: (M / V) * K <= HINM_PACK_STATIC_MAX_SCORES (one binary64
 * score per tile and column, 4 MiB per GPU, held from the library's load until the process ends);
 * larger layers return HINM_ERR_WORKSPACE before anything is launched.  The call allocates and
 * frees nothing and records kernel launches only.  All calls on one GPU share the one array: two
 * calls whose kernels may overlap there (different streams, no ordering between them) race and
 * give unspecified packed arrays; calls on one stream, or ordered by events, are safe.  Nothing in
 * the array has to be cleared between calls (every score that is read was written by the same
 * call).  The first call on a device looks up the array's address and, like every entry point of
 * this library, may set a kernel attribute: make one call per device outside stream capture first. */
#define HINM_PACK_STATIC_MAX_SCORES 524288
hinm_status hinm_pack_static(const hinm_shape* shape, const void* W,
                             void* vals, uint8_t* nm_idx, int32_t* vec_idx, void* stream);

/* Section 3.2 ("tile-wise input channel permutation"; the per-tile orders sigma_i^t of Section 4.2):
 * hinm_pack with a caller-given order of the kept column vectors.  tile_order is int32 [T][K] in
 * device memory, row t a permutation of the input channels 0..K-1; the surviving columns of tile t
 * (chosen exactly as by hinm_pack) are written to vec_idx in the order in which they appear in
 * that row instead of ascending, and every four consecutive ones form a 2:4 group.  The product
 * kernels need nothing else: they follow vec_idx.  tile_order == NULL is hinm_pack.  The rows are
 * not checked for being permutations: entries outside [0,K) are skipped, and a row that is not a
 * permutation leaves an unspecified vector index whose entries are surviving columns of the tile.
 * K above 393216 returns HINM_ERR_UNSUPPORTED.  Workspace as for hinm_pack. */
hinm_status hinm_pack_ordered(const hinm_shape* shape, const void* W, const int32_t* tile_order,
                              void* vals, uint8_t* nm_idx, int32_t* vec_idx,
                              void* workspace, size_t workspace_bytes, void* stream);

/* Section 4.2 (the output-channel search ends in an order of the output channels; Section 3.2: that
 * order is applied offline, to the rows of the weight matrix, before the layer is packed):
 * dst row r = src row row_order[r], for matrices of `rows` rows of row_bytes bytes each (the weights,
 * and a caller's saliency matrix alike; row_bytes a multiple of 4), all in device memory, src and dst
 * distinct and not overlapping.  row_order is int32 [rows]; it is not checked for being a
 * permutation: a destination row whose entry is outside [0, rows) is left unwritten. */
hinm_status hinm_apply_row_order(const void* src, void* dst, const int32_t* row_order, int32_t rows,
                                 size_t row_bytes, void* stream);

/* Section 3.2 (every arrangement of a tile's kept vectors is a valid layer; Section 4.2 searches over
 * them): the order of all K input channels that makes hinm_pack_ordered / hinm_pack_scored /
 * hinm_pack_vectors reproduce a given arrangement.  vec_idx is int32 [T][Kv] in device memory, row t
 * the kept channels of tile t in some arrangement (as hinm_icp_search leaves them); tile_order,
 * int32 [T][K] in device memory, receives for every tile those Kv channels in that arrangement
 * followed by the remaining K - Kv channels in ascending order.  Rows of vec_idx are not checked:
 * entries outside [0,K) are copied as they are, and a row with repeated or out-of-range entries
 * gives a row of tile_order that is not a permutation (hinm_pack_ordered tolerates that).  K above
 * 393216 returns HINM_ERR_UNSUPPORTED.  No workspace. */
hinm_status hinm_tile_order(const hinm_shape* shape, const int32_t* vec_idx, int32_t* tile_order, void* stream);

/* Section 4.1 (the saliency rho of Eq. 1-3; Section 5.1 names magnitude and second-order scores):
 * hinm_pack with caller-given scores.  rho is float32 [M][K] in device memory, one score per
 * weight, free of NaN.  Vector saliency = the sum of the V scores of the vector, accumulated in
 * IEEE binary64 in ascending row order starting from +0; the Kv largest sums survive (signed
 * comparison), equal sums -> lower column.  Inside every group of four surviving entries the two
 * largest scores are kept (signed comparison, -0 equals +0), equal -> lower position.  vals holds
 * bit copies of W at the kept places, as in hinm_pack.  tile_order as in hinm_pack_ordered, or
 * NULL.  Workspace as for hinm_pack. */
hinm_status hinm_pack_scored(const hinm_shape* shape, const void* W, const float* rho,
                             const int32_t* tile_order,
                             void* vals, uint8_t* nm_idx, int32_t* vec_idx,
                             void* workspace, size_t workspace_bytes, void* stream);

/* Section 3.1 (first step) / Section 5.1.2 (gradual pruning keeps a layer in this state until the
 * target vector sparsity is reached): column-vector pruning alone, no 2:4 step.  vals_v is
 * 16-bit [M][Kv] in device memory, 16-byte aligned: vals_v[r][j] = W[r][vec_idx[r / V][j]], a
 * bit copy; vec_idx as written by hinm_pack.  rho (as in hinm_pack_scored) and tile_order (as in
 * hinm_pack_ordered) may each be NULL.  Applying 2:4 to every four consecutive entries of a row of
 * vals_v gives what hinm_pack stores.  Workspace as for hinm_pack. */
hinm_status hinm_pack_vectors(const hinm_shape* shape, const void* W, const float* rho,
                              const int32_t* tile_order,
                              void* vals_v, int32_t* vec_idx,
                              void* workspace, size_t workspace_bytes, void* stream);

/* Section 4.1 (Eq. 3) / Section 4.2: tile-wise input-channel permutation search of gyro-permutation.
 * Re-arranges the kept column vectors of every tile (vec_idx, int32 [T][Kv] as written by hinm_pack,
 * hinm_pack_scored or hinm_pack_vectors; updated in place) so that the 2:4 step over every four
 * consecutive ones (one partition) prunes less saliency.  Saliency of an entry: rho (float32 [M][K],
 * as in hinm_pack_scored), or |w| when rho is NULL (then W, 16-bit [M][K], must be given).  One
 * iteration per tile: one vector leaves every partition -- samples, uint8 [iters][T][Kv/4] in device
 * memory, names the member (0..3, only the two low bits are read) and is drawn by the caller --;
 * cost[i][j] (Eq. 4) = the saliency 2:4 would prune in partition i with sample j in the vacated slot
 * (per row the two smallest of the four values, rows added in IEEE binary64 in ascending order); the
 * samples are assigned to the partitions at minimal total cost (an exact linear-assignment solver;
 * when several assignments reach the minimum, which one is taken is unspecified); every sample moves
 * into the slot its partition vacated.  objective, double [iters][T] or NULL, receives that minimal
 * total cost = the saliency the 2:4 step prunes in the tile after the iteration; it never increases.
 * The result is a re-ordering of each row of vec_idx; hand it to hinm_pack_ordered /
 * hinm_pack_scored as a tile order (followed by the pruned channels in any order) to pack with it.
 * Kv above 4096 returns HINM_ERR_UNSUPPORTED.  workspace: hinm_icp_sizes bytes, 256-byte aligned.
 * iters == 0 does nothing. */
hinm_status hinm_icp_sizes(const hinm_shape* shape, size_t* workspace_bytes);
hinm_status hinm_icp_search(const hinm_shape* shape, const void* W, const float* rho,
                            int32_t* vec_idx, const uint8_t* samples, int32_t iters,
                            double* objective,
                            void* workspace, size_t workspace_bytes, void* stream);

/* Section 4.1 (Eq. 2) / Section 4.2: output-channel permutation search of gyro-permutation.
 * Re-distributes the output channels over the tiles so that column-vector pruning (keep the Kv
 * columns of largest summed saliency per tile) removes less saliency.  row_order, int32 [M] in device
 * memory, updated in place: row_order[t V + p] = the channel (row of W / rho) at position p of tile
 * t; start from 0..M-1.  Saliency as in hinm_icp_search (rho, or |w| when rho is NULL).  One
 * iteration: n_samples channels leave every tile -- samples, int32 [iters][T][n_samples], distinct
 * positions 0..V-1, drawn by the caller --; the T n_samples sampled channels (item q = sample
 * q % n_samples of tile q / n_samples) are grouped into T clusters -- clusters, int32
 * [iters][T][n_samples], a permutation of the items, computed by the caller (the paper uses balanced
 * K-means), or NULL = every tile's own samples --; cost[i][j] (Eq. 4) = the saliency vector pruning
 * would remove from tile i's remaining channels plus cluster j (sum of the K - Kv smallest column
 * scores, binary64); clusters are assigned to tiles at minimal total cost; the channels of the
 * assigned cluster fill the vacated positions in order.  objective, double [iters] or NULL: that
 * minimal total cost.  Apply the result by packing the rows of W in this order (and composing pi_out
 * with it).  Entries of samples, clusters and row_order are not checked; out-of-range values are
 * clamped into range, which gives a meaningless order.  T above 1024, K above 16384 or V above 4096
 * return HINM_ERR_UNSUPPORTED.  workspace: hinm_ocp_sizes bytes, 256-byte aligned. */
hinm_status hinm_ocp_sizes(const hinm_shape* shape, int32_t n_samples, size_t* workspace_bytes);
hinm_status hinm_ocp_search(const hinm_shape* shape, const void* W, const float* rho,
                            int32_t* row_order, const int32_t* samples, const int32_t* clusters,
                            int32_t n_samples, int32_t iters, double* objective,
                            void* workspace, size_t workspace_bytes, void* stream);

/* Section 4.2, clustering phase of the output-channel search.  The paper names balanced K-means
 * and gives no detail; this entry point implements one reading, stated here in full.  Points: the
 * T n_samples channels sampled for one iteration (row_order and samples [T][n_samples] as for
 * hinm_ocp_search; item q = sample q % n_samples of tile q / n_samples), features: their saliency rows
 * (rho, or |w|).  T clusters of exactly n_samples points.  A round: squared Euclidean distance of
 * every point to every centroid in IEEE binary64 (columns added in ascending order, product and sum
 * rounded separately); the points are assigned to the clusters at minimal total distance under the
 * size constraint (an exact linear assignment of the points to the (cluster, slot) pairs; which of
 * several minimal assignments is taken is unspecified); every centroid becomes the sum of its
 * members' features in ascending item order, divided by n_samples.  centroids, double [T][K] in
 * device memory, in/out: with init_centroids != 0 they first become the features of the first sample
 * of every tile.  clusters, int32 [T][n_samples] out: the items of every cluster in ascending order,
 * the `clusters` argument of hinm_ocp_search.  objective, double [rounds] or NULL: the total distance
 * reached by each round's assignment; it never increases.  rounds >= 1.  T * n_samples above 1024
 * returns HINM_ERR_UNSUPPORTED (as do the limits of hinm_ocp_search).  workspace:
 * hinm_ocp_cluster_sizes bytes, 256-byte aligned. */
hinm_status hinm_ocp_cluster_sizes(const hinm_shape* shape, int32_t n_samples, size_t* workspace_bytes);
hinm_status hinm_ocp_cluster(const hinm_shape* shape, const void* W, const float* rho,
                             const int32_t* row_order, const int32_t* samples, int32_t n_samples,
                             int32_t rounds, double* centroids, int32_t init_centroids,
                             int32_t* clusters, double* objective,
                             void* workspace, size_t workspace_bytes, void* stream);

/* Inverse of hinm_pack: W_out [M][K] = W_HiNM (zeros where pruned).
 * W_out is fully overwritten. */
hinm_status hinm_unpack(const hinm_shape* shape, const void* vals, const uint8_t* nm_idx,
                        const int32_t* vec_idx, void* W_out, void* stream);

/* Section 3.2 / Section 5.3: Y = P_out ( W_HiNM ( P_in X ) ), fp32 accumulation,
 * output rounded to nearest-even in the storage type (or written as float32
 * with HINM_OUT_F32).  Input rows are fetched through vec_idx composed with
 * pi_in; output rows are stored through pi_out.  N >= 1.  X and Y must not
 * overlap.  workspace may be NULL (no kernel of this build needs one). */
hinm_status hinm_spmm(const hinm_shape* shape, int32_t N,
                      const void* vals, const uint8_t* nm_idx, const int32_t* vec_idx,
                      const int32_t* pi_in, const int32_t* pi_out,
                      const void* X, int64_t ldx, void* Y, int64_t ldy,
                      uint32_t flags, void* workspace, size_t workspace_bytes, void* stream);

/* Section 5.1.2 (a layer of a gradually pruned model before its 2:4 step) with the channel orders
 * of Section 3.2 / Section 5.3:
 *     Y[pi_out[r]][n] = sum_j vals_v[r][j] * X[pi_in[vec_idx[r / V][j]]][n],
 * vals_v and vec_idx as written by hinm_pack_vectors (vals_v 16-byte aligned).  fp32 accumulation,
 * rounding, pi_in / pi_out, ldx / ldy and alignment rules as for hinm_spmm.  flags: HINM_EPI_RELU,
 * HINM_OUT_F32, HINM_KERNEL_REFERENCE (one thread per output element), the variant bits (1 =
 * register-staged tile kernel, 2 / 3 = direct-to-LDS tile kernel with 256- / 512-column blocks,
 * 4 / 5 = the same with twice as many waves of half the width; 2..5 need Kv % 64 == 0); anything else returns HINM_ERR_UNSUPPORTED.  V in {32, 64, 96, 128}
 * with N > 1 runs on the dense MFMA, other shapes on the plain kernel.  Needs no workspace. */
hinm_status hinm_spmm_vectors(const hinm_shape* shape, int32_t N,
                              const void* vals_v, const int32_t* vec_idx,
                              const int32_t* pi_in, const int32_t* pi_out,
                              const void* X, int64_t ldx, void* Y, int64_t ldy,
                              uint32_t flags, void* stream);

/* ---- device-tuned form -----------------------------------------------------------------------
 * Section 3.2 settles every layer's channel orders offline and rewrites the vector indices
 * accordingly, so that at run time the kernel follows a single index per input row.
 * hinm_prepare does that rewriting once per layer, on the GPU: it composes the vector index
 * with pi_in into a gather table, keeps pi_out, and re-orders the stored values and NM nibbles into
 * the lane order of the sparse-MFMA operands so that the kernels stream them with full-width
 * contiguous loads.  The result is an opaque buffer (a pure re-ordering of the canonical arrays
 * plus the two permutations; parity is judged on the canonical arrays and on the products).
 * Needs V % 32 == 0 (HINM_ERR_UNSUPPORTED otherwise: use hinm_spmm).  `prepared` is 256-byte
 * aligned device memory of hinm_prepare_sizes bytes; it must stay unchanged while products that
 * use it are in flight. */
hinm_status hinm_prepare_sizes(const hinm_shape* shape, size_t* prepared_bytes);
hinm_status hinm_prepare(const hinm_shape* shape, const void* vals, const uint8_t* nm_idx,
                         const int32_t* vec_idx, const int32_t* pi_in, const int32_t* pi_out,
                         void* prepared, size_t prepared_bytes, void* stream);

/* Same product as hinm_spmm, computed from a prepared layer (its pi_in / pi_out are the ones given
 * to hinm_prepare).  Flags: HINM_EPI_RELU, HINM_OUT_F32.
 * Few-column shapes (N <= 64, and small layers up to N = 2048) split each tile's kept columns over
 * the waves of one workgroup, which add their fp32 partial tiles in LDS in a fixed order, so results
 * are reproducible bit for bit.  Columns of X between N and ldx are never used in a result.
 * hinm_spmm_prepared_workspace gives the bytes of device workspace a shape needs: 0 for every kernel
 * of this build, so `workspace` may be NULL (the argument stays in the ABI for kernels that split a
 * tile over workgroups; one that needs it returns HINM_ERR_WORKSPACE when it is missing, misaligned
 * (256 bytes) or too small). */
hinm_status hinm_spmm_prepared_workspace(const hinm_shape* shape, int32_t N, size_t* workspace_bytes);
hinm_status hinm_spmm_prepared(const hinm_shape* shape, int32_t N, const void* prepared,
                               const void* X, int64_t ldx, void* Y, int64_t ldy, uint32_t flags,
                               void* workspace, size_t workspace_bytes, void* stream);

/* Measurement aid: which kernel(s) hinm_spmm_prepared would launch for this shape, N, leading
 * dimensions and flags, as text in `text` (NUL-terminated, truncated to text_bytes): one entry per
 * launch, "name<template configuration> grid=... block=...", entries separated by "; ".  *launches
 * (may be NULL) receives their number.  Launches nothing and touches no device; returns what
 * hinm_spmm_prepared would return for such a call with valid pointers and a sufficient workspace. */
hinm_status hinm_spmm_prepared_plan(const hinm_shape* shape, int32_t N, int64_t ldx, int64_t ldy,
                                    uint32_t flags, char* text, size_t text_bytes, int32_t* launches);

typedef struct {
  hinm_shape shape;
  const void* vals;       /* canonical arrays; may be NULL when `prepared` is given */
  const uint8_t* nm_idx;
  const int32_t* vec_idx;
  const int32_t* pi_in;   /* NULL = identity (ignored when `prepared` is given) */
  const int32_t* pi_out;  /* NULL = identity (ignored when `prepared` is given) */
  uint32_t flags;         /* HINM_EPI_RELU and kernel choice; HINM_OUT_F32 only on the last layer */
  const void* prepared;   /* NULL, or the layer's hinm_prepare buffer (then the fast kernels run) */
} hinm_layer;

/* Bytes of `scratch` hinm_chain needs for L layers at N columns (the
 * intermediates between layers, in the storage type). */
hinm_status hinm_chain_sizes(int32_t L, const hinm_layer* layers, int32_t N, size_t* scratch_bytes);

/* Section 3.2 ("maintaining layer consistency"): L consecutive layers, layer
 * l+1's K equal to layer l's M and the same dtype.  Every layer's call is validated
 * (shape, leading dimensions, pinned kernel against shape) before the first launch, so
 * an error status means nothing was enqueued, HINM_ERR_DEVICE excepted.  Every layer writes its
 * output rows in its own pi_out order and the next layer reads them through
 * its own pi_in; no permute kernel runs in between.  Intermediates are rounded
 * to the storage type.  `scratch` is 256-byte aligned device memory. */
hinm_status hinm_chain(int32_t L, const hinm_layer* layers, int32_t N,
                       const void* X, int64_t ldx, void* Y, int64_t ldy,
                       void* scratch, size_t scratch_bytes, void* stream);

const char* hinm_status_str(hinm_status s);

/* Library version, 1000*major + minor. */
int32_t hinm_version(void);

#ifdef __cplusplus
}
#endif
#endif /* HINM_H */
