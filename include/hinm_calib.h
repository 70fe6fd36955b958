/*
 * hinm_calib.h -- measurement aids of libhinm (gfx950): plain kernels of known work that calibrate the
 * ceilings the HiNM kernels are priced against (streaming copy / fill / read rates, the issue rate of
 * the sparse matrix instruction, the cost of an empty launch, the rate at which a compute unit draws
 * cache-resident data into LDS, and a store-only pass that writes rows in a permuted order as the
 * output-channel scatter of the product does).  None of them is part of the method and none is called
 * by the product or packing entry points; the benchmark uses them to report fractions against
 * measured as well as nominal peaks.
 *
 * All pointers are DEVICE memory owned by the caller unless stated; all work is asynchronous on
 * `stream` (a hipStream_t, NULL = the default stream); nothing is allocated and nothing synchronises.
 * Status codes as in hinm.h; argument errors are reported before anything is launched.
 */
#ifndef HINM_CALIB_H
#define HINM_CALIB_H

#include "hinm.h"

#ifdef __cplusplus
extern "C" {
#endif

/* dst[0..bytes) = src[0..bytes), 16 bytes per lane and step, grid-stride over 2048 workgroups.
 * bytes a multiple of 16, both pointers 16-byte aligned, ranges must not overlap.
 * nontemporal != 0: loads and stores carry the non-temporal hint. */
hinm_status hinm_calib_copy(const void* src, void* dst, size_t bytes, int32_t nontemporal, void* stream);

/* dst[0..bytes) = a constant byte pattern (store-only stream); same rules as hinm_calib_copy. */
hinm_status hinm_calib_fill(void* dst, size_t bytes, int32_t nontemporal, void* stream);

/* Reads src[0..bytes) once (load-only stream); every lane folds what it read into one 32-bit word and
 * the lanes whose word is 0x9E3779B9 (practically none) write it to sink[0]: the loads cannot be
 * dropped.  sink: 4 bytes. */
hinm_status hinm_calib_read(const void* src, size_t bytes, int32_t nontemporal, uint32_t* sink, void* stream);

/* Store-only pass shaped like the product's epilogue: an M x N matrix of 16-bit elements (leading
 * dimension ld elements, a multiple of 8) is written in pieces of piece_bytes contiguous bytes
 * (64, 128, 256, 512 or 1024; N * 2 a multiple of it), row r of the work going to row rows[r] of dst
 * (rows: int32 [M], a permutation; NULL = natural order).  Non-temporal stores. */
hinm_status hinm_calib_scatter_rows(void* dst, int32_t M, int32_t N, int64_t ld, const int32_t* rows,
                                    int32_t piece_bytes, void* stream);

/* Register-resident loop of the 32x32x32 structured-sparse matrix instruction (dtype HINM_F16 or
 * HINM_BF16): 2048 workgroups of four waves, every wave issues iterations x 4 instructions on four
 * independent accumulators with no memory traffic.  sink: float [2048 * 256], receives one value per
 * lane.  *stored_value_flops (HOST pointer, may be NULL) = flops of the launch counted on the stored
 * values, 2 * 32 * 16 * 32 per instruction (the hardware rating counts twice that). */
hinm_status hinm_calib_smfmac(int32_t dtype, int32_t iterations, float* sink, double* stored_value_flops,
                              void* stream);

/* One workgroup of one wave that does nothing: the cost of a launch (or of a graph node). */
hinm_status hinm_calib_empty(void* stream);

/* Compute units draw data into LDS with direct-to-LDS loads of 16 bytes per lane: `workgroups` workgroups
 * of 512 lanes; workgroup w copies chunks_per_workgroup consecutive 8 KiB chunks of the region (region_bytes,
 * a multiple of 8192, 16-byte aligned), starting at byte (w * start_stride_bytes) % region_bytes (a
 * multiple of 8192) and wrapping at the region's end, with eight copies per wave in flight (64 KiB per
 * workgroup).  A small region with a small stride stays cache-resident (every workgroup walks the same
 * bytes); a large region with start_stride_bytes = region_bytes / workgroups gives every workgroup bytes
 * that nobody else reads.  Total bytes drawn = workgroups * chunks_per_workgroup * 8192. */
hinm_status hinm_calib_lds_stream(const void* region, size_t region_bytes, size_t start_stride_bytes,
                                  int64_t chunks_per_workgroup, int32_t workgroups, void* stream);

/* The request pattern of the tile kernels' gathered input rows, without their stages and barriers: the
 * first `waves` (1..8) waves of each of `workgroups` workgroups copy copies_per_wave row segments of
 * 1 KB each straight into LDS, `outstanding` (4, 8 or 16) copies in flight per wave.  The rows are
 * taken at a fixed stride through [0, rows) of a matrix of `rows` rows of row_pitch_bytes (>= 8192, a
 * multiple of 16) that starts at `region` (device memory, 16-byte aligned, at least rows x
 * row_pitch_bytes bytes; only read).  Few rows = a stream of L2 hits, many rows = a stream from
 * beyond the caches.  Moves workgroups x waves x copies_per_wave KB. */
hinm_status hinm_calib_gather_stream(const void* region, size_t region_bytes, int64_t row_pitch_bytes, int32_t rows,
                                     int32_t waves, int32_t outstanding, int32_t copies_per_wave,
                                     int32_t workgroups, void* stream);

/* One part of the tile kernel that hinm_spmm_prepared would launch for this shape and N, on a real
 * prepared layer (hinm_prepare) and a real X: part 1 = only its copy stream (gathered rows of X and the
 * stored values through L2 into LDS, with the kernel's own barriers and waits; no LDS reads, no MFMAs),
 * part 2 = only its LDS reads and MFMAs (no copies after the first stages, so the operands are stale).
 * Nothing is stored.  For the shapes of the named workloads that run on the tile kernel in one launch
 * (V of 64 or 128); HINM_ERR_UNSUPPORTED otherwise.  The two times say which side bounds the product. */
hinm_status hinm_calib_tile_part(const hinm_shape* shape, int32_t N, const void* prepared, const void* X,
                                 int64_t ldx, int32_t part, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* HINM_CALIB_H */
