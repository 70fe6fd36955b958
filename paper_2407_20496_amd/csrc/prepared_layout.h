// Layout of the device-tuned ("prepared") form of one HiNM layer.
//
// The kept columns of a tile are padded to Kp = 64 * ceil(Kv / 64) and walked in S = Kp / 64 steps;
// the V rows of a tile form RB = V / 32 row blocks.  For every (tile t, step s, row block rb) one
// 2304-byte block holds what a wave needs for two 32x32x32 sparse MFMAs (32 kept columns each):
//     bytes    0..2047  stored values, [sub 0..1][lane 0..63][8 x 16 bit]:
//                       lane = 32 * qa + i holds, for row 32 rb + i of the tile, the stored values of
//                       groups 16 s + 8 sub + 4 qa + (0..3)  (canonical vals[row][2 * group + {0,1}])
//     bytes 2048..2303  NM nibbles, [lane] x 32 bit: bits 0..15 the four nibbles of the lane's groups in
//                       sub 0, bits 16..31 those of sub 1 (the index register of the two MFMAs,
//                       selected by ABID 0 / 1); padded groups get value 0 and nibble 0x4
// Blocks are ordered [t][s][rb]: everything a tile needs for one step is contiguous.
//
// Further sections, each 256-byte aligned, in this order:
//     gather  int32 [T][Kp]   row of X that kept column j of tile t reads (vector index composed with
//                             pi_in); -1 for padded j
//     pi_out  int32 [M]       row of Y that row r of the layer writes
//     zeros   1024 bytes      an all-zero row segment (source of padded / out-of-range copies)
//     panel   uint32 [T][Kp]  the same gather table as LDS byte addresses for the kernel that keeps a
//                             64-column panel of X (all K rows, 128 bytes each) in LDS: row g sits at
//                             128 g with its 32-byte units XOR-swizzled by bit 1 of g, so the entry is
//                             128 g | ((g & 2) << 5); padded j point at the all-zero row 8 ceil(K / 8)
#pragma once

#include <stddef.h>
#include <stdint.h>

#include "hinm.h"

namespace hinm {

constexpr int kPrepBlockBytes = 2304;
constexpr int kPrepIdxOffset = 2048;
constexpr int kPrepZeroBytes = 1024;

struct PreparedLayout {
  int T, RB, S, Kp;
  size_t a_offset, gather_offset, pi_out_offset, zero_offset, panel_offset, total_bytes;
};

__host__ __device__ inline size_t prep_align256(size_t x) { return (x + 255) / 256 * 256; }

__host__ inline PreparedLayout prepared_layout(const hinm_shape& s) {
  PreparedLayout L;
  L.T = s.M / s.V;
  L.RB = s.V / 32;
  L.Kp = (s.Kv + 63) / 64 * 64;
  L.S = L.Kp / 64;
  L.a_offset = 0;
  L.gather_offset = prep_align256((size_t)L.T * L.S * L.RB * kPrepBlockBytes);
  L.pi_out_offset = L.gather_offset + prep_align256((size_t)L.T * L.Kp * 4);
  L.zero_offset = L.pi_out_offset + prep_align256((size_t)s.M * 4);
  L.panel_offset = L.zero_offset + kPrepZeroBytes;
  L.total_bytes = L.panel_offset + prep_align256((size_t)L.T * L.Kp * 4);
  return L;
}

__host__ __device__ inline uint32_t panel_entry_of_row(int g, int K) {
  const uint32_t row = (g >= 0) ? (uint32_t)g : (uint32_t)((K + 7) / 8 * 8);
  return (row << 7) | ((g >= 0) ? (((uint32_t)g & 2u) << 5) : 0u);
}

}  // namespace hinm
