// Blocked, swizzled bf16 matrix layout used for every bf16 tensor the matrix units read.
//
// A matrix [rows][cols] is cut into 32x32 blocks of 2 KiB, stored block-row by block-row.
// Inside a block, row r is 64 bytes = 4 units of 8 elements, and unit q sits at position
// q ^ ((r / 4) % 4).  Why:
//   * a GEMM tile is a run of whole blocks whichever way the matrix is used -- R rows x 32 k
//     (k along the columns) is R/32 blocks, 32 k x R columns (k along the rows) is R/32
//     consecutive blocks, i.e. one contiguous stretch -- so tiles are fetched from HBM as
//     contiguous 2..16 KiB pieces instead of 64-byte slivers of many rows (measured: +38 % on
//     the forward GEMM), and a tile lands in LDS by a straight copy;
//   * with the swizzle, both the 128-bit fragment reads (lanes on consecutive rows) and the
//     transposing reads (4 rows x 32 bytes per 16 lanes) are free of LDS bank conflicts.
// Rows and columns are padded to multiples of 32 with zeros.
#pragma once
#include <stdint.h>

namespace lsam {

__host__ __device__ inline int b32s_blocks(int n) { return (n + 31) >> 5; }

// Element offset of (r, c) in a matrix stored with `cblocks` column blocks.
__host__ __device__ inline int64_t b32s_offset(int r, int c, int cblocks) {
  return ((int64_t)(r >> 5) * cblocks + (c >> 5)) * 1024 + (r & 31) * 32 +
         ((((c & 31) >> 3) ^ ((r >> 2) & 3)) << 3) + (c & 7);
}

// Elements occupied by a [rows][cols] matrix.
__host__ __device__ inline int64_t b32s_size(int rows, int cols) {
  return (int64_t)b32s_blocks(rows) * b32s_blocks(cols) * 1024;
}

// Where the bf16 operand copy of each weight matrix lives, for the kernels that stream the
// flat fp32 parameter vector and refresh that copy on the way.
struct ShadowMap {
  int32_t n;                    // number of weight matrices
  int32_t ldw[LSAM_MAX_LAYERS];      // row pitch of W_l in the flat layout (floats)
  int32_t cblocks[LSAM_MAX_LAYERS];  // column blocks of the stored copy
  int64_t begin[LSAM_MAX_LAYERS];    // flat offset of W_l inside a replica
  int64_t end[LSAM_MAX_LAYERS];      // begin + out_l * ldw_l
  int64_t shadow[LSAM_MAX_LAYERS];   // offset of the copy of W_l inside a replica's operand copy
};

// Offset in a replica's operand copy of the 4 elements starting at flat offset `flat`
// (a multiple of 4), or -1 if they belong to no weight matrix (biases, padding).
__device__ inline int64_t shadow_offset4(const ShadowMap& m, int64_t flat) {
  for (int s = 0; s < m.n; ++s) {
    if (flat >= m.begin[s] && flat < m.end[s]) {
      const unsigned rel = (unsigned)(flat - m.begin[s]);
      const unsigned row = rel / (unsigned)m.ldw[s];
      const unsigned col = rel - row * (unsigned)m.ldw[s];
      return m.shadow[s] + b32s_offset((int)row, (int)col, m.cblocks[s]);
    }
  }
  return -1;
}

}  // namespace lsam
