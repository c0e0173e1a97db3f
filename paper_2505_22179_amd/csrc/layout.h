// Streaming layout of a packed W4A16 weight, shared by the pack/unpack/dequant and GEMM kernels.
//
// The weight [K, N] (N padded up to a multiple of 128 with zero codes, scales and zero-points) is
// cut into records.  Record (nb, g) covers the 128 columns nb*128 .. nb*128+127 of the
// quantisation group g (rows g*128 .. g*128+127) and holds, in this order,
//   codes   8 tiles x 64 lanes x 16 B = 8192 B
//   scales  16 x 8 fp16              =  256 B
//   zeros   16 x u32                 =   64 B
// Records are stored g-fastest: record index = nb * (K/128) + g, so a wavefront that walks down K
// for one column block reads one contiguous stream.
//
// codes: tile t (columns nb*128 + t*16 .. +15), lane l = 16*r + c of a 64-wide wavefront owns the
// 16 bytes at t*1024 + l*16 = four 32-bit words j = 0..3.  Word j holds the eight codes of column
// nb*128 + t*16 + c at rows g*128 + 32*j + 8*r + p, p = 0..7, with code p in 4-bit field
// (p >> 1) + 4*(p & 1).  This is exactly the second operand of one 16x16x32 fp16 MFMA step j for
// that lane (row/column index = l % 16, eight consecutive k per 16-lane group), and the field
// order lets two masks and one shift split a word into four fp16 pairs (p0,p1) (p2,p3) (p4,p5)
// (p6,p7) in register order.
//
// scales: fp16 at 8192 + c*16 + t*2 is the scale of column nb*128 + t*16 + c -- the eight scales
// a lane needs for its eight tiles are one 16-byte load.
// zeros: u32 at 8448 + c*4 holds, in field t, the zero-point of column nb*128 + t*16 + c.
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace w4 {

constexpr int kGroup = 128;           // quantisation group size G (rows)
constexpr int kBlockCols = 128;       // columns per record
constexpr int kTiles = 8;             // 16-column tiles per record
constexpr int kCodesBytes = 8192;
constexpr int kScalesOff = 8192;
constexpr int kZerosOff = 8448;
constexpr int kRecordBytes = 8512;

__host__ __device__ inline int pad_cols(int N) { return (N + kBlockCols - 1) / kBlockCols * kBlockCols; }
__host__ __device__ inline size_t record_offset(int nb, int g, int groups)
{
    return ((size_t)nb * (size_t)groups + (size_t)g) * (size_t)kRecordBytes;
}
// position of code p (0..7) inside a packed word, and its inverse
__host__ __device__ inline int field_of_p(int p) { return (p >> 1) + 4 * (p & 1); }
__host__ __device__ inline int p_of_field(int f) { return ((f & 3) << 1) | (f >> 2); }

}  // namespace w4
