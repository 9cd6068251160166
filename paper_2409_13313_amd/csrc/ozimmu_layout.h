// Packed INT8 slice layout shared by the split, export and GEMM kernels.
//
// A slice stack holds k slices of a matrix with `rows` scaled vectors (rows of
// A, or columns of B) of inner length n.  Rows are padded to a multiple of
// TILE_R, the inner index to a multiple of TILE_K, padding is zero.  One slice
// is stored tile-major: tile (rt, kt) = TILE_R rows x TILE_K inner bytes is one
// contiguous 32 KiB block, tiles of one row block are consecutive in kt, so a
// workgroup streaming along the inner dimension reads consecutive blocks.
// Inside a tile, row r occupies 128 consecutive bytes made of eight 16-byte
// chunks; logical chunk c sits at physical chunk c ^ ((r >> 1) & 7).  That XOR
// is the LDS bank swizzle of the GEMM kernel applied ahead of time, so a tile
// is copied to LDS as a plain linear 32 KiB copy and the 16-byte operand
// fetches of v_mfma_i32_32x32x32_i8 (32 consecutive rows, one chunk) spread
// over all 64 LDS banks (measured 151 B/clk against 128 B/clk for c ^ (r & 7)
// and 32 B/clk unswizzled).
#pragma once
#include <cstdint>
#include <cstddef>

namespace ozl {

constexpr int TILE_R = 256;                  // rows per tile
constexpr int TILE_K = 128;                  // inner bytes per tile
constexpr int CHUNK = 16;                    // bytes per MFMA operand fetch
constexpr int TILE_BYTES = TILE_R * TILE_K;  // 32 KiB

__host__ __device__ inline int64_t round_up(int64_t x, int64_t q) { return (x + q - 1) / q * q; }
__host__ __device__ inline int64_t rows_padded(int64_t rows) { return round_up(rows, TILE_R); }
__host__ __device__ inline int64_t inner_padded(int64_t n) { return round_up(n, TILE_K); }
__host__ __device__ inline int64_t slice_bytes(int64_t rows, int64_t n) { return rows_padded(rows) * inner_padded(n); }

__host__ __device__ inline int swizzle(int r, int c) { return c ^ ((r >> 1) & 7); }

// Byte offset inside one slice of element (row R, inner index l); KT = inner_padded(n) / TILE_K.
__host__ __device__ inline int64_t packed_offset(int64_t R, int64_t l, int64_t KT)
{
    int64_t rt = R / TILE_R, kt = l / TILE_K;
    int r = (int)(R % TILE_R), lk = (int)(l % TILE_K);
    int c = lk / CHUNK, b = lk % CHUNK;
    return ((rt * KT + kt) * TILE_R + r) * TILE_K + swizzle(r, c) * CHUNK + b;
}

}  // namespace ozl
