// Packed INT8 slice layout shared by the split, export and GEMM kernels.
//
// A slice stack holds k slices of a matrix with `rows` scaled vectors (rows of
// A, or columns of B) of inner length n.  Rows are padded to a multiple of
// TILE_R, the inner index to a multiple of KPAD, padding is zero.  One slice is
// stored tile-major: tile (rt, kt) = TILE_R rows x TILE_K inner bytes is one
// contiguous 16 KiB block, tiles of one row block are consecutive in kt, so a
// workgroup streaming along the inner dimension reads consecutive blocks and
// no power-of-two row pitch ever reaches the memory channels.
// Inside a tile, row r occupies 64 consecutive bytes made of four 16-byte
// chunks; logical chunk c sits at physical chunk c ^ ((r >> 2) & 3).  That XOR
// is the LDS bank swizzle of the GEMM kernel applied ahead of time: a tile is
// copied to LDS as a plain linear 16 KiB copy (which is what the
// global-load-to-LDS instruction can do: lane i lands at base + 16 i), and the
// 16-byte operand fetches of v_mfma_i32_16x16x64_i8 (16 consecutive rows; the
// four groups of 16 lanes take logical chunks 0, 3, 1, 2) cover all 64 LDS banks
// once in each of the four cycles a ds_read_b128 takes (see k_gemm for the lanes
// that share a cycle).
//
// Stored bytes are OFFSET-ENCODED: a stack carries one offset c and the byte of
// an element is q + c, q being the slice integer of the method (inner padding
// is q = 0 like any zero; padding ROWS may hold anything that is consistent
// with their row sums: their results are never stored).  Round-to-nearest
// slices obey |q| <= 2^(beta-1) and are stored with c = 2^(beta-1) - 1 (63 for
// beta = 7: bytes in [-1, 127], practically all non-negative); other slices
// with c = 0.  Why: the matrix cores draw measurably less power on operands of
// one sign (their sustained clock is higher), and
//   sum_l (a'_l - cA)(b'_l - cB) = sum_l a'_l b'_l - cB sum_l a'_l - cA sum_l b'_l + N cA cB
// (l over the N = inner_padded(n) stored positions) gives the product of the
// slice integers back exactly from the product of the stored bytes and the row
// sums of the stored bytes, in INT32: |a'|, |b'| <= 2^beta - 1 is the magnitude
// the paper's bound on the chunk length is derived for, so the sums of stored
// bytes fit as the sums of slice integers do.  Behind the k slices a stack
// therefore holds, for every padded row R, the PREFIX sums P[s][R] = sum over
// slices 1..s+1 and all inner l of the stored bytes (k arrays of rows_padded
// INT32; the sum over any range of consecutive slices is a difference of two
// entries), and a 256-byte trailer whose first INT32 is c.
#pragma once
#include <cstdint>
#include <cstddef>

namespace ozl {

constexpr int TILE_R = 256;                  // rows per tile
constexpr int TILE_K = 64;                   // inner bytes per tile
constexpr int KPAD = 256;                    // inner padding granule (4 tiles: the GEMM unrolls 4 stages)
constexpr int CHUNK = 16;                    // bytes per MFMA operand fetch
constexpr int NCHUNK = TILE_K / CHUNK;       // 4
constexpr int TILE_BYTES = TILE_R * TILE_K;  // 16 KiB
constexpr int ROWPAD = 0;                    // bytes of padding after the tiles of one row block (0: 256 B .. 4 KiB measured no faster)

__host__ __device__ inline int64_t round_up(int64_t x, int64_t q) { return (x + q - 1) / q * q; }
__host__ __device__ inline int64_t rows_padded(int64_t rows) { return round_up(rows, TILE_R); }
__host__ __device__ inline int64_t inner_padded(int64_t n) { return round_up(n, KPAD); }
// bytes from one row block (TILE_R rows, all inner tiles) to the next
__host__ __device__ inline int64_t rowblock_bytes(int64_t KT) { return KT * TILE_BYTES + ROWPAD; }
__host__ __device__ inline int64_t slice_bytes(int64_t rows, int64_t n)
{
    return rows_padded(rows) / TILE_R * rowblock_bytes(inner_padded(n) / TILE_K);
}

// a whole stack of k slices: slices, prefix row sums, trailer
__host__ __device__ inline int64_t sums_bytes(int64_t rows, int64_t k) { return round_up(4 * k * rows_padded(rows), 256); }
constexpr int64_t TRAILER_BYTES = 256;
__host__ __device__ inline int64_t sums_offset(int64_t rows, int64_t n, int64_t k) { return k * slice_bytes(rows, n); }
__host__ __device__ inline int64_t trailer_offset(int64_t rows, int64_t n, int64_t k)
{
    return sums_offset(rows, n, k) + sums_bytes(rows, k);
}
__host__ __device__ inline int64_t stack_bytes(int64_t rows, int64_t n, int64_t k)
{
    return trailer_offset(rows, n, k) + TRAILER_BYTES;
}

__host__ __device__ inline int swizzle(int r, int c) { return c ^ ((r >> 2) & 3); }

// Byte offset inside one slice of element (row R, inner index l); KT = inner_padded(n) / TILE_K.
__host__ __device__ inline int64_t packed_offset(int64_t R, int64_t l, int64_t KT)
{
    int64_t rt = R / TILE_R, kt = l / TILE_K;
    int r = (int)(R % TILE_R), lk = (int)(l % TILE_K);
    int c = lk / CHUNK, b = lk % CHUNK;
    return rt * rowblock_bytes(KT) + ((kt * TILE_R + r) * TILE_K + swizzle(r, c) * CHUNK + b);
}

}  // namespace ozl
