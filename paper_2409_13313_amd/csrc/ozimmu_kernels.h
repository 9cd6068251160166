// Internal launcher declarations (host side).  Every launcher enqueues on
// `stream`, checks nothing (the C-ABI layer validates) and returns the HIP
// error of the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace ozk {

// Step (i): row exponents + slices of A.  split_mode 0: round to nearest, ceil exponent (Algorithm 8);
// 1: bit-mask digits, floor exponent (Algorithm 3).  SA is a whole stack (ozl::stack_bytes): slices, prefix row
// sums, trailer; `offset` is the stack's offset c (stored byte = slice integer + c; needs |q + c| <= 127).
hipError_t launch_split_A(int64_t m, int64_t n, const double* A, int64_t lda, int k, int beta, int split_mode,
                          int offset, int8_t* SA, int32_t* eA, hipStream_t st);
// Step (ii): column exponents + slices of B (the same applied to B^T).
// also_zero: optional array of also_zero_count 32-bit words that the first kernel of the split clears on the way
// (the soft-barrier counters of the GEMM that follows: one launch less per call)
hipError_t launch_split_B(int64_t n, int64_t p, const double* B, int64_t ldb, int k, int beta, int split_mode,
                          int offset, int8_t* SB, int32_t* eB, hipStream_t st, uint32_t* also_zero = nullptr,
                          int also_zero_count = 0);
// Algorithm 5: round-to-nearest slices with one scale per slice.  e holds k arrays of exponents (slice-major);
// rem is scratch for the remainders: m x inner_padded(n) doubles for A, n x p doubles for B.
hipError_t launch_split_A_per_slice(int64_t m, int64_t n, const double* A, int64_t lda, int k, int beta, int8_t* SA,
                                    int32_t* eA, double* rem, hipStream_t st);
hipError_t launch_split_B_per_slice(int64_t n, int64_t p, const double* B, int64_t ldb, int k, int beta, int8_t* SB,
                                    int32_t* eB, double* rem, hipStream_t st);
hipError_t launch_export(int64_t rows, int64_t n, int k, const int8_t* packed, int8_t* out, hipStream_t st);

constexpr int QUEUE_ROUND_TILES = 256;  // tiles per round of the queue schedule (see GemmArgs::queue_sets)
constexpr int SYNC_WORDS = 128;  // 32-bit soft-barrier counters at the start of the GEMM scratch (16 per XCD)

struct GemmArgs {
    const int8_t* SA;      // packed stack of A slices
    const int8_t* SB;      // packed stack of B slices
    const int32_t* PA;     // prefix sums over the slices of the row sums of the stored bytes of A: k arrays of pstrideA
    const int32_t* PB;     // the same for B
    int64_t pstrideA, pstrideB;  // = padded rows of the stack
    const int32_t* cA;     // device: offset of the A stack (stored byte = slice integer + offset)
    const int32_t* cB;     // device: offset of the B stack
    int64_t strideA;       // bytes per A slice
    int64_t strideB;       // bytes per B slice
    int KT;                // inner tiles per slice
    // chunk schedule: for g = g_lo..g_hi, chunks of at most r consecutive s out of s_lo(g)..s_hi(g);
    // s_lo = 1, s_hi = g-1 for the full schedule of Algorithm 6; a single chunk sets g_lo == g_hi
    // and gives its own s range in s0, s1 (s0 > 0)
    int g_lo, g_hi, r;
    int s0, s1;
    int64_t m, p;          // valid output extent
    int32_t* C;            // INT32 output (mode 0, single chunk only); fused == 3: one 256 x 256 block per tile of
    int64_t ldc;           // the launch, in the order of the launch's tiles, each in the kernel's own element
                           // order (launch_accumulate_tiles / _chunks read it back; ldc unused)
    double* D;             // FP64 accumulate target (mode 1)
    int64_t ldd;
    const int32_t* eA;
    const int32_t* eB;
    int64_t estrideA, estrideB;  // fused == 2 only: elements from the exponents of slice s to those of slice s+1
    int zsplit;            // fused == 3 only: parts the inner range of a chunk is cut into (<= KT / 4)
    int nchunks;           // fused == 3 only: 0, or the number of chunks of the full schedule g_lo..g_hi: the launch
                           // then runs every chunk, C holding nchunks x tile_count blocks (chunk-major)
    // fused == 3 with nchunks > 0 and queue_sets > 0 ("queue" schedule): the work items run round by round (256
    // tiles, all their chunks), C holds queue_sets sets of nchunks x queue_stride blocks that the rounds take in turn, and the
    // workgroup that finishes the last chunk of a tile adds the tile's chunks up into D (step (iv), and (v) when
    // finish is set).  done: tile_count + number-of-rounds + 1 counters (+ the words of xq), zero at launch (the last one is set if a wait for a
    // set ever ran out of patience: the result is then invalid).  zsplit must be 1.
    int queue_sets;
    int queue_stride;      // blocks per chunk in a set: min(tile_count, 256)
    unsigned* xq;          // queue schedule: 8 x 40 words behind the counters, 8-byte aligned, zero at launch: the
                           // per-XCD ticket batches (see k_gemm); nullptr: single tickets
    int queue_block_rounds;  // the launch covers a whole tile grid made of 16 x 16 blocks: a round is such a block
    unsigned* done;
    int tile_begin, tile_count;  // the launch covers tiles tile_begin .. tile_begin + tile_count - 1 of the band order
    int dma_ok;            // D is 16-byte aligned and ldd even: rows of D can be copied 16 bytes per lane
    int beta;              // shift of group g is 2 - beta * g
    int first;             // D is zero before the first chunk: overwrite
    // step (v) in the epilogue of a tile's last chunk (fused modes): out = fl(fl(alpha d) + fl(cbeta c_old)) into
    // Cout (leading dimension ldco); cbeta == 0: c_old is not read, and Cout must be D itself
    int finish;
    double alpha, cbeta;
    double* Cout;
    int64_t ldco;
    unsigned* sync;        // 8 x 16 counters, zeroed by launch_gemm: [16 x] per-XCD soft barrier, [1] whole grid
    int spin_limit;        // polls before the soft barrier of an XCD's team gives up
    int grid_spin_limit;   // the same for the soft barrier of the whole grid (0: workgroups arrive, none waits)
    int num_cu;            // compute units of the device: the persistent grid has one workgroup on each
    int sync_epoch;        // 0: launch_gemm zeroes the counters; e > 0: e single-chunk launches of this very geometry
    int sync_zeroed;       // the caller has zeroed the counters already (with sync_epoch 0: no fill launch)
                           // have used them since (the split-inner schedule: one reset for all its chunks)
};
// Steps (iii) (+ (iv) when fused is 1 or 2) for the chunks of the schedule (Algorithm 6).  fused == 2: one scale
// per slice (Algorithm 5), r must be 1.  fused == 3: INT32 partial sums of a.zsplit inner parts added to a
// zeroed C (single chunk).
hipError_t launch_gemm(const GemmArgs& a, int fused, hipStream_t st);
// One-time set-up of the current device for launch_gemm (raises the dynamic LDS limit of the chunk GEMM kernels).
hipError_t setup_gemm_kernels();
hipError_t launch_fill_zero_i32(int64_t count, int32_t* x, hipStream_t st);
hipError_t launch_fill_zero_i32_2d(int64_t m, int64_t p, int32_t* C, int64_t ldc, hipStream_t st);
// Step (iv) alone.
hipError_t launch_accumulate(int64_t m, int64_t p, const int32_t* C, int64_t ldc, const int32_t* eA,
                             const int32_t* eB, int shift, int first, double* D, int64_t ldd, hipStream_t st);
// Step (iv) for the tiles tile_begin .. tile_begin + tile_count - 1 (band order) of one chunk (group g, slices
// s0 .. s1 of A) from per-tile 256 x 256 INT32 blocks holding the chunk sums (as launch_gemm with fused == 3 leaves
// them); the blocks are left zeroed.
// finish: step (v) as in GemmArgs.
struct TileAccArgs {
    int tile_begin, tile_count, TM, TP;  // TM, TP are filled in by the launcher
    int64_t m, p;
    int32_t* Ct;
    int parts;             // zsplit of the launch that left the blocks (it decides their element order)
    const int32_t* eA;
    const int32_t* eB;
    int shift, first;
    double* D;
    int64_t ldd;
    int finish;
    double alpha, cbeta;
    double* Cout;
    int64_t ldco;
};
hipError_t launch_accumulate_tiles(const TileAccArgs& t, hipStream_t st);
// Step (iv) for ALL chunks of the schedule (groups 2..k+1, chunks of r) at once: the chunk sums of chunk q lie in
// blocks Ct[q][tile]; they are added in schedule order, one rounded FP64 addition each.  Uses t.tile_*, m, p, Ct,
// eA, eB, D, ldd and the finish fields; shift / first are ignored.
hipError_t launch_accumulate_chunks(const TileAccArgs& t, int k, int r, int beta, hipStream_t st);
// Step (v): C <- alpha D + beta C (beta == 0: C not read).
hipError_t launch_axpby(int64_t m, int64_t p, double alpha, const double* D, int64_t ldd, double beta, double* C,
                        int64_t ldc, hipStream_t st);
hipError_t launch_fill_zero_f64(int64_t m, int64_t p, double* D, int64_t ldd, hipStream_t st);

}  // namespace ozk
