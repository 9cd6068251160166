// Steps (iii) and (iv) of the scheme on the gfx950 matrix cores.
//
// k_gemm computes, for one chunk of one group g (Algorithm 6 of the paper),
//     C'' = sum_{s = s0..s1} A''_s B''_{g-s}          (INT8 x INT8 -> INT32, exact)
// as ONE GEMM whose inner dimension is the concatenation of the chunk's slice
// pairs, and then either stores C'' (mode 0) or, fused, applies
//     D <- D + 2^(2 - beta g) diag(2^eA) FP64(C'') diag(2^eB)     (mode 1)
// from registers.  The conversion and the power-of-two scaling are exact, so the
// single FP64 addition per chunk is the only rounding on the whole path.
//
// Tiling: 256 x 256 outputs per workgroup, 4 waves in a 2 x 2 grid, each wave
// 128 x 128 = 4 x 4 tiles of v_mfma_i32_32x32x32_i8 (256 INT32 accumulators per
// lane).  Operands arrive in the packed layout of ozimmu_layout.h: a stage is
// one 32 KiB tile of A and one of B (256 rows x 128 inner bytes each), copied
// linearly into LDS (the bank swizzle is already in the layout) and double
// buffered (128 KiB of the 160 KiB LDS).  The inner order of an integer dot
// product is free, so each lane simply fetches 16 consecutive inner bytes.
#include "ozimmu_kernels.h"
#include "ozimmu_layout.h"

namespace {

using namespace ozl;

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int STAGE_BYTES = 2 * TILE_BYTES;  // A tile + B tile
constexpr int NLOAD = TILE_BYTES / (256 * 16);  // 16-byte loads per thread and operand tile = 8

// Map the linear workgroup id to an output tile so that (a) the workgroups
// resident on one XCD (ids congruent mod 8 land on the same XCD) own a
// contiguous range of tiles and (b) consecutive tiles of that range form
// GROUP-row bands walked column by column, which keeps the operand working
// set of the 32 CUs of an XCD inside its private 4 MiB L2.
constexpr int NXCD = 8;
constexpr int GROUP = 8;
__device__ inline void tile_of_block(int bid, int TM, int TP, int& tm, int& tp)
{
    const int T = TM * TP;
    const int xcd = bid % NXCD, idx = bid / NXCD;
    const int base = T / NXCD, rem = T % NXCD;
    const int lin = xcd * base + (xcd < rem ? xcd : rem) + idx;
    const int width = GROUP * TP;
    const int band = lin / width;
    const int first = band * GROUP;
    const int gsz = (TM - first) < GROUP ? (TM - first) : GROUP;
    const int in_band = lin % width;
    tm = first + in_band % gsz;
    tp = in_band / gsz;
}

template <int MODE>
__global__ __launch_bounds__(256) void k_gemm(ozk::GemmArgs a, int TM, int TP)
{
    extern __shared__ __align__(16) int8_t lds[];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    int tm, tp;
    tile_of_block(blockIdx.x, TM, TP, tm, tp);

    const int KT = a.KT;
    const int nstage = (a.s1 - a.s0 + 1) * KT;

    // operand fetch of lane l for MFMA row tile i and k-step kk: row = w*128 + i*32 + l%32,
    // logical 16-byte chunk = kk*2 + l/32
    const int lr = lane & 31, lh = lane >> 5;

    v16i acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = (v16i){0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

    auto stage_ptrs = [&](int it, const int8_t*& pa, const int8_t*& pb) {
        const int s = a.s0 + it / KT, kt = it % KT;
        pa = a.SA + (int64_t)(s - 1) * a.strideA + ((int64_t)tm * KT + kt) * TILE_BYTES;
        pb = a.SB + (int64_t)(a.g - s - 1) * a.strideB + ((int64_t)tp * KT + kt) * TILE_BYTES;
    };

    v4i ra[NLOAD], rb[NLOAD];
    auto load_global = [&](int it) {
        const int8_t *pa, *pb;
        stage_ptrs(it, pa, pb);
#pragma unroll
        for (int j = 0; j < NLOAD; ++j) {
            ra[j] = *reinterpret_cast<const v4i*>(pa + (j * 256 + t) * 16);
            rb[j] = *reinterpret_cast<const v4i*>(pb + (j * 256 + t) * 16);
        }
    };
    auto store_lds = [&](int buf) {
        int8_t* base = lds + buf * STAGE_BYTES;
#pragma unroll
        for (int j = 0; j < NLOAD; ++j) {
            *reinterpret_cast<v4i*>(base + (j * 256 + t) * 16) = ra[j];
            *reinterpret_cast<v4i*>(base + TILE_BYTES + (j * 256 + t) * 16) = rb[j];
        }
    };
    auto compute = [&](int buf) {
        const int8_t* baseA = lds + buf * STAGE_BYTES;
        const int8_t* baseB = baseA + TILE_BYTES;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            v4i fa[4], fb[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int rowA = wm * 128 + i * 32 + lr;
                const int rowB = wn * 128 + i * 32 + lr;
                fa[i] = *reinterpret_cast<const v4i*>(baseA + rowA * TILE_K + swizzle(rowA, kk * 2 + lh) * CHUNK);
                fb[i] = *reinterpret_cast<const v4i*>(baseB + rowB * TILE_K + swizzle(rowB, kk * 2 + lh) * CHUNK);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    };

    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int it = 0; it < nstage; ++it) {
        const bool more = it + 1 < nstage;
        if (more) load_global(it + 1);
        compute(it & 1);
        if (more) store_lds((it + 1) & 1);
        __syncthreads();
    }

    // Epilogue.  Accumulator register r of tile (i, j) in lane l holds output
    // row 8*(r/4) + 4*(l/32) + r%4 and column l%32 of that 32 x 32 tile.
    const int64_t row0 = (int64_t)tm * 256 + wm * 128;
    const int64_t col0 = (int64_t)tp * 256 + wn * 128;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int64_t col = col0 + j * 32 + lr;
        if (col >= a.p) continue;
        int eb = 0;
        if (MODE == 1) eb = a.eB[col] + a.shift;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = row0 + i * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
                if (row >= a.m) continue;
                if (MODE == 0) {
                    a.C[row * a.ldc + col] = acc[i][j][r];
                } else {
                    const double term = ldexp((double)acc[i][j][r], a.eA[row] + eb);
                    double* d = a.D + row * a.ldd + col;
                    *d = a.first ? term : (*d + term);
                }
            }
        }
    }
}

// Step (iv) alone: one thread per element, lanes along a row of D.
__global__ __launch_bounds__(256) void k_accumulate(int64_t m, int64_t p, const int32_t* __restrict__ C, int64_t ldc,
                                                    const int32_t* __restrict__ eA, const int32_t* __restrict__ eB,
                                                    int shift, int first, double* __restrict__ D, int64_t ldd)
{
    const int64_t j = (int64_t)blockIdx.y * 256 + threadIdx.x;
    const int64_t i0 = (int64_t)blockIdx.x * 8;
    if (j >= p) return;
    const int eb = eB[j] + shift;
    for (int64_t i = i0; i < i0 + 8 && i < m; ++i) {
        const double term = ldexp((double)C[i * ldc + j], eA[i] + eb);
        double* d = D + i * ldd + j;
        *d = first ? term : (*d + term);
    }
}

__global__ __launch_bounds__(256) void k_zero_f64(int64_t m, int64_t p, double* __restrict__ D, int64_t ldd)
{
    const int64_t j = (int64_t)blockIdx.y * 256 + threadIdx.x;
    const int64_t i = blockIdx.x;
    if (j < p && i < m) D[i * ldd + j] = 0.0;
}

}  // namespace

namespace ozk {

hipError_t launch_gemm(const GemmArgs& a, int fused, hipStream_t st)
{
    const int TM = (int)(ozl::rows_padded(a.m) / ozl::TILE_R), TP = (int)(ozl::rows_padded(a.p) / ozl::TILE_R);
    const size_t smem = 2 * STAGE_BYTES;
    static bool attr_set[64] = {false};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (!attr_set[dev]) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm<0>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm<1>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)smem);
        if (e != hipSuccess) return e;
        attr_set[dev] = true;
    }
    dim3 grid((unsigned)(TM * TP)), block(256);
    if (fused)
        hipLaunchKernelGGL(k_gemm<1>, grid, block, smem, st, a, TM, TP);
    else
        hipLaunchKernelGGL(k_gemm<0>, grid, block, smem, st, a, TM, TP);
    return hipGetLastError();
}

hipError_t launch_accumulate(int64_t m, int64_t p, const int32_t* C, int64_t ldc, const int32_t* eA,
                             const int32_t* eB, int shift, int first, double* D, int64_t ldd, hipStream_t st)
{
    dim3 grid((unsigned)((m + 7) / 8), (unsigned)((p + 255) / 256));
    hipLaunchKernelGGL(k_accumulate, grid, dim3(256), 0, st, m, p, C, ldc, eA, eB, shift, first, D, ldd);
    return hipGetLastError();
}

hipError_t launch_fill_zero_f64(int64_t m, int64_t p, double* D, int64_t ldd, hipStream_t st)
{
    dim3 grid((unsigned)m, (unsigned)((p + 255) / 256));
    hipLaunchKernelGGL(k_zero_f64, grid, dim3(256), 0, st, m, p, D, ldd);
    return hipGetLastError();
}

}  // namespace ozk
