// Steps (iii) and (iv) of the scheme on the gfx950 matrix cores.
//
// k_gemm computes, for one chunk of one group g (Algorithm 6 of the paper),
//     C'' = sum_{s = s0..s1} A''_s B''_{g-s}          (INT8 x INT8 -> INT32, exact)
// as ONE GEMM whose inner dimension is the concatenation of the chunk's slice
// pairs, and then either stores C'' (MODE 0) or, fused, applies
//     D <- D + 2^(2 - beta g) diag(2^eA) FP64(C'') diag(2^eB)     (MODE 1)
// from registers.  The conversion and the power-of-two scaling are exact, so the
// single FP64 addition per chunk is the only rounding on the whole path.
//
// Tiling: 256 x 256 outputs per workgroup, 4 waves in a 2 x 2 grid, each wave
// 128 x 128 = 4 x 4 tiles of v_mfma_i32_32x32x32_i8 (256 INT32 accumulators per
// lane, one wave per SIMD).  A stage is one packed 16 KiB tile of A and one of B
// (256 rows x 64 inner bytes each, see ozimmu_layout.h).  Stages travel from
// global memory straight into a ring of NS LDS buffers with
// global_load_lds_dwordx4 (no VGPR staging; the bank swizzle is already in the
// packed layout, so the copy is linear), NS - 2 stages ahead of the math.
// Operand fragments are double buffered in registers and fetched one k-step
// ahead, across stage boundaries, so LDS latency hides behind the 16 MFMAs of
// the current k-step.  The inner order of an integer dot product is free, so
// each lane simply fetches 16 consecutive inner bytes.
//
// Synchronisation per stage `it` (buffer it % NS), one barrier:
//   k-step 0 math | wait until this thread's copies of stage it+1 landed |
//   barrier | fetch fragments of stage it+1 | issue copies of stage it+NS-1 into
//   the buffer of stage it-1 (every wave has finished reading it: its data fed
//   MFMAs issued before the barrier) | k-step 1 math.
// The LDS-writing loads are issued from inline assembly, so the compiler does
// not track them; the vmcnt waits that order them are written out below.
#include "ozimmu_kernels.h"
#include "ozimmu_layout.h"

namespace {

using namespace ozl;

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int STAGE_BYTES = 2 * TILE_BYTES;       // A tile + B tile = 32 KiB
constexpr int NLOAD = TILE_BYTES / (256 * 16);    // 16-byte copies per thread and operand tile = 4

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

// One 16-byte-per-lane copy global -> LDS: lane i of the wave writes LDS bytes
// [m0 + 16 i, m0 + 16 i + 16) with the 16 bytes at gbase + voff (voff per lane).
__device__ inline void copy16_to_lds(uint32_t m0, uint32_t voff, const int8_t* gbase)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(m0), "v"(voff), "s"(gbase)
                 : "memory");
}

template <int N>
__device__ inline void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <int MODE, int NS>
__global__ __launch_bounds__(256) void k_gemm(ozk::GemmArgs a, int TM, int TP)
{
    extern __shared__ __align__(16) int8_t lds[];
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int lr = lane & 31, lh = lane >> 5;
    int tm, tp;
    tile_of_block(blockIdx.x, TM, TP, tm, tp);

    const int KT = a.KT;
    const int nstage = (a.s1 - a.s0 + 1) * KT;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)lds;
    const uint32_t voff = (uint32_t)t * 16u;
    const uint32_t m0_wave = lds_base + (uint32_t)wave * 1024u;

    // pointers of the next stage to copy (advanced stage by stage; they stop at the last stage,
    // so the copies issued past the end re-read valid memory into buffers nobody reads)
    int cp_kt = 0, cp_it = 0;
    const int8_t* cp_a = a.SA + (int64_t)(a.s0 - 1) * a.strideA + (int64_t)tm * KT * TILE_BYTES;
    const int8_t* cp_b = a.SB + (int64_t)(a.g - a.s0 - 1) * a.strideB + (int64_t)tp * KT * TILE_BYTES;
    // moving on to the next slice pair of the chunk: A slice s -> s+1, B slice g-s -> g-s-1, inner tile KT-1 -> 0
    const int64_t wrapA = a.strideA - (int64_t)(KT - 1) * TILE_BYTES;
    const int64_t wrapB = -a.strideB - (int64_t)(KT - 1) * TILE_BYTES;
    auto issue_copy = [&](int buf) {
        const uint32_t m0 = m0_wave + (uint32_t)buf * STAGE_BYTES;
#pragma unroll
        for (int j = 0; j < NLOAD; ++j) copy16_to_lds(m0 + j * 4096, voff, cp_a + j * 4096);
#pragma unroll
        for (int j = 0; j < NLOAD; ++j) copy16_to_lds(m0 + TILE_BYTES + j * 4096, voff, cp_b + j * 4096);
        // branch-free advance (all scalar)
        const bool adv = cp_it + 1 < nstage;
        const bool wrap = adv && (cp_kt + 1 == KT);
        cp_it += adv ? 1 : 0;
        cp_kt = wrap ? 0 : cp_kt + (adv ? 1 : 0);
        cp_a += wrap ? wrapA : (adv ? (int64_t)TILE_BYTES : 0);
        cp_b += wrap ? wrapB : (adv ? (int64_t)TILE_BYTES : 0);
    };

    // per-lane fragment offsets inside a stage: row = w*128 + i*32 + lane%32, logical chunk = kk*2 + lane/32;
    // i*32 rows = i*2048 bytes and does not change the swizzle, so only kk needs its own offset
    uint32_t fragA[2], fragB[2];
    {
        const int rowA = wm * 128 + lr, rowB = wn * 128 + lr;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            fragA[kk] = lds_base + rowA * TILE_K + swizzle(rowA, kk * 2 + lh) * CHUNK;
            fragB[kk] = lds_base + TILE_BYTES + rowB * TILE_K + swizzle(rowB, kk * 2 + lh) * CHUNK;
        }
    }
    typedef __attribute__((address_space(3))) const v4i* lds_v4i_ptr;
    auto fetch = [&](v4i* fa, v4i* fb, int buf, int kk) {
        const uint32_t pa = fragA[kk] + (uint32_t)buf * STAGE_BYTES;
        const uint32_t pb = fragB[kk] + (uint32_t)buf * STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            fa[i] = *(lds_v4i_ptr)(uintptr_t)(pa + i * 2048);
            fb[i] = *(lds_v4i_ptr)(uintptr_t)(pb + i * 2048);
        }
    };

    v16i acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = (v16i){0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

    // MFMAs of one k-step for A row tiles i0 .. i0+1 (8 of the 16)
    auto math_half = [&](const v4i* fa, const v4i* fb, int i0) {
#pragma unroll
        for (int i = i0; i < i0 + 2; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
    };
    // ask the scheduler for the pattern 1 LDS read : 2 MFMA over a k-step (8 reads, 16 MFMAs)
    auto interleave = [&]() {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // DS read
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);  // MFMA
        }
    };

    v4i fa0[4], fb0[4], fa1[4], fb1[4];

    // prologue: stages 0 .. NS-2 in flight, stage 0 landed and visible, its first fragments fetched
#pragma unroll
    for (int sidx = 0; sidx < NS - 1; ++sidx) issue_copy(sidx);
    wait_vmcnt<2 * NLOAD * (NS - 2)>();
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    fetch(fa0, fb0, 0, 0);

    int buf = 0;
    for (int it = 0; it < nstage; ++it) {
        const int buf_next = (buf + 1 == NS) ? 0 : buf + 1;
        const int buf_prev = (buf == 0) ? NS - 1 : buf - 1;
        // k-step 0 of stage it; fragments of k-step 1 on their way
        fetch(fa1, fb1, buf, 1);
        math_half(fa0, fb0, 0);
        math_half(fa0, fb0, 2);
        interleave();
        // stage it+1 complete in LDS for every wave
        wait_vmcnt<2 * NLOAD * (NS - 3)>();
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        // k-step 1 of stage it; first fragments of stage it+1 on their way; refill the freed buffer
        fetch(fa0, fb0, buf_next, 0);
        math_half(fa1, fb1, 0);
        issue_copy(buf_prev);
        math_half(fa1, fb1, 2);
        buf = buf_next;
    }
    wait_vmcnt<0>();  // no copy may still be writing LDS when the workgroup retires

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

constexpr int NSTAGES = 4;

}  // namespace

namespace ozk {

hipError_t launch_gemm(const GemmArgs& a, int fused, hipStream_t st)
{
    const int TM = (int)(ozl::rows_padded(a.m) / ozl::TILE_R), TP = (int)(ozl::rows_padded(a.p) / ozl::TILE_R);
    const size_t smem = (size_t)NSTAGES * STAGE_BYTES;
    static bool attr_set[64] = {false};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (!attr_set[dev]) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm<0, NSTAGES>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm<1, NSTAGES>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_set[dev] = true;
    }
    dim3 grid((unsigned)(TM * TP)), block(256);
    if (fused)
        hipLaunchKernelGGL((k_gemm<1, NSTAGES>), grid, block, smem, st, a, TM, TP);
    else
        hipLaunchKernelGGL((k_gemm<0, NSTAGES>), grid, block, smem, st, a, TM, TP);
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
