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

// Linear tile order: bands of GROUP tile rows, each walked column by column, so
// that 32 consecutive tiles form an 8 x 4 patch (8 A tiles + 4 B tiles per stage).
constexpr int NXCD = 8;
constexpr int GROUP = 8;
__device__ inline void tile_of_linear(int lin, int TM, int TP, int& tm, int& tp)
{
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

// Soft barrier between the workgroups of one XCD ("team").  They share one L2 and
// stream the same A / B tiles; the L2 holds only some twenty stages of the team's
// working set, so operand reuse in L2 lives on the team advancing in lockstep.
// Nothing but timing depends on it: a workgroup that has waited `spin_limit`
// polls goes on alone, so the barrier always ends.  Called by every thread;
// thread 0 arrives and polls, the rest meet it at the next s_barrier.
__device__ inline void team_arrive_and_wait(unsigned* ctr, unsigned target, int spin_limit)
{
    if (threadIdx.x == 0) {
        __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        for (int i = 0; i < spin_limit; ++i) {
            if (__hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= target) break;
            __builtin_amdgcn_s_sleep(8);
        }
    }
}

// Persistent kernel: gridDim.x workgroups (one per CU), workgroup b belongs to
// XCD b % 8 (hardware dispatch order) and is member b / 8 of that XCD's team.
// The tiles of the output are split into 8 contiguous ranges, one per XCD, in
// band order (GROUP tile rows walked column by column); in round q the team
// works on tiles q*team .. q*team+team-1 of its range, i.e. an 8 x 4 patch
// whose A and B tiles are shared through the XCD's L2.  For its tile a
// workgroup runs every chunk of the schedule in the order of Algorithm 6.
template <int MODE, int NS>
__global__ __launch_bounds__(256) void k_gemm(ozk::GemmArgs a, int TM, int TP)
{
    extern __shared__ __align__(16) int8_t lds[];
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int lr = lane & 31, lh = lane >> 5;

    const int KT = a.KT;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)lds;
    const uint32_t voff = (uint32_t)t * 16u;
    const uint32_t m0_wave = lds_base + (uint32_t)wave * 1024u;
    // moving on to the next slice pair of a chunk: A slice s -> s+1, B slice g-s -> g-s-1, inner tile KT-1 -> 0
    const int64_t wrapA = a.strideA - (int64_t)(KT - 1) * TILE_BYTES;
    const int64_t wrapB = -a.strideB - (int64_t)(KT - 1) * TILE_BYTES;

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
    // team geometry
    const int nwg = gridDim.x, bid = blockIdx.x;
    const int xcd = bid % NXCD, member = bid / NXCD;
    const int team = nwg / NXCD + (xcd < nwg % NXCD ? 1 : 0);
    const int T = TM * TP;
    const int tiles_base = T / NXCD, tiles_rem = T % NXCD;
    const int range_off = xcd * tiles_base + (xcd < tiles_rem ? xcd : tiles_rem);
    const int range_cnt = tiles_base + (xcd < tiles_rem ? 1 : 0);
    unsigned* const sync_ctr = a.sync + xcd * 16;
    unsigned sync_target = 0;
    // sync_every is a power of two (or 0: never inside a chunk)
    const int sync_mask = a.sync_every > 0 ? a.sync_every - 1 : 0x7fffffff;

    for (int local = member; local < range_cnt; local += team) {
        const int round_first = local - member;
        const unsigned participants = (unsigned)((range_cnt - round_first) < team ? (range_cnt - round_first) : team);
        int tm, tp;
        tile_of_linear(range_off + local, TM, TP, tm, tp);
        const int64_t row0 = (int64_t)tm * 256 + wm * 128;
        const int64_t col0 = (int64_t)tp * 256 + wn * 128;
        int first = a.first;

        for (int g = a.g_lo; g <= a.g_hi; ++g) {
            const int s_lo = a.s0 > 0 ? a.s0 : 1;
            const int s_hi = a.s0 > 0 ? a.s1 : g - 1;
            for (int c0 = s_lo; c0 <= s_hi; c0 += a.r) {
                const int c1 = (c0 + a.r - 1 < s_hi) ? c0 + a.r - 1 : s_hi;  // chunk: s = c0..c1
                const int nstage = (c1 - c0 + 1) * KT;

                // Copy cursors: tile pointers of the next stage to copy, one per operand (the B half of a
                // stage is issued half an iteration after its A half).  They stop at the last stage, so the
                // copies issued past the end re-read valid memory into buffers nobody reads.
                struct Cursor {
                    const int8_t* ptr;
                    int kt, it;
                };
                Cursor ca = {a.SA + (int64_t)(c0 - 1) * a.strideA + (int64_t)tm * rowblock_bytes(KT), 0, 0};
                Cursor cb = {a.SB + (int64_t)(g - c0 - 1) * a.strideB + (int64_t)tp * rowblock_bytes(KT), 0, 0};
                auto advance = [&](Cursor& c, int64_t wrap_step) {  // branch-free, all scalar
                    const bool adv = c.it + 1 < nstage;
                    const bool wrap = adv && (c.kt + 1 == KT);
                    c.it += adv ? 1 : 0;
                    c.kt = wrap ? 0 : c.kt + (adv ? 1 : 0);
                    c.ptr += wrap ? wrap_step : (adv ? (int64_t)TILE_BYTES : 0);
                };
                // one 16-byte-per-lane copy (quarter q of a tile) of the A / B tile under the cursor into ring buffer `buf`
                auto copy_a = [&](int buf, int q) {
                    copy16_to_lds(m0_wave + (uint32_t)buf * STAGE_BYTES + q * 4096, voff, ca.ptr + q * 4096);
                };
                auto copy_b = [&](int buf, int q) {
                    copy16_to_lds(m0_wave + (uint32_t)buf * STAGE_BYTES + TILE_BYTES + q * 4096, voff, cb.ptr + q * 4096);
                };

                v16i acc[4][4];
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[i][j] = (v16i){0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
                // the 4 MFMAs of A row tile i for one k-step
                auto math_row = [&](const v4i* fa, const v4i* fb, int i) {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
                };
                // fragment i of A and of B for k-step kk of ring buffer `buf`
                auto fetch_one = [&](v4i* fa, v4i* fb, int buf, int kk, int i) {
                    fa[i] = *(lds_v4i_ptr)(uintptr_t)(fragA[kk] + (uint32_t)buf * STAGE_BYTES + i * 2048);
                    fb[i] = *(lds_v4i_ptr)(uintptr_t)(fragB[kk] + (uint32_t)buf * STAGE_BYTES + i * 2048);
                };

                v4i fa0[4], fb0[4], fa1[4], fb1[4];

                // prologue: every wave is past the math of the previous chunk (the LDS ring is free),
                // stages 0 .. NS-3 and the A half of stage NS-2 go in flight, the team lines up, stage 0
                // lands, first fragments fetched
                __builtin_amdgcn_s_barrier();
#pragma unroll
                for (int sidx = 0; sidx < NS - 1; ++sidx) {
#pragma unroll
                    for (int q = 0; q < NLOAD; ++q) copy_a(sidx, q);
                    advance(ca, wrapA);
                    if (sidx < NS - 2) {
#pragma unroll
                        for (int q = 0; q < NLOAD; ++q) copy_b(sidx, q);
                        advance(cb, wrapB);
                    }
                }
                sync_target += participants;
                team_arrive_and_wait(sync_ctr, sync_target, a.spin_limit);
                wait_vmcnt<NLOAD*(2 * (NS - 2) - 1)>();
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
#pragma unroll
                for (int i = 0; i < 4; ++i) fetch_one(fa0, fb0, 0, 0, i);

                // Main loop.  Per stage: 32 MFMAs, 16 fragment fetches and 8 copies, interleaved as
                // (2 fetches, 4 MFMAs, 1 copy) so that no copy or fetch ever waits behind a burst of its
                // own kind while the matrix pipe runs dry.
                int buf = 0;  // ring buffer of stage it
                for (int it = 0; it < nstage; ++it) {
                    const int buf_next = (buf + 1 == NS) ? 0 : buf + 1;
                    const int buf_prev = (buf == 0) ? NS - 1 : buf - 1;
                    const int buf_b = (buf + NS - 2 >= NS) ? buf - 2 : buf + NS - 2;  // buffer of stage it+NS-2
                    // k-step 0 of stage it; fragments of k-step 1 on their way; B half of stage it+NS-2
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        fetch_one(fa1, fb1, buf, 1, q);
                        math_row(fa0, fb0, q);
#ifndef OZ_NOCOPY
                        copy_b(buf_b, q);
#endif
                    }
                    advance(cb, wrapB);
                    if (((it + 1) & sync_mask) == 0 && it + 1 < nstage) {  // every sync_every stages
                        sync_target += participants;
                        team_arrive_and_wait(sync_ctr, sync_target, a.spin_limit);
                    }
                    // stage it+1 complete in LDS for every wave; every wave done reading stage it-1
                    wait_vmcnt<2 * NLOAD * (NS - 3)>();
#ifndef OZ_NOBARRIER
                    __builtin_amdgcn_s_barrier();
#endif
                    asm volatile("" ::: "memory");
                    // k-step 1 of stage it; first fragments of stage it+1 on their way; A half of stage
                    // it+NS-1 into the buffer of stage it-1
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        fetch_one(fa0, fb0, buf_next, 0, q);
                        math_row(fa1, fb1, q);
#ifndef OZ_NOCOPY
                        copy_a(buf_prev, q);
#endif
                    }
                    advance(ca, wrapA);
                    buf = buf_next;
                }
                wait_vmcnt<0>();  // no copy may still be writing LDS when the ring is reused or the workgroup retires

                // Epilogue.  Accumulator register r of tile (i, j) in lane l holds output
                // row 8*(r/4) + 4*(l/32) + r%4 and column l%32 of that 32 x 32 tile.  Addresses are a
                // wave-uniform base plus a 32-bit lane offset, rebuilt for every chunk (the empty asm
                // keeps the compiler from hoisting 64 element addresses per lane out of the chunk loops).
                const int shift = 2 - a.beta * g;
                int64_t er0 = row0, ec0 = col0;
                asm volatile("" : "+s"(er0), "+s"(ec0));
                const bool lane_col_ok[4] = {ec0 + lr < a.p, ec0 + 32 + lr < a.p, ec0 + 64 + lr < a.p,
                                             ec0 + 96 + lr < a.p};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    int eb = 0;
                    if (MODE == 1 && lane_col_ok[j]) eb = a.eB[ec0 + j * 32 + lr] + shift;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int64_t urow = er0 + i * 32 + 8 * (r / 4) + (r % 4);  // uniform part of the row
                            const bool ok = lane_col_ok[j] && (urow + 4 * lh < a.m);
                            if (MODE == 0) {
                                int32_t* base = a.C + urow * a.ldc + ec0 + j * 32;
                                const uint32_t off = (uint32_t)(4 * lh) * (uint32_t)a.ldc + (uint32_t)lr;
                                if (ok) base[off] = acc[i][j][r];
                            } else {
                                double* base = a.D + urow * a.ldd + ec0 + j * 32;
                                const uint32_t off = (uint32_t)(4 * lh) * (uint32_t)a.ldd + (uint32_t)lr;
                                if (ok) {
                                    const double term = ldexp((double)acc[i][j][r], a.eA[urow + 4 * lh] + eb);
                                    base[off] = first ? term : (base[off] + term);
                                }
                            }
                        }
                        // one 32 x 32 tile at a time keeps the epilogue's loads within the register budget
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                first = 0;
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

// zero the soft-barrier counters (a kernel rather than a memset so that the call can be captured in a graph)
__global__ void k_fill_u32_gemm(unsigned* x) { x[threadIdx.x] = 0u; }

#ifndef OZ_NS
#define OZ_NS 4
#endif
constexpr int NSTAGES = OZ_NS;

}  // namespace

namespace ozk {

hipError_t launch_gemm(const GemmArgs& a, int fused, hipStream_t st)
{
    const int TM = (int)(ozl::rows_padded(a.m) / ozl::TILE_R), TP = (int)(ozl::rows_padded(a.p) / ozl::TILE_R);
    const size_t smem = (size_t)NSTAGES * STAGE_BYTES;
    static bool attr_set[64] = {false};
    static int num_cu[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (!attr_set[dev]) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm<0, NSTAGES>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm<1, NSTAGES>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        e = hipDeviceGetAttribute(&num_cu[dev], hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return e;
        attr_set[dev] = true;
    }
    // one workgroup per CU (the LDS ring allows no second one), never more workgroups than tiles
    const int64_t tiles = (int64_t)TM * TP;
    int nwg = num_cu[dev] > 0 ? num_cu[dev] : 1;
    if (tiles < nwg) nwg = (int)tiles;
    hipLaunchKernelGGL(k_fill_u32_gemm, dim3(1), dim3(NXCD * 16), 0, st, a.sync);
    dim3 grid((unsigned)nwg), block(256);
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
