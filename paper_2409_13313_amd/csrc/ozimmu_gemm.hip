// Steps (iii) and (iv) of the scheme on the gfx950 matrix cores.
//
// k_gemm computes, for one chunk of one group g (Algorithm 6 of the paper),
//     C'' = sum_{s = s0..s1} A''_s B''_{g-s}          (INT8 x INT8 -> INT32, exact)
// as ONE GEMM whose inner dimension is the concatenation of the chunk's slice
// pairs, and then either stores C'' (MODE 0) or, fused, applies
//     D <- D + 2^(2 - beta g) diag(2^eA) FP64(C'') diag(2^eB)     (MODE 1)
// from registers.  The conversion and the power-of-two scaling are exact, so the
// single FP64 addition per chunk is the only rounding on the whole path.
// MODE 2 is MODE 1 for slices that carry one scale each (Algorithm 5): every chunk
// is one pair (s, t) and the factor is 2^(2 - 2 beta) diag(2^eA_s) . diag(2^eB_t).
// MODE 3 is MODE 0 for tiles too few to fill the chip, its output one 256 x 256 block
// per work item in the accumulators' own order (see lane_major_coords): the inner range
// of the chunk is cut into Z parts that run on different workgroups and add their INT32
// partial sums to zeroed per-tile blocks with integer atomics (exact in any order).  With
// a.nchunks > 0 one MODE 3 launch covers ALL chunks of the schedule at once: a work
// item is (chunk, part, tile), every chunk has a block per tile of its own, and a
// separate kernel adds the chunks up in FP64 in the order of Algorithm 6.  With
// a.queue_sets > 0 as well (the "queue" schedule, the default for larger outputs)
// the items are (chunk, tile), handed out round by round, the blocks are recycled,
// and the workgroup that completes a tile adds its chunks up itself (accumulate_tile:
// steps (iv) and (v) inside the launch); see the item loop of k_gemm.
// A launch covers a range of tiles (tile_begin, tile_count) of the band order.
//
// The stored bytes are the slice integers plus the offset of their stack (cA for A, cB for B, see
// ozimmu_layout.h), so the MFMAs sum a' b'.  The offsets are taken out by STARTING the accumulators of a
// chunk at -(ra[i] + cb[j]) instead of zero,
//     ra[i] = cB SA'[i] - pairs N cA cB,   cb[j] = cA SB'[j],
// SA' / SB' being the sums of the stored bytes of row i / column j over the chunk's slices (differences of
// the prefix sums the split kernels left behind the slices) and N the padded inner length: what the
// epilogue finds in the accumulators is then C'' itself.  With h = 2^(beta-1) and the offsets h - 1 every partial
// sum on the way is a sum of terms q_a q_b in [-h^2, h^2] and -(h-1)(q_a + q_b + h - 1) in (-3 h^2, h^2): below
// 0.75 x 4^beta x (inner length of the chunk) in magnitude, inside INT32 by the paper's choice of the chunk length.
// With `finish` set the last chunk of a tile also applies step (v) of the scheme in its epilogue:
//     out = fl(fl(alpha d) + fl(cbeta c_old))   (cbeta == 0: c_old is not read),  d the finished sum.
//
// Tiling: 256 x 256 outputs per workgroup, 4 waves in a 2 x 2 grid, each wave
// 128 x 128 = 8 x 8 tiles of v_mfma_i32_16x16x64_i8 (256 INT32 accumulators per
// lane, one wave per SIMD).  Of the two INT8 MFMA shapes of gfx950 this is the one
// the chip sustains the higher rate on (register-only loop, slice-like bytes:
// 4.09 against 3.47 POP/s for 32 x 32 x 32 - the same operations per cycle on paper,
// half the accumulator traffic per operation; the whole kernel: 10 % faster).
// A stage is one packed 16 KiB tile of A and one of B
// (256 rows x 64 inner bytes each, see ozimmu_layout.h).  Stages travel from
// global memory straight into a ring of NS LDS buffers with
// global_load_lds_dwordx4 (no VGPR staging; the bank swizzle is already in the
// packed layout, so the copy is linear), NS - 2 stages ahead of the math.
// One MFMA takes the 64 inner bytes of a stage, so a stage is one k-step of 64
// MFMAs; it runs as four quarters of 4 x 4 tiles on four sets of four operand
// fragments, each set refilled as soon as its last quarter is over, every fragment
// 16 MFMAs ahead of its first use, across stage boundaries (see `stage` in k_gemm).
// The inner order of an integer dot product is free, so each lane simply fetches
// 16 consecutive inner bytes.
//
// Synchronisation per stage `it` (buffer it % NS), one barrier:
//   quarters 0, 1 | wait until this thread's copies of stage it+1 landed |
//   barrier | quarters 2, 3, fetching the first fragments of stage it+1; copies of
//   stage it+NS-1 go into the buffer of stage it-1 (every wave has finished reading
//   it: its data fed MFMAs issued before the barrier).
// The LDS-writing loads are issued from inline assembly, so the compiler does
// not track them; the vmcnt waits that order them are written out below.
// The compiler's own memory waits use the same counter: an ordinary load (or
// a spill reload) still pending when the loop is entered would make it put a
// vmcnt wait into the loop that also waits for the copies in flight.  Hence
// every ordinary load of a chunk prologue is consumed before the loop, and the
// accumulators are pinned to their registers when they are initialised (see
// there); tests/test_kernel_codegen.py checks the generated loop for it.
// The fused epilogue of later chunks uses the same copies to bring the old values
// of D through the then idle ring (see there).
#include "ozimmu_kernels.h"
#include "ozimmu_layout.h"
#include <type_traits>

namespace {

using namespace ozl;

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int STAGE_BYTES = 2 * TILE_BYTES;       // A tile + B tile = 32 KiB
constexpr int NLOAD = TILE_BYTES / (256 * 16);    // 16-byte copies per thread and operand tile = 4
constexpr int EPI_ROWS = 8;                       // 16 x 16 tiles per batch of the plain epilogue (4 D loads in flight per lane each)
// behind the ring in LDS: (exponent, offset correction) of the tile's 256 rows and 256 columns; the work-item ticket
// (64 bytes); the list of completed tiles that the workgroup still has to add up (queue schedule, 256 bytes)
constexpr int EXP_BYTES = 2 * 256 * 8 + 64 + 256;

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

// Tile of index `lin` in the order of the queue schedule.  Its rounds are 256 consecutive indices: in band order
// 8 tile rows x 32 tile columns; when the tile grid is made of 16 x 16 blocks, one such block (blocks in
// boustrophedon order), walked as eight 8 x 4 patches, so that tickets drawn one after the other share operand
// tiles (fewer operand panels per round, 32 instead of 40: measured 0.7 to 0.9 % at 8192^3 and 16384^3).
__device__ inline void tile_of_queue(int lin, int TM, int TP, bool block_rounds, int& tm, int& tp)
{
    if (!block_rounds) {
        tile_of_linear(lin, TM, TP, tm, tp);
        return;
    }
    const int q = lin / 256, u = lin % 256;
    const int sbr = q / (TP / 16), sbc0 = q % (TP / 16);
    const int sbc = (sbr & 1) ? (TP / 16 - 1 - sbc0) : sbc0;
    const int patch = u / 32, mem = u % 32;
    tm = sbr * 16 + (patch / 4) * 8 + mem % 8;
    tp = sbc * 16 + (patch % 4) * 4 + mem / 8;
}

// Global -> LDS copies, 16 bytes per lane: lane i of the wave writes LDS bytes [M0 + offset + 16 i, + 16) with
// the 16 bytes at gbase + voff + offset (voff per lane; the instruction's offset moves both addresses alike).
// M0 carries the LDS address; one wait state must separate its write from the copy.
// Quarter Q of a wave's 4 KiB of an operand tile: the wave's lanes copy bytes [4096 w + 1024 Q + 16 lane, + 16) of
// the tile to the same place of the LDS buffer at m0_base + IMM; M0 is set for quarter 0 and used by the other three
// (nothing else in the main loop touches M0), so that three of four copies are a single instruction between two
// MFMAs (with M0 set up for every copy: 1 % slower at 16384^3).
template <int IMM, int Q>
__device__ inline void copy_tile_quarter(uint32_t m0_base, uint32_t voff, const int8_t* gbase)
{
    if constexpr (Q == 0)
        asm volatile("s_add_u32 m0, %0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3" ::"s"(m0_base), "n"(IMM),
                     "v"(voff), "s"(gbase)
                     : "memory", "scc");
    else
        asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2" ::"v"(voff), "s"(gbase), "n"(Q * 1024) : "memory");
}

// One copy with an M0 of its own and the non-temporal hint (data that is read once).
template <int IMM>
__device__ inline void copy16_to_lds_nt(uint32_t m0_base, uint32_t voff, const void* gbase)
{
    asm volatile("s_add_u32 m0, %0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3 nt" ::"s"(m0_base), "n"(IMM),
                 "v"(voff), "s"(gbase)
                 : "memory", "scc");
}

template <int N>
__device__ inline void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <int I, int N, class F>
__device__ inline void static_for(F&& f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// Layout of a 256 x 256 INT32 block of a MODE 3 launch: "lane-major".  The four accumulators of 16 x 16 tile
// (i, j) of thread t (wave t / 64 = 2 wm + wn, lane l = t % 64) are the 16 bytes at int index
// (G * 256 + t) * 4 with the group number G = ((i / 2) * 8 + j) * 2 + i % 2; they belong to rows
// wm * 128 + i * 16 + 4 (l / 16) + 0 .. 3 and column wn * 128 + j * 16 + l % 16 of the block.  A workgroup writes
// a block with 64 fully coalesced 16-byte stores per thread (256 4-byte stores in row-major order cost 10 us more
// per work item), and thread t of the workgroup that adds the tile up reads back what a thread t wrote.
constexpr int QBLOCK_GROUP_BYTES = 256 * 16;  // one group (a tile's accumulators of all 256 threads)
// Every MODE 3 launch leaves its blocks in this layout (the kernels that add the blocks of the other schedules up
// read it back with the same thread numbering); launches that cut the inner range (partial sums added with integer
// atomics) put register r of thread t of group G at int index G * 1024 + r * 256 + t instead.  Row (of register 0; registers 1 .. 3 follow) and column inside the
// 256 x 256 block of group G of thread t:
__device__ inline void lane_major_coords(int G, int t, int& row, int& col)
{
    const int wave = t >> 6, lane = t & 63;
    const int i = 2 * (G >> 4) + (G & 1), j = (G >> 1) & 7;
    row = (wave >> 1) * 128 + i * 16 + 4 * (lane >> 4);
    col = (wave & 1) * 128 + j * 16 + (lane & 15);
}

// Steps (iv) and (v) for one tile by one workgroup (the queue schedule): the tile's chunk sums lie in `w` lane-major
// INT32 blocks, `cstride` elements apart, in schedule order; every element gets them added in that order with one
// rounded FP64 addition each (Algorithm 6), exactly as k_accumulate_chunks does.  A step covers two register
// groups (8 rows x 1 column per thread) and up to 8 chunks: 16 loads of 16 bytes per thread, issued two steps
// ahead of their use, so that the loads of a step fly while the previous one is added up (three steps: spills).
// The loads are buffer loads of agent scope (they see what other XCDs have written through) and streaming (the
// 2 MiB of a tile must not displace the operand tiles that the XCD's workgroups share in L2: with plain or merely
// agent-scope loads the whole launch ran 5 % slower); D is stored non-temporally, 128 contiguous bytes per 16 lanes.
// lds_rows: 512 ints of LDS for the row and column exponents.
__device__ inline void accumulate_tile(const ozk::GemmArgs& a, const int32_t* blocks, int64_t cstride, int w, int tm,
                                       int tp, int* lds_rows)
{
    typedef int v4si __attribute__((ext_vector_type(4)));
    // (the thread index is made opaque to the optimiser: what is derived from it below is then computed here, per
    // call, and not at kernel entry, from where it would live - and be spilled - across the MFMA loop)
    int t = threadIdx.x;
    asm volatile("" : "+v"(t));
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int lc = lane & 15, lq = lane >> 4;  // the lane holds rows 4 lq .. 4 lq + 3 of column lc of a 16 x 16 tile
    const int64_t col0 = (int64_t)tp * 256 + wn * 128 + lc;  // this lane's column in column tile j: col0 + 16 j
    {
        const int64_t gr = (int64_t)tm * 256 + t, gc = (int64_t)tp * 256 + t;
        lds_rows[t] = gr < a.m ? a.eA[gr] : 0;
        lds_rows[256 + t] = gc < a.p ? a.eB[gc] : 0;
    }
    __syncthreads();
    // step u covers the register groups 2 u, 2 u + 1 of the block, tiles (2 (u / 8) + qq, u % 8): 8 rows of one
    // column per thread
    auto col_tile = [&](int u) { return u & 7; };
    auto row_in_wave = [&](int u, int qq, int ss) { return (2 * (u >> 3) + qq) * 16 + 4 * lq + ss; };
    const bool last_c = a.finish && a.cbeta != 0.0;
    double* const obase = a.finish ? a.Cout : a.D;
    const int64_t opitch = a.finish ? a.ldco : a.ldd;
    const int nbatch = (w + 7) / 8;
    const int nstep = 32 * nbatch;
    v4si v[2][8][2];
    double d[2][4];
    int g = a.g_lo, c0 = 1;
    bool first = true;
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t*>(blocks), 0, 0x7fffffff, 0x00020000);
    constexpr int POLICY = (1 << 4) | (1 << 1);
    // step (v) with cbeta != 0: the old values of C travel with the loads of the step that will store them
    double cold[2][2][4];
    auto issue = [&](auto BUF, int s) {
        constexpr int buf = decltype(BUF)::value;
        const int u = s / nbatch, cq = (s - u * nbatch) * 8;  // u = (i * 4 + j) * 2 + half
        if (last_c && s - u * nbatch == nbatch - 1) {
            const int64_t col = col0 + 16 * col_tile(u);
#pragma unroll
            for (int qq = 0; qq < 2; ++qq)
#pragma unroll
                for (int ss = 0; ss < 4; ++ss) {
                    const int64_t row = (int64_t)tm * 256 + wm * 128 + row_in_wave(u, qq, ss);
                    cold[buf][qq][ss] =
                        (col < a.p && row < a.m) ? __builtin_nontemporal_load(obase + row * opitch + col) : 0.0;
                }
        }
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const int cb = (cq + b < w) ? cq + b : w - 1;  // (past the last chunk: read it again, unused)
#pragma unroll
            for (int qq = 0; qq < 2; ++qq) {
                const int soff = (int)((int64_t)cb * cstride * 4) + (u * 2 + qq) * QBLOCK_GROUP_BYTES;
                v[buf][b][qq] = __builtin_bit_cast(v4si, __builtin_amdgcn_raw_buffer_load_b128(rsrc, t * 16, soff, POLICY));
            }
        }
    };
    auto consume = [&](auto BUF, int s) {
        constexpr int buf = decltype(BUF)::value;
        const int u = s / nbatch, bq = s - u * nbatch, cq = bq * 8;
        if (bq == 0) {
            g = a.g_lo;
            c0 = 1;
            first = true;
        }
        const int ebj = lds_rows[256 + wn * 128 + 16 * col_tile(u) + lc];
        int ea[2][4];
#pragma unroll
        for (int qq = 0; qq < 2; ++qq)
#pragma unroll
            for (int ss = 0; ss < 4; ++ss) ea[qq][ss] = lds_rows[wm * 128 + row_in_wave(u, qq, ss)];
        const int nb = (w - cq) < 8 ? (w - cq) : 8;
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            if (b < nb) {
                const int shift = 2 - a.beta * g;
#pragma unroll
                for (int qq = 0; qq < 2; ++qq)
#pragma unroll
                    for (int ss = 0; ss < 4; ++ss) {
                        const double term = ldexp((double)v[buf][b][qq][ss], ea[qq][ss] + ebj + shift);
                        d[qq][ss] = first ? term : d[qq][ss] + term;
                    }
                first = false;
                c0 += a.r;
                if (c0 > g - 1) {
                    ++g;
                    c0 = 1;
                }
            }
        }
    };
    auto store = [&](auto BUF, int s) {
        constexpr int buf = decltype(BUF)::value;
        const int u = s / nbatch, bq = s - u * nbatch;
        if (bq != nbatch - 1) return;
        const int64_t col = col0 + 16 * col_tile(u);
        if (col >= a.p) return;
#pragma unroll
        for (int qq = 0; qq < 2; ++qq)
#pragma unroll
            for (int ss = 0; ss < 4; ++ss) {
                const int64_t row = (int64_t)tm * 256 + wm * 128 + row_in_wave(u, qq, ss);
                if (row >= a.m) continue;
                double val = d[qq][ss];
                double* out = obase + row * opitch + col;
                if (a.finish) {
                    val = a.alpha * val;
                    if (last_c) val = val + a.cbeta * cold[buf][qq][ss];
                }
                __builtin_nontemporal_store(val, out);
            }
    };
    issue(std::integral_constant<int, 0>{}, 0);
    issue(std::integral_constant<int, 1>{}, 1);
    for (int s = 0; s < nstep; s += 2) {
        // (a step's stores before the buffer's next loads: those bring new old values of C into the same registers)
        consume(std::integral_constant<int, 0>{}, s);
        store(std::integral_constant<int, 0>{}, s);
        if (s + 2 < nstep) issue(std::integral_constant<int, 0>{}, s + 2);
        consume(std::integral_constant<int, 1>{}, s + 1);
        store(std::integral_constant<int, 1>{}, s + 1);
        if (s + 3 < nstep) issue(std::integral_constant<int, 1>{}, s + 3);
    }
}

// Soft barrier between the workgroups of one XCD ("team").  They share one L2 and
// stream the same A / B tiles; the L2 holds only some twenty stages of the team's
// working set, so operand reuse in L2 lives on the team advancing in lockstep
// (measured: 6.4 GB instead of 22 GB fetched from HBM per slice pair at 16384^3).
// Nothing but timing depends on it: a workgroup that has waited `spin_limit`
// polls goes on alone, so the barrier always ends.  Called by every thread;
// thread 0 arrives and polls, the rest meet it at the next s_barrier.
// Two counters at once (the whole grid, then the XCD's team): both arrivals go out before the first poll.
// Waiting for the whole grid keeps the XCDs on the same operand panels, which the memory-side cache then
// serves to all of them; it also makes every workgroup update its tile of D at the same moment, and the
// matrix cores idle while that traffic drains.  The first effect grows with the inner dimension, the
// second does not, so the host asks for the grid-wide wait only for long inner dimensions
// (`spin_limit_a` = 0 otherwise: measured 3 to 7 % faster at inner dimensions up to 8192, 1 to 3 %
// slower from 9216 on).
__device__ inline void arrive_and_wait2(unsigned* ctr_a, unsigned target_a, int spin_limit_a, unsigned* ctr_b,
                                        unsigned target_b, int spin_limit)
{
    if (threadIdx.x == 0) {
        __hip_atomic_fetch_add(ctr_a, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_fetch_add(ctr_b, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        for (int i = 0; i < spin_limit_a; ++i) {
            if (__hip_atomic_load(ctr_a, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= target_a) break;
            __builtin_amdgcn_s_sleep(8);
        }
        for (int i = 0; i < spin_limit; ++i) {
            if (__hip_atomic_load(ctr_b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= target_b) break;
            __builtin_amdgcn_s_sleep(8);
        }
    }
}

// Copy cursor: tile pointer of the next stage to copy for one operand.  The inner tiles of a slice are
// consecutive 16 KiB blocks; `groups_left` counts the groups of NS stages left in the current slice.
struct Cursor {
    const int8_t* ptr;
    int groups_left;
};

// Persistent kernel: gridDim.x workgroups (one per CU), workgroup b belongs to
// XCD b % 8 (hardware dispatch order) and is member b / 8 of that XCD's team.
// The tiles of the output are split into 8 contiguous ranges, one per XCD, in
// band order (GROUP tile rows walked column by column); in round q the team
// works on tiles q*team .. q*team+team-1 of its range, i.e. an 8 x 4 patch
// whose A and B tiles are shared through the XCD's L2.  (Tile grids made of
// 16 x 16 blocks place the eight patches of a round side by side instead, see
// below.)  For its tile a workgroup runs every chunk of the schedule in the order
// of Algorithm 6.
//
// The main loop is unrolled NS times so that every LDS address is a register
// plus an immediate and every M0 value one scalar add: with one wave per SIMD
// every instruction that is not an MFMA competes with the MFMAs for the wave's
// issue slots (one instruction per 4 cycles), so the loop carries as few of them
// as it can (per stage 64 MFMAs, 16 LDS reads, 8 copies of 3 instructions, two
// cursor updates, one barrier).
template <int MODE, int NS>
__global__ __launch_bounds__(256) void k_gemm(ozk::GemmArgs a, int TM, int TP)
{
    extern __shared__ __align__(16) int8_t lds[];
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave >> 1, wn = wave & 1;

    const int KT = a.KT;  // a multiple of NS (inner padding granule KPAD)
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)lds;
    // operand tile copies: wave w brings bytes [4096 w, 4096 w + 4096) of a tile, 1 KiB per copy
    const uint32_t m0_tile = lds_base + (uint32_t)wave * 4096u;
    const uint32_t voff_tile = (uint32_t)wave * 4096u + (uint32_t)lane * 16u;
    // moving on to the next slice pair of a chunk: A slice s -> s+1, B slice g-s -> g-s-1, inner tile KT-1 -> 0
    // (on top of the usual step of one tile)
    const int64_t wrapA = a.strideA - (int64_t)KT * TILE_BYTES;
    const int64_t wrapB = -a.strideB - (int64_t)KT * TILE_BYTES;

    // Per-lane fragment addresses: row = w*128 + i*16 + lane%16; one MFMA takes the 64 inner bytes of a stage, the
    // lanes l/16 = 0, 1, 2, 3 supplying its logical chunks 0, 3, 1, 2 (the same for A and B: the inner order of an
    // integer dot product is free).  That order keeps the fetches off each other's banks: a ds_read_b128 serves 16
    // lanes per cycle, and these are not consecutive ones - lanes 0-3, 12-15, 20-23, 24-27 go together, then 4-11,
    // 16-19, 28-31, and the same in the upper half (measured with single-wave probes under SQ_LDS_BANK_CONFLICT); with
    // rows 0-3, 12-15 of one chunk and rows 4-11 of another in a cycle, the chunk pairs (0, 3) and (1, 2) are the ones
    // whose swizzled positions c ^ (row / 4 % 4) never meet.  (Chunks in lane order: every fetch takes 8 cycles
    // instead of 4.)  i*16 rows = i*1024 bytes and does not change the swizzle; ring buffer u adds u*32 KiB.
    // ds_read offsets are 16-bit immediates, so one base register serves two ring buffers (h = u / 2).
    constexpr int NH = (NS + 1) / 2;
    uint32_t fragA[NH], fragB[NH];
    {
        const int rowA = wm * 128 + (lane & 15), rowB = wn * 128 + (lane & 15);
        const int chunk = (0x9c >> (2 * (lane >> 4))) & 3;  // 0, 3, 1, 2
#pragma unroll
        for (int h = 0; h < NH; ++h) {
            fragA[h] = lds_base + h * 2 * STAGE_BYTES + rowA * TILE_K + swizzle(rowA, chunk) * CHUNK;
            fragB[h] = lds_base + h * 2 * STAGE_BYTES + rowB * TILE_K + swizzle(rowB, chunk) * CHUNK;
            // (registers of their own: otherwise the second base is re-made from the first by an add inside the loop)
            asm volatile("" : "+v"(fragA[h]), "+v"(fragB[h]));
        }
    }
    typedef __attribute__((address_space(3))) const v4i* lds_v4i_ptr;

    // offsets of the two stacks (stored byte = slice integer + offset)
    const int cA = a.cA[0], cB = a.cB[0];
    const bool offsets = (cA | cB) != 0;

    // team geometry
    const int nwg = gridDim.x, bid = blockIdx.x;
    const int xcd = bid % NXCD, member = bid / NXCD;
    const int team = nwg / NXCD + (xcd < nwg % NXCD ? 1 : 0);
    // MODE 3 cuts the inner range of every chunk into Z parts; a work item is (part, tile), or, when the launch
    // covers all chunks of the schedule (a.nchunks > 0), (chunk, part, tile)
    const int Z = (MODE == 3) ? a.zsplit : 1;
    const bool all_chunks = (MODE == 3) && a.nchunks > 0;
    const int T = a.tile_count * Z * (all_chunks ? a.nchunks : 1);
    const int tiles_base = T / NXCD, tiles_rem = T % NXCD;
    const int range_off = xcd * tiles_base + (xcd < tiles_rem ? xcd : tiles_rem);
    const int range_cnt = tiles_base + (xcd < tiles_rem ? 1 : 0);
    unsigned* const sync_ctr = a.sync + xcd * 16;
    // launches of the same geometry may share the counters without a reset: launch number `sync_epoch` starts
    // from what its predecessors added (every work item arrives once per chunk, one chunk per such launch)
    unsigned sync_target = (unsigned)a.sync_epoch * (unsigned)range_cnt;
    // second counter for all workgroups of the grid: the XCDs walk the tile columns in the same order, so
    // lining them up at every chunk start lets B tiles fetched for one XCD serve the others from the
    // memory-side cache (measured: 0.6 % at 16384^3, nothing elsewhere)
    unsigned* const all_ctr = a.sync + 1;
    unsigned all_target = (unsigned)a.sync_epoch * (unsigned)T;

    // A launch over all chunks of the schedule hands its work items out through a counter instead: the items
    // differ in length (1 to r slice pairs), the longest come first, and whoever is free takes the next one.
    // The static ranges above would give one XCD all the long chunks.  Every workgroup leaves once the counter
    // has passed the last item.  (The counter is one of the soft-barrier words, zero at the start of a launch.)
    unsigned* const ticket_ctr = a.sync + 2;
    volatile int* const lds_ticket = reinterpret_cast<volatile int*>(lds + NS * STAGE_BYTES + 2 * 256 * 8);

    // Queue schedule: tiles this workgroup has completed (it stored the last of their blocks) and still has to add
    // up: ring of 16 entries (tile, round) in LDS; [0] head, [1] tail.  They are added up at the top of the next
    // turn of the loop below, after the next ticket has been drawn.
    volatile int* const pend = lds_ticket + 16;
    if (t == 0) {
        pend[0] = 0;
        pend[1] = 0;
    }
    for (int local = member; all_chunks || local < range_cnt; local += team) {
        int item = range_off + local;
        if (all_chunks) {
            if (t == 0) {
                if (a.xq) {
                    // Tickets in batches of 32 per XCD.  32 consecutive work items are one 8 x 4 patch of tiles of
                    // one chunk: taken by workgroups of ONE XCD at about the same time, they share their operand
                    // tiles in that XCD's L2.  (With single tickets that happens by itself only when the workgroups
                    // of an XCD happen to finish together: measured between 16 and 31.5 of 32 consecutive tickets
                    // on one XCD, 258 to 710 GB fetched, 112 to 125 ms per launch at 16384^3 with k = 8, depending
                    // on the build and the box.)  The workgroup that draws position 0 of its XCD's next batch takes
                    // 32 tickets from the global counter and publishes their base in a ring of 16 slots, tagged
                    // with the batch number; the others of the XCD read it there.  Whoever drew position 0 is
                    // running and waits for nothing, so the wait is short; it is bounded all the same (half a minute), and a
                    // workgroup whose wait ran out sets the flag behind the counters and leaves.
                    unsigned* const xq = a.xq + xcd * 40;  // [0] positions handed out; [8 + 2 s] slot s (64 bits)
                    const unsigned i = __hip_atomic_fetch_add(xq, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    const unsigned bnum = i >> 5, pos = i & 31u;
                    unsigned long long* const slot = reinterpret_cast<unsigned long long*>(xq + 8) + (bnum & 15u);
                    unsigned base = 0x7fffffffu;
                    if (pos == 0) {
                        base = __hip_atomic_fetch_add(ticket_ctr, 32u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        __hip_atomic_store(slot, ((unsigned long long)(bnum + 1) << 32) | base, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
                    } else {
                        int polls = 0;
                        for (; polls < (1 << 25); ++polls) {
                            const unsigned long long v = __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            if ((unsigned)(v >> 32) == bnum + 1) {
                                base = (unsigned)v;
                                break;
                            }
                            __builtin_amdgcn_s_sleep(2);
                        }
                        if (polls == (1 << 25)) a.done[a.tile_count + (a.tile_count + 255) / 256] = 1u;
                    }
                    const unsigned it = base + pos;
                    *lds_ticket = it > 0x7fffffffu ? 0x7fffffff : (int)it;
                } else {
                    *lds_ticket = (int)__hip_atomic_fetch_add(ticket_ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
            __syncthreads();  // (the next write to the ticket word is a whole work item away)
            item = __builtin_amdgcn_readfirstlane(*lds_ticket);
            if (a.queue_sets > 0) {
                for (;;) {
                    __syncthreads();
                    const int head = __builtin_amdgcn_readfirstlane(pend[0]), tail = __builtin_amdgcn_readfirstlane(pend[1]);
                    if (head == tail) break;
                    const int slot = 2 + 2 * (head & 15);
                    const int zt = __builtin_amdgcn_readfirstlane(pend[slot]), qr = __builtin_amdgcn_readfirstlane(pend[slot + 1]);
                    int ptm, ptp;
                    tile_of_queue(a.tile_begin + zt, TM, TP, a.queue_block_rounds != 0, ptm, ptp);
                    const int first_block = __builtin_amdgcn_readfirstlane(
                        (qr % a.queue_sets) * a.nchunks * a.queue_stride + (zt - qr * ozk::QUEUE_ROUND_TILES));
                    accumulate_tile(a, a.C + (int64_t)first_block * (256 * 256), (int64_t)a.queue_stride * (256 * 256),
                                    a.nchunks, ptm, ptp, reinterpret_cast<int*>(lds + NS * STAGE_BYTES));
                    __syncthreads();  // every thread has used what it loaded from the blocks
                    if (t == 0) {
                        __hip_atomic_fetch_add(a.done + a.tile_count + qr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        pend[0] = head + 1;
                    }
                }
            }
            if (item >= T) break;
        }
        const int round_first = local - member;
        const unsigned participants = (unsigned)((range_cnt - round_first) < team ? (range_cnt - round_first) : team);
        unsigned all_participants = 0;  // workgroups of all XCDs that work on a tile in this round
        {
            const int q = round_first / team;  // round index (the same in every XCD)
            for (int y = 0; y < NXCD; ++y) {
                const int team_y = nwg / NXCD + (y < nwg % NXCD ? 1 : 0);
                const int cnt_y = tiles_base + (y < tiles_rem ? 1 : 0);
                int left = cnt_y - q * team_y;
                left = left < 0 ? 0 : (left > team_y ? team_y : left);
                all_participants += (unsigned)left;
            }
        }
        int tm, tp;
        // MODE 3: part-major order, so that the 32 work items of a team are 32 tiles cut at the same place of
        // the inner dimension and share operand tiles in L2 like the tiles of the un-cut kernel
        // (integer divisions run on the vector unit: readfirstlane tells the compiler the results are uniform)
        int zpart = (MODE == 3) ? __builtin_amdgcn_readfirstlane((item / a.tile_count) % Z) : 0;
        int ztile = (MODE == 3) ? __builtin_amdgcn_readfirstlane(item % a.tile_count) : item;
        // Queue schedule: rounds of QR tiles, inside a round chunk-major (longest chunks first), Z = 1.  Round q puts
        // its blocks into set q % queue_sets, once round q - queue_sets has been added up (in practice long before:
        // the items of a round are all handed out before the first of the next one).
        constexpr int QR = ozk::QUEUE_ROUND_TILES;
        const bool queued = (MODE == 3) && all_chunks && a.queue_sets > 0;
        int q_round = 0, q_chunk = 0;
        if (queued) {
            const int per_round = QR * a.nchunks;
            q_round = __builtin_amdgcn_readfirstlane(item / per_round);
            const int rem = item - q_round * per_round;
            int rt = a.tile_count - q_round * QR;  // tiles of this round
            rt = rt > QR ? QR : rt;
            q_chunk = __builtin_amdgcn_readfirstlane(a.nchunks - 1 - rem / rt);
            ztile = __builtin_amdgcn_readfirstlane(q_round * QR + rem % rt);
            zpart = 0;
            if (q_round >= a.queue_sets) {
                // (Every lane polls the same word, so that the loop is uniform.  Bounded: some seconds.  Whoever
                // holds an item of that old round is running and waits for nothing, so the wait ends; if it ever
                // does not, the flag behind the counters says so.)
                unsigned* const rd = a.done + a.tile_count + (q_round - a.queue_sets);
                int polls = 0;
                while ((unsigned)__builtin_amdgcn_readfirstlane(
                           (int)__hip_atomic_load(rd, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) < (unsigned)QR) {
                    __builtin_amdgcn_s_sleep(16);
                    if (++polls > (1 << 23)) {
                        if (t == 0) a.done[a.tile_count + (a.tile_count + QR - 1) / QR] = 1u;
                        break;
                    }
                }
            }
        }
        // the INT32 block this item's chunk sums go to (MODE 3)
        const int64_t block_no =
            queued ? ((int64_t)(q_round % a.queue_sets) * a.nchunks + q_chunk) * a.queue_stride + (ztile - q_round * QR) : 0;
        // the chunks this work item runs: all of the schedule, or the one chunk given by the launch, or (all_chunks)
        // chunk number `chunk_no` of the schedule, found by walking it.  Long chunks (late groups) come first in
        // the item order, so that the short ones fill the gaps at the end.
        int it_g_lo = a.g_lo, it_g_hi = a.g_hi, it_s0 = a.s0, it_s1 = a.s1, chunk_no = 0;
        if (all_chunks) {
            chunk_no = __builtin_amdgcn_readfirstlane(queued ? q_chunk : a.nchunks - 1 - item / (a.tile_count * Z));
            int q = 0;
            for (int g = a.g_lo; g <= a.g_hi; ++g)
                for (int c0 = 1; c0 <= g - 1; c0 += a.r, ++q)
                    if (q == chunk_no) {
                        it_g_lo = it_g_hi = g;
                        it_s0 = c0;
                        it_s1 = (c0 + a.r - 1 < g - 1) ? c0 + a.r - 1 : g - 1;
                    }
            // the same in every lane: say so (operand addresses built from these go into scalar registers)
            it_g_lo = it_g_hi = __builtin_amdgcn_readfirstlane(it_g_lo);
            it_s0 = __builtin_amdgcn_readfirstlane(it_s0);
            it_s1 = __builtin_amdgcn_readfirstlane(it_s1);
            chunk_no = __builtin_amdgcn_readfirstlane(chunk_no);
        }
        if (MODE != 3 && TM % 16 == 0 && TP % 16 == 0 && nwg == 32 * NXCD && a.tile_count == TM * TP) {
            // Tile grid made of 16 x 16 blocks and a full grid of workgroups: in round q the 8 x 4 patches of
            // the eight XCDs tile block q (2 x 4 patches), so that all XCDs together stream 16 A and 16 B
            // tile rows (instead of 64 + 4 when every XCD walks a band of its own) and the memory-side cache
            // serves what another XCD has just fetched.  Blocks in boustrophedon order.  (1.4 % at 16384^3.)
            const int q = local / 32, mem = local % 32;
            const int sbr = q / (TP / 16), sbc0 = q % (TP / 16);
            const int sbc = (sbr & 1) ? (TP / 16 - 1 - sbc0) : sbc0;
            tm = sbr * 16 + (xcd / 4) * 8 + mem % 8;
            tp = sbc * 16 + (xcd % 4) * 4 + mem / 8;
        } else {
            if (queued)
                tile_of_queue(a.tile_begin + ztile, TM, TP, a.queue_block_rounds != 0, tm, tp);
            else
                tile_of_linear(a.tile_begin + ztile, TM, TP, tm, tp);
        }
        const int64_t row0 = (int64_t)tm * 256 + wm * 128;
        const int64_t col0 = (int64_t)tp * 256 + wn * 128;
        int first = a.first;
        // per row [0, 256) and column [256, 512) of the tile: scale exponents (fused modes) and the start values
        // of the chunk's accumulators (minus the offset corrections)
        int* const lds_exp = reinterpret_cast<int*>(lds + NS * STAGE_BYTES);
        int* const lds_corr = lds_exp + 512;
        if (MODE == 1) {
            // exponents of this tile's rows and columns go to LDS once (every wave is past the previous
            // tile's epilogue; the chunk prologue's barrier publishes them)
            __builtin_amdgcn_s_barrier();
            // (row / column indices fit 32 bits: outer sizes are at most 2^22; a uniform base plus a 32-bit lane
            // offset needs no 64-bit address arithmetic per lane)
            const uint32_t gr = (uint32_t)tm * 256u + (uint32_t)t, gc = (uint32_t)tp * 256u + (uint32_t)t;
            lds_exp[t] = (int64_t)gr < a.m ? a.eA[gr] : 0;
            lds_exp[256 + t] = (int64_t)gc < a.p ? a.eB[gc] : 0;
        }

        for (int g = it_g_lo; g <= it_g_hi; ++g) {
            const int s_lo = it_s0 > 0 ? it_s0 : 1;
            const int s_hi = it_s0 > 0 ? it_s1 : g - 1;
            for (int c0 = s_lo; c0 <= s_hi; c0 += a.r) {
                const int c1 = (c0 + a.r - 1 < s_hi) ? c0 + a.r - 1 : s_hi;  // chunk: s = c0..c1
                int nstage = (c1 - c0 + 1) * KT;
                int pair0 = 0, kt0 = 0;  // slice pair and inner tile this workgroup starts at
                if (MODE == 3) {
                    // part zpart of the chunk's groups of NS stages (the host keeps Z <= KT / NS: no part is empty)
                    const int groups = nstage / NS;
                    const int g0 = (int)((int64_t)zpart * groups / Z), g1 = (int)((int64_t)(zpart + 1) * groups / Z);
                    pair0 = g0 * NS / KT;
                    kt0 = g0 * NS % KT;
                    nstage = (g1 - g0) * NS;
                }
                Cursor ca = {a.SA + (int64_t)(c0 - 1 + pair0) * a.strideA + (int64_t)tm * rowblock_bytes(KT) +
                                 (int64_t)kt0 * TILE_BYTES,
                             (KT - kt0) / NS};
                Cursor cb = {a.SB + (int64_t)(g - c0 - 1 - pair0) * a.strideB + (int64_t)tp * rowblock_bytes(KT) +
                                 (int64_t)kt0 * TILE_BYTES,
                             (KT - kt0) / NS};
                // A cursor that has just copied the last inner tile of a slice jumps to the next slice pair.  The
                // bookkeeping is cut into pieces of two or three scalar instructions that the stage below puts into
                // different gaps between MFMAs (in one piece at the end of the stage it made a bubble of a dozen
                // instructions: 0.5 % of the launch): count the group and note whether the slice ends ...
                auto wrap_count = [&](Cursor& c) -> bool { return --c.groups_left == 0; };
                // ... and the cursor's step for this stage
                auto wrap_step = [&](Cursor& c, bool wr, int64_t extra) -> int64_t {
                    c.groups_left = wr ? KT / NS : c.groups_left;
                    return wr ? extra + TILE_BYTES : (int64_t)TILE_BYTES;
                };

                // 8 x 8 tiles of 16 x 16 per wave; A fragments of row tiles 0..3 / 4..7 in faL / faH, B likewise
                v4i acc[8][8];
                v4i faL[4], faH[4], fbL[4], fbH[4];
                // sub-step ss of a quarter: row tile ss against the four column tiles (by_col: column tile ss against
                // the four row tiles) - the operand that has just been fetched is the one taken one fragment per sub-step
                auto math = [&](const v4i* fa, const v4i* fb, int i0, int j0, int ss, bool by_col, int x0, int x1) {
#pragma unroll
                    for (int x = x0; x < x1; ++x) {
                        const int y = (ss & 1) ? 3 - x : x;
                        const int ii = by_col ? y : ss, jj = by_col ? ss : y;
                        acc[i0 + ii][j0 + jj] =
                            __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[ii], fb[jj], acc[i0 + ii][j0 + jj], 0, 0, 0);
                    }
                };

                // prologue: every wave is past the math of the previous chunk (the LDS ring is free),
                // stages 0 .. NS-3 and the A half of stage NS-2 go in flight, the team lines up, stage 0
                // lands, first fragments fetched
                __builtin_amdgcn_s_barrier();
                if (MODE == 2) {
                    // one scale per slice: this chunk is the single pair (c0, g - c0); every wave is past the
                    // previous epilogue, and the barriers of the main loop publish the new exponents
                    const uint32_t gr = (uint32_t)tm * 256u + (uint32_t)t, gc = (uint32_t)tp * 256u + (uint32_t)t;
                    const int32_t* ea_s = a.eA + (int64_t)(c0 - 1) * a.estrideA;       // uniform
                    const int32_t* eb_t = a.eB + (int64_t)(g - c0 - 1) * a.estrideB;
                    lds_exp[t] = (int64_t)gr < a.m ? ea_s[gr] : 0;
                    lds_exp[256 + t] = (int64_t)gc < a.p ? eb_t[gc] : 0;
                }
                // sums of the stored bytes over the chunk's slices (A: c0 .. c1, B: g - c1 .. g - c0) for this
                // thread's row and column of the tile, as differences of prefix sums; the loads are in flight
                // while the first stages are issued and the team lines up, the corrections go to LDS after that
                int sumA = 0, sumB = 0;
                if (offsets) {
                    // row / column inside the padded stacks; uniform slice bases plus a 32-bit lane offset (opaque, so
                    // that no per-lane 64-bit address is formed once per tile and kept alive through the chunks)
                    uint32_t gr = (uint32_t)tm * 256u + (uint32_t)t, gc = (uint32_t)tp * 256u + (uint32_t)t;
                    asm volatile("" : "+v"(gr), "+v"(gc));
                    const int t_lo = g - c1, t_hi = g - c0;
                    const int32_t* pa_hi = a.PA + (int64_t)(c1 - 1) * a.pstrideA;
                    const int32_t* pa_lo = a.PA + (int64_t)(c0 > 1 ? c0 - 2 : 0) * a.pstrideA;
                    const int32_t* pb_hi = a.PB + (int64_t)(t_hi - 1) * a.pstrideB;
                    const int32_t* pb_lo = a.PB + (int64_t)(t_lo > 1 ? t_lo - 2 : 0) * a.pstrideB;
                    sumA = pa_hi[gr] - (c0 > 1 ? pa_lo[gr] : 0);
                    sumB = pb_hi[gc] - (t_lo > 1 ? pb_lo[gc] : 0);
                }
                static_for<0, NS - 1>([&](auto S) {
                    constexpr int sidx = decltype(S)::value;
                    static_for<0, NLOAD>([&](auto Q) {
                        constexpr int q = decltype(Q)::value;
                        copy_tile_quarter<sidx * STAGE_BYTES, q>(m0_tile, voff_tile, ca.ptr);
                    });
                    ca.ptr += TILE_BYTES;
                    if constexpr (sidx < NS - 2) {
                        static_for<0, NLOAD>([&](auto Q) {
                            constexpr int q = decltype(Q)::value;
                            copy_tile_quarter<sidx * STAGE_BYTES + TILE_BYTES, q>(m0_tile, voff_tile, cb.ptr);
                        });
                        cb.ptr += TILE_BYTES;
                    }
                });
                sync_target += participants;
                all_target += all_participants;
                // (launches whose work items are not lined up - spin limits 0 - leave the counters alone)
                if (a.spin_limit | a.grid_spin_limit)
                    arrive_and_wait2(all_ctr, all_target, a.grid_spin_limit, sync_ctr, sync_target, a.spin_limit);
                {
                    // every wave is past the previous chunk (first barrier above); the barrier below publishes
                    const uint32_t pairs_n = (uint32_t)(c1 - c0 + 1) * (uint32_t)(KT * TILE_K);
                    lds_corr[t] = (int)(pairs_n * (uint32_t)(cA * cB) - (uint32_t)cB * (uint32_t)sumA);  // -ra
                    lds_corr[256 + t] = (int)(0u - (uint32_t)cA * (uint32_t)sumB);                       // -cb
                }
                wait_vmcnt<NLOAD*(2 * (NS - 2) - 1)>();
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    faL[i] = *(lds_v4i_ptr)(uintptr_t)(fragA[0] + i * 1024);
                    fbL[i] = *(lds_v4i_ptr)(uintptr_t)(fragB[0] + TILE_BYTES + i * 1024);
                }
                // accumulators start at -(ra[row] + cb[column]) (see the head of this file); of a chunk that is cut
                // into parts (MODE 3) only part 0 carries the start value, the others start at zero
                {
                    // lane parts of the LDS addresses made opaque here: otherwise the addresses are formed at kernel
                    // entry, live through everything and get spilled
                    int lqi = lane >> 4, lci = lane & 15;
                    asm volatile("" : "+v"(lqi), "+v"(lci));
                    int ncb[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) ncb[j] = lds_corr[256 + wn * 128 + j * 16 + lci];
                    const bool carries = (MODE != 3) || zpart == 0;
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        int nra[4];
#pragma unroll
                        for (int r = 0; r < 4; ++r) nra[r] = lds_corr[wm * 128 + i * 16 + 4 * lqi + r];
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
#pragma unroll
                            for (int r = 0; r < 4; ++r) acc[i][j][r] = carries ? (int)((uint32_t)nra[r] + (uint32_t)ncb[j]) : 0;
                            // the tile goes to its accumulation registers now, not when the first MFMA asks for it
                            // (256 start values waiting in ordinary registers would not fit)
                            asm volatile("" : "+a"(acc[i][j]));
                            __builtin_amdgcn_sched_barrier(0);
                        }
                    }
                }

                // One stage whose ring buffer index U is a compile-time constant: one k-step of 64 MFMAs (a
                // 16 x 16 x 64 MFMA takes the 64 inner bytes of a stage at once), run as four quarters of 4 x 4 tiles.
                // Stages in even position: (A lo, B lo), (A lo, B hi), (A hi, B hi), (A hi, B lo); odd: (A lo, B hi),
                // (A lo, B lo), (A hi, B lo), (A hi, B hi) - every quarter shares one fragment set with the one
                // before, and the set that has just come free takes the fragments needed two quarters later (after
                // the barrier in mid-stage: those of the next stage).  A quarter takes the set that was fetched last
                // one fragment per sub-step (by columns when that is a B set), so that every fragment is fetched four
                // sub-steps = 16 MFMAs ahead of its first use.  Per sub-step 1 fetch, 4 MFMAs and, every other time,
                // 1 copy.  The stage copied in position u is NS-1 (A half) or NS-2 (B half) ahead, so a cursor reaches
                // the end of a slice in one fixed position of the unrolled group: A in position 0, B in position 1.
                // In the last group of a chunk (TAIL) the copies that would run past the chunk are left out.
                auto stage = [&](auto U, auto TAIL) {
                    constexpr int u = decltype(U)::value;
                    constexpr bool tail = decltype(TAIL)::value;
                    constexpr bool odd = (u % 2) != 0;
                    constexpr int un = (u + 1) % NS, up = (u + NS - 1) % NS, ub = (u + NS - 2) % NS;
                    constexpr bool copy_b = !tail || u < 2;
                    constexpr bool copy_a = !tail || u < 1;
                    constexpr bool fetch_next = !tail || u < NS - 1;
                    constexpr uint32_t curA = (u % 2) * STAGE_BYTES, curB = (u % 2) * STAGE_BYTES + TILE_BYTES;
                    constexpr uint32_t nxtA = (un % 2) * STAGE_BYTES, nxtB = (un % 2) * STAGE_BYTES + TILE_BYTES;
                    // the B set the stage starts on (column tiles j_first ..) and the other one
                    v4i* const fb_first = odd ? fbH : fbL;
                    v4i* const fb_other = odd ? fbL : fbH;
                    constexpr int j_first = odd ? 4 : 0, j_other = odd ? 0 : 4;
                    // a sub-step: one fetch, two MFMAs, a copy or a piece of cursor bookkeeping (taking turns), two
                    // MFMAs - a 4-pass MFMA leaves three issue slots behind it, and whatever does not fit delays the next
                    constexpr bool wraps_b = copy_b && u == 1 && !tail, wraps_a = copy_a && u == 0 && !tail;
                    bool wr_b = false, wr_a = false;
                    int64_t step_b = TILE_BYTES, step_a = TILE_BYTES;
                    // quarter 0: B fragments of the other half of this stage come in
                    static_for<0, 4>([&](auto Q) {
                        constexpr int q = decltype(Q)::value;
                        fb_other[q] = *(lds_v4i_ptr)(uintptr_t)(fragB[u / 2] + curB + (j_other + q) * 1024);
                        math(faL, fb_first, 0, j_first, q, true, 0, 2);
                        __builtin_amdgcn_sched_barrier(0);
                        if constexpr (copy_b && q % 2 == 0)
                            copy_tile_quarter<ub * STAGE_BYTES + TILE_BYTES, q / 2>(m0_tile, voff_tile, cb.ptr);
                        if constexpr (wraps_b && q == 1) wr_b = wrap_count(cb);
                        if constexpr (wraps_b && q == 3) step_b = wrap_step(cb, wr_b, wrapB);
                        math(faL, fb_first, 0, j_first, q, true, 2, 4);
                        __builtin_amdgcn_sched_barrier(0);
                    });
                    // quarter 1: A fragments of the upper half of this stage
                    static_for<0, 4>([&](auto Q) {
                        constexpr int q = decltype(Q)::value;
                        faH[q] = *(lds_v4i_ptr)(uintptr_t)(fragA[u / 2] + curA + (4 + q) * 1024);
                        math(faL, fb_other, 0, j_other, q, true, 0, 2);
                        __builtin_amdgcn_sched_barrier(0);
                        if constexpr (copy_b && q % 2 == 0)
                            copy_tile_quarter<ub * STAGE_BYTES + TILE_BYTES, 2 + q / 2>(m0_tile, voff_tile, cb.ptr);
                        if constexpr (copy_b && q == 3) cb.ptr += step_b;
                        math(faL, fb_other, 0, j_other, q, true, 2, 4);
                        __builtin_amdgcn_sched_barrier(0);
                    });
                    if constexpr (tail && u >= 2)
                        wait_vmcnt<0>();
                    else
                        wait_vmcnt<2 * NLOAD * (NS - 3)>();
                    __builtin_amdgcn_s_barrier();
                    asm volatile("" ::: "memory");
                    // quarter 2: first A fragments of the next stage
                    static_for<0, 4>([&](auto Q) {
                        constexpr int q = decltype(Q)::value;
                        if constexpr (fetch_next) faL[q] = *(lds_v4i_ptr)(uintptr_t)(fragA[un / 2] + nxtA + q * 1024);
                        math(faH, fb_other, 4, j_other, q, false, 0, 2);
                        __builtin_amdgcn_sched_barrier(0);
                        if constexpr (copy_a && q % 2 == 0)
                            copy_tile_quarter<up * STAGE_BYTES, q / 2>(m0_tile, voff_tile, ca.ptr);
                        if constexpr (wraps_a && q == 1) wr_a = wrap_count(ca);
                        if constexpr (wraps_a && q == 3) step_a = wrap_step(ca, wr_a, wrapA);
                        math(faH, fb_other, 4, j_other, q, false, 2, 4);
                        __builtin_amdgcn_sched_barrier(0);
                    });
                    // quarter 3: the B fragments the next stage starts with (its first set is this stage's other one)
                    static_for<0, 4>([&](auto Q) {
                        constexpr int q = decltype(Q)::value;
                        if constexpr (fetch_next)
                            fb_other[q] = *(lds_v4i_ptr)(uintptr_t)(fragB[un / 2] + nxtB + (j_other + q) * 1024);
                        math(faH, fb_first, 4, j_first, q, false, 0, 2);
                        __builtin_amdgcn_sched_barrier(0);
                        if constexpr (copy_a && q % 2 == 0)
                            copy_tile_quarter<up * STAGE_BYTES, 2 + q / 2>(m0_tile, voff_tile, ca.ptr);
                        if constexpr (copy_a && q == 3) ca.ptr += step_a;
                        math(faH, fb_first, 4, j_first, q, false, 2, 4);
                        __builtin_amdgcn_sched_barrier(0);
                    });
                };
                static_assert(NS == 4, "the tail logic below is written for a ring of 4 stages");
                for (int it = 0; it < nstage - NS; it += NS)
                    static_for<0, NS>([&](auto U) { stage(U, std::false_type{}); });
                static_for<0, NS>([&](auto U) { stage(U, std::true_type{}); });
                wait_vmcnt<0>();  // no copy may still be writing LDS when the ring is reused or the workgroup retires
                if constexpr (MODE == 1 || MODE == 2) {
                    // (the fused epilogues are long: left alone, the register allocator parks three tiles of
                    // accumulators in scratch memory during the last stage and reloads them a dozen times)
#pragma unroll
                    for (int i = 0; i < 8; ++i)
#pragma unroll
                        for (int j = 0; j < 8; ++j) asm volatile("" : "+a"(acc[i][j]));
                }

                // Epilogue.  Accumulator register r of tile (i, j) in lane l holds output row 4*(l/16) + r and
                // column l%16 of that 16 x 16 tile.  Addresses are a wave-uniform base plus a 32-bit lane offset,
                // rebuilt for every chunk (the empty asm keeps the compiler from hoisting 64 element addresses per
                // lane out of the chunk loops).
                const int shift = MODE == 2 ? 2 - 2 * a.beta : 2 - a.beta * g;
                int64_t er0 = row0, ec0 = col0;
                asm volatile("" : "+s"(er0), "+s"(ec0));
                // lane parts of the output coordinates, opaque to the optimiser so that the per-lane row indices of
                // a chunk are formed here and not at kernel entry (where they would be spilled)
                int lqe = lane >> 4, lce = lane & 15;
                asm volatile("" : "+v"(lqe), "+v"(lce));
                if (MODE == 3) {
                    // The whole block, lane-major (see lane_major_coords), written through: in the queue schedule
                    // another XCD's workgroup may add the tile up.  No bounds: rows and columns past the edge of D exist
                    // in the block.  The block: the queue's, or block (chunk, tile) of the launch.
                    const int64_t blk = queued ? block_no : (int64_t)chunk_no * a.tile_count + ztile;
                    int32_t* const bptr = a.C + (int64_t)__builtin_amdgcn_readfirstlane((int)blk) * (256 * 256);
                    int voff = lqe * 256 + lce * 16 + wave * 1024;  // 16 t, from the lane parts made opaque above
                    asm volatile("" : "+v"(voff));
                    if (Z > 1) {
                        // partial sum of one part of the inner range: integer adds commute, the block starts at zero
#pragma unroll
                        for (int i = 0; i < 8; ++i)
#pragma unroll
                            for (int j = 0; j < 8; ++j)
#pragma unroll
                                for (int r = 0; r < 4; ++r)
                                    // (register r of all 256 threads side by side inside the group: 64 consecutive
                                    // integers per wave and instruction; in lane-major order, 16 bytes apart, the
                                    // atomics take twice as long)
                                    __hip_atomic_fetch_add(bptr + (((i >> 1) * 8 + j) * 2 + (i & 1)) * (QBLOCK_GROUP_BYTES / 4) +
                                                               r * 256 + (voff >> 4),
                                                           acc[i][j][r], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    } else {
                        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(bptr, 0, 256 * 256 * 4, 0x00020000);
#pragma unroll
                        for (int i = 0; i < 8; ++i)
#pragma unroll
                            for (int j = 0; j < 8; ++j) {
                                typedef int v4si __attribute__((ext_vector_type(4)));
                                // (through ordinary registers, said explicitly: asked to store the accumulation
                                // registers directly, the register allocator spills whole tiles; and one group at a
                                // time: left alone, the scheduler copies all 256 accumulators first)
                                int x0 = acc[i][j][0], x1 = acc[i][j][1], x2 = acc[i][j][2], x3 = acc[i][j][3];
                                asm volatile("" : "+v"(x0), "+v"(x1), "+v"(x2), "+v"(x3));
                                const v4si val = {x0, x1, x2, x3};
                                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(__attribute__((__vector_size__(4 * sizeof(unsigned int)))) unsigned int, val),
                                                                       rsrc, voff, (((i >> 1) * 8 + j) * 2 + (i & 1)) * QBLOCK_GROUP_BYTES, 1 << 4);
                                __builtin_amdgcn_sched_barrier(0);
                            }
                    }
                } else if (MODE == 0) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const bool col_ok = ec0 + 16 * j + lce < a.p;
#pragma unroll
                        for (int i = 0; i < 8; ++i)
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                const int64_t urow = er0 + i * 16 + r;  // (the lane's row: + 4 lqe)
                                int32_t* base = a.C + urow * a.ldc + ec0 + j * 16;
                                const uint32_t off = (uint32_t)(4 * lqe) * (uint32_t)a.ldc + (uint32_t)lce;
                                if (col_ok && urow + 4 * lqe < a.m) base[off] = acc[i][j][r];
                            }
                    }
                } else {
                    // Exponents come from LDS (the compiler cannot prove that D does not alias eA / eB and would
                    // order global exponent loads behind every store).  D is
                    // touched once per chunk, a millisecond apart: non-temporal accesses keep it from displacing
                    // the operand tiles the team shares in L2 (1 % at 16384^3).
                    // The last chunk of a tile applies step (v) when asked to (finish): its result goes to Cout.
                    const bool last = a.finish && g == a.g_hi && c1 == s_hi;
                    const bool with_c = last && a.cbeta != 0.0;
                    // the FP64 addend of this chunk for accumulator (i, j, r)
                    auto addend = [&](int i, int j, int r) -> double {
                        const int ea = lds_exp[wm * 128 + i * 16 + 4 * lqe + r];
                        const int eb = lds_exp[256 + wn * 128 + j * 16 + lce];
                        return ldexp((double)acc[i][j][r], ea + eb + shift);
                    };
                    const uint32_t off = (uint32_t)(4 * lqe) * (uint32_t)a.ldd + (uint32_t)lce;
                    // Later chunks of a tile that lies wholly inside D (and D aligned for 16-byte copies): the old
                    // values of D come in through the LDS ring, which is idle now, with the same global -> LDS
                    // copies as the operands.  They need no registers, so the next half block (64 rows x 32
                    // columns of this wave) is already on its way while the current one is added and stored, and
                    // no load ever waits for a store to be acknowledged.  Wave w owns ring buffer w (32 KiB = two
                    // half blocks).  Copy t of a half block brings rows 4t .. 4t+3 into 1 KiB: lane l row l / 16,
                    // columns 2 c, 2 c + 1 with c = l % 16 for even t and (l % 16) ^ 8 for odd t.  The swap of the two
                    // 16-column halves in every other copy keeps the reads below off each other's banks: lanes
                    // 0 .. 15 read 128 bytes of one row, lanes 16 .. 31 the same columns four rows (one copy) on.
                    const bool staged = !first && !with_c && a.dma_ok && (int64_t)tm * 256 + 256 <= a.m &&
                                        (int64_t)tp * 256 + 256 <= a.p;
                    if (staged) {
                        __builtin_amdgcn_s_barrier();  // every wave has read its last fragments from the ring
                        const uint32_t region = lds_base + (uint32_t)wave * (uint32_t)STAGE_BYTES;
                        // lane-dependent offsets are rebuilt here (the empty asm keeps them from being computed at
                        // kernel entry and held in registers through the main loop)
                        uint32_t ln = (uint32_t)lane;
                        asm volatile("" : "+v"(ln));
                        const uint32_t dvoff[2] = {((ln >> 4) * (uint32_t)a.ldd + (ln & 15u) * 2u) * 8u,
                                                   ((ln >> 4) * (uint32_t)a.ldd + ((ln & 15u) ^ 8u) * 2u) * 8u};
                        // this lane's element of column tile jj (0, 1) of the half block, row 4 (ln / 16) of row tile 0
                        const uint32_t lq1 = (ln >> 4) & 1u, lc = ln & 15u;
                        const uint32_t rd_lane[2] = {region + (ln >> 4) * 1024u + (lq1 * 8u + (lc >> 1)) * 16u + (lc & 1u) * 8u,
                                                     region + (ln >> 4) * 1024u + ((lq1 ^ 1u) * 8u + (lc >> 1)) * 16u + (lc & 1u) * 8u};
                        const int64_t row_step = 4 * a.ldd;  // elements between the rows of consecutive copies
                        auto issue = [&](auto HB) {          // half block hb = 2 j + h into buffer hb % 2
                            constexpr int hb = decltype(HB)::value, j = hb / 2, h = hb % 2;
                            const double* gp = a.D + (er0 + 64 * h) * a.ldd + ec0 + 32 * j;
                            static_for<0, 16>([&](auto TT) {
                                constexpr int tt = decltype(TT)::value;
                                asm volatile("" : "+s"(gp));  // one running pointer, not sixteen precomputed ones
                                copy16_to_lds_nt<(hb % 2) * 16384 + tt * 1024>(region, dvoff[tt % 2], gp);
                                gp += row_step;
                            });
                        };
                        typedef __attribute__((address_space(3))) const double* lds_f64_ptr;
                        const double alpha = last ? a.alpha : 1.0;  // fl(1.0 * x) = x
                        issue(std::integral_constant<int, 0>{});
                        issue(std::integral_constant<int, 1>{});
                        static_for<0, 8>([&](auto HB) {
                            constexpr int hb = decltype(HB)::value, j = hb / 2, h = hb % 2;
                            // copies of half block hb have landed; later ones and the stores may still fly
                            if constexpr (hb == 0)
                                wait_vmcnt<16>();
                            else if constexpr (hb == 7)
                                wait_vmcnt<32>();
                            else
                                wait_vmcnt<48>();
                            asm volatile("" ::: "memory");
#pragma unroll
                            for (int ip = 0; ip < 2; ++ip) {  // two row tiles at a time: 16 values per lane
                                double old[2][2][4];
#pragma unroll
                                for (int ii = 0; ii < 2; ++ii)
#pragma unroll
                                    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                                        for (int r = 0; r < 4; ++r)
                                            old[ii][jj][r] = *(lds_f64_ptr)(uintptr_t)(rd_lane[jj] + (hb % 2) * 16384 +
                                                                                       (2 * ip + ii) * 4096 + r * 256);
#pragma unroll
                                for (int ii = 0; ii < 2; ++ii)
#pragma unroll
                                    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                                        for (int r = 0; r < 4; ++r) {
                                            const int i = 4 * h + 2 * ip + ii, jt = 2 * j + jj;
                                            const int64_t urow = er0 + i * 16 + r;
                                            double* base = a.D + urow * a.ldd + ec0 + jt * 16;
                                            __builtin_nontemporal_store(alpha * (old[ii][jj][r] + addend(i, jt, r)), &base[off]);
                                        }
                                __builtin_amdgcn_sched_barrier(0);
                            }
                            // the buffer is read out (the sums above needed every value): refill it
                            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                            if constexpr (hb + 2 < 8) issue(std::integral_constant<int, hb + 2>{});
                            __builtin_amdgcn_sched_barrier(0);
                        });
                    } else {
                        // Edge tiles, first chunks, unaligned D, and the last chunk when it also reads the old C:
                        // per column of 16 x 16 tiles and per batch of ROWS row tiles, 4 ROWS loads of D (and of C)
                        // in flight, then the adds and stores.
                        auto plain = [&](auto ROWS, auto WITH_C, auto LAST) {
                            constexpr int rows = decltype(ROWS)::value;
                            constexpr bool wc = decltype(WITH_C)::value;
                            constexpr bool fin = decltype(LAST)::value;
                            const uint32_t offc = (uint32_t)(4 * lqe) * (uint32_t)a.ldco + (uint32_t)lce;
#pragma unroll
                            for (int j = 0; j < 8; ++j) {
                                const bool col_ok = ec0 + 16 * j + lce < a.p;
#pragma unroll
                                for (int ih = 0; ih < 8; ih += rows) {
                                    double old[rows][4], cold[wc ? rows : 1][4];
                                    if (!first) {
#pragma unroll
                                        for (int i = 0; i < rows; ++i)
#pragma unroll
                                            for (int r = 0; r < 4; ++r) {
                                                const int64_t urow = er0 + (ih + i) * 16 + r;
                                                const double* base = a.D + urow * a.ldd + ec0 + j * 16;
                                                old[i][r] = (col_ok && urow + 4 * lqe < a.m) ? __builtin_nontemporal_load(&base[off]) : 0.0;
                                            }
                                    }
                                    if constexpr (wc) {
#pragma unroll
                                        for (int i = 0; i < rows; ++i)
#pragma unroll
                                            for (int r = 0; r < 4; ++r) {
                                                const int64_t urow = er0 + (ih + i) * 16 + r;
                                                const double* cbase = a.Cout + urow * a.ldco + ec0 + j * 16;
                                                cold[i][r] = (col_ok && urow + 4 * lqe < a.m) ? __builtin_nontemporal_load(&cbase[offc]) : 0.0;
                                            }
                                    }
                                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                                    for (int i = 0; i < rows; ++i) {
#pragma unroll
                                        for (int r = 0; r < 4; ++r) {
                                            const int64_t urow = er0 + (ih + i) * 16 + r;
                                            const double term = addend(ih + i, j, r);
                                            double val = first ? term : (old[i][r] + term);
                                            if constexpr (fin) {
                                                val = a.alpha * val;                                   // t1 = fl(alpha d)
                                                if constexpr (wc) val = val + a.cbeta * cold[i][r];    // fl(t1 + fl(cbeta c))
                                                double* cbase = a.Cout + urow * a.ldco + ec0 + j * 16;
                                                if (col_ok && urow + 4 * lqe < a.m) __builtin_nontemporal_store(val, &cbase[offc]);
                                            } else {
                                                double* base = a.D + urow * a.ldd + ec0 + j * 16;
                                                if (col_ok && urow + 4 * lqe < a.m) __builtin_nontemporal_store(val, &base[off]);
                                            }
                                        }
                                    }
                                    __builtin_amdgcn_sched_barrier(0);
                                }
                            }
                        };
                        if (with_c)
                            plain(std::integral_constant<int, EPI_ROWS / 2>{}, std::true_type{}, std::true_type{});
                        else if (last)
                            plain(std::integral_constant<int, EPI_ROWS>{}, std::false_type{}, std::true_type{});
                        else
                            plain(std::integral_constant<int, EPI_ROWS>{}, std::false_type{}, std::false_type{});
                    }
                }
                first = 0;
            }
        }
        if (queued) {
            // This item's block is complete.  The workgroup that completes the last block of a tile adds the
            // tile's chunks up.  No cache-wide fence (its L2 write-back and invalidation would cost every workgroup
            // of the XCD its operand tiles): the blocks are stored and loaded with agent-scope accesses, which go
            // through to memory, every thread waits for its stores to be acknowledged before the counter is
            // touched, and the loads of the adding workgroup are issued after it has seen the count.
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            if (t == 0)
                lds_ticket[1] = (int)__hip_atomic_fetch_add(a.done + ztile, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
            if (__builtin_amdgcn_readfirstlane(lds_ticket[1]) == a.nchunks - 1 && t == 0) {
                const int tail = pend[1];  // (at most one entry is ever waiting: the list is emptied every turn)
                pend[2 + 2 * (tail & 15)] = ztile;
                pend[3 + 2 * (tail & 15)] = q_round;
                pend[1] = tail + 1;
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

// Step (iv) for a range of tiles whose INT32 chunk sums lie in per-tile lane-major 256 x 256 blocks (the
// split-inner schedule); the blocks are cleared after use for the next chunk's integer atomics.
// A workgroup handles two groups of a block: thread t the 8 rows x 1 column that thread t of the GEMM held there.
// t.finish: step (v) on the result.
__global__ __launch_bounds__(256) void k_accumulate_tiles(ozk::TileAccArgs t)
{
    const int local = blockIdx.x / 32, sub = blockIdx.x % 32;
    int tm, tp;
    tile_of_linear(t.tile_begin + local, t.TM, t.TP, tm, tp);
    typedef int v4si __attribute__((ext_vector_type(4)));
    for (int gq = 0; gq < 2; ++gq) {
        const int G = 2 * sub + gq;
        int row, col;
        lane_major_coords(G, (int)threadIdx.x, row, col);
        v4si v;
        if (t.parts > 1) {
            int32_t* c = t.Ct + (int64_t)local * (256 * 256) + G * 1024 + threadIdx.x;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                v[q] = c[q * 256];
                c[q * 256] = 0;
            }
        } else {
            v4si* c = reinterpret_cast<v4si*>(t.Ct + (int64_t)local * (256 * 256)) + G * 256 + threadIdx.x;
            v = *c;
            *c = (v4si){0, 0, 0, 0};
        }
        const int64_t j = (int64_t)tp * 256 + col;
        if (j >= t.p) continue;
        const int eb = t.eB[j] + t.shift;
        for (int q = 0; q < 4; ++q) {
            const int64_t i = (int64_t)tm * 256 + row + q;
            if (i >= t.m) break;
            const double term = ldexp((double)v[q], t.eA[i] + eb);
            double* d = t.D + i * t.ldd + j;
            double val = t.first ? term : (*d + term);
            if (t.finish) {
                val = t.alpha * val;
                double* out = t.Cout + i * t.ldco + j;
                if (t.cbeta != 0.0) val = val + t.cbeta * *out;
                *out = val;
            } else {
                *d = val;
            }
        }
    }
}

// Step (iv) over all chunks of the schedule for a range of tiles: chunk q's INT32 sums lie in lane-major blocks
// Ct[q * tile_count + tile]; D = fl(...fl(fl(T_1 + T_2) + T_3)...) in schedule order (g ascending, chunks of r
// ascending), T_q = 2^(2 - beta g) diag(2^eA) FP64(C''_q) diag(2^eB), the first addend taken as it is.
// Work split as in k_accumulate_tiles.
__global__ __launch_bounds__(256) void k_accumulate_chunks(ozk::TileAccArgs t, int k, int r, int beta)
{
    const int local = blockIdx.x / 32, sub = blockIdx.x % 32;
    int tm, tp;
    tile_of_linear(t.tile_begin + local, t.TM, t.TP, tm, tp);
    typedef int v4si __attribute__((ext_vector_type(4)));
    const int64_t chunk_stride = (int64_t)t.tile_count * (256 * 256);
    for (int gq = 0; gq < 2; ++gq) {
        const int G = 2 * sub + gq;
        int row, col;
        lane_major_coords(G, (int)threadIdx.x, row, col);
        const int64_t j = (int64_t)tp * 256 + col;
        if (j >= t.p) continue;
        const int eb = t.eB[j];
        int e[4];
        for (int q = 0; q < 4; ++q) {
            const int64_t i = (int64_t)tm * 256 + row + q;
            e[q] = i < t.m ? t.eA[i] + eb : 0;
        }
        const int32_t* c = t.Ct + (int64_t)local * (256 * 256) + G * 1024 + (t.parts > 1 ? (int)threadIdx.x : 4 * (int)threadIdx.x);
        double d[4] = {0.0, 0.0, 0.0, 0.0};
        bool first = true;
        for (int g = 2; g <= k + 1; ++g)
            for (int c0 = 1; c0 <= g - 1; c0 += r, c += chunk_stride) {
                v4si v;
                if (t.parts > 1) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) v[q] = c[q * 256];
                } else {
                    v = *reinterpret_cast<const v4si*>(c);
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const double term = ldexp((double)v[q], e[q] + 2 - beta * g);
                    d[q] = first ? term : d[q] + term;
                }
                first = false;
            }
        for (int q = 0; q < 4; ++q) {
            const int64_t i = (int64_t)tm * 256 + row + q;
            if (i >= t.m) break;
            double val = d[q];
            double* out = t.D + i * t.ldd + j;
            if (t.finish) {
                val = t.alpha * val;
                out = t.Cout + i * t.ldco + j;
                if (t.cbeta != 0.0) val = val + t.cbeta * *out;
            }
            *out = val;
        }
    }
}

__global__ __launch_bounds__(256) void k_zero_f64(int64_t m, int64_t p, double* __restrict__ D, int64_t ldd)
{
    const int64_t j = (int64_t)blockIdx.y * 256 + threadIdx.x;
    const int64_t i = blockIdx.x;
    if (j < p && i < m) D[i * ldd + j] = 0.0;
}

__global__ __launch_bounds__(256) void k_zero_i32_2d(int64_t m, int64_t p, int32_t* __restrict__ C, int64_t ldc)
{
    const int64_t j = (int64_t)blockIdx.y * 256 + threadIdx.x;
    const int64_t i = blockIdx.x;
    if (j < p && i < m) C[i * ldc + j] = 0;
}

// Step (v) of the scheme: c <- fl(fl(alpha d) + fl(beta c)); beta == 0 leaves the old c unread.
// HBM-bound: 8 bytes read (16 with beta != 0) and 8 written per element.
__global__ __launch_bounds__(256) void k_axpby(int64_t m, int64_t p, double alpha, const double* __restrict__ D,
                                               int64_t ldd, double beta, double* __restrict__ C, int64_t ldc)  // D == nullptr: D = 0
{
    const int64_t j = (int64_t)blockIdx.y * 256 + threadIdx.x;
    const int64_t i0 = (int64_t)blockIdx.x * 8;
    if (j >= p) return;
    for (int64_t i = i0; i < i0 + 8 && i < m; ++i) {
        const double t1 = D ? alpha * D[i * ldd + j] : 0.0;
        double* c = C + i * ldc + j;
        if (beta == 0.0) {
            *c = t1;
        } else {
            const double t2 = beta * *c;
            *c = t1 + t2;
        }
    }
}

__global__ __launch_bounds__(256) void k_zero_i32(int64_t count, int32_t* __restrict__ x)
{
    // 16 bytes per thread where the array allows it (x is 16-byte aligned: blocks and counters of the workspace)
    typedef int v4si __attribute__((ext_vector_type(4)));
    const int64_t i0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i0 + 3 < count && (reinterpret_cast<uintptr_t>(x) & 15) == 0) {
        *reinterpret_cast<v4si*>(x + i0) = (v4si){0, 0, 0, 0};
        return;
    }
#pragma unroll
    for (int q = 0; q < 4; ++q)
        if (i0 + q < count) x[i0 + q] = 0;
}

// zero the soft-barrier counters (a kernel rather than a memset so that the call can be captured in a graph)
__global__ void k_fill_u32_gemm(unsigned* x) { x[threadIdx.x] = 0u; }

constexpr int NSTAGES = 4;  // ring depth: 4 x 32 KiB of the 160 KiB LDS (3 and 5 measured no faster)

}  // namespace

namespace ozk {

hipError_t launch_gemm(const GemmArgs& a_in, int fused, hipStream_t st)
{
    GemmArgs a = a_in;
    // the fused epilogue may fetch the old D through LDS with 16-byte copies: needs the alignment for them
    a.dma_ok = (fused == 1 || fused == 2) && reinterpret_cast<uintptr_t>(a.D) % 16 == 0 && a.ldd % 2 == 0 &&
               4 * a.ldd * 8 < ((int64_t)1 << 31);
    const int TM = (int)(ozl::rows_padded(a.m) / ozl::TILE_R), TP = (int)(ozl::rows_padded(a.p) / ozl::TILE_R);
    const size_t smem = (size_t)NSTAGES * STAGE_BYTES + EXP_BYTES;
    // one workgroup per CU (the LDS ring allows no second one), never more workgroups than tiles
    const int64_t tiles = (int64_t)a.tile_count * (fused == 3 ? a.zsplit : 1) * (fused == 3 && a.nchunks > 0 ? a.nchunks : 1);
    if (a.tile_count <= 0 || a.tile_begin < 0 || (int64_t)a.tile_begin + a.tile_count > (int64_t)TM * TP)
        return hipErrorInvalidValue;
    int nwg = a.num_cu > 0 ? a.num_cu : 1;
    if (tiles < nwg) nwg = (int)tiles;
    static_assert(NXCD * 16 == SYNC_WORDS, "soft-barrier counters: 16 words per XCD");
    if (a.sync_epoch == 0 && !a.sync_zeroed)
        hipLaunchKernelGGL(k_fill_u32_gemm, dim3(1), dim3(SYNC_WORDS), 0, st, a.sync);
    dim3 grid((unsigned)nwg), block(256);
    if (fused == 3)
        hipLaunchKernelGGL((k_gemm<3, NSTAGES>), grid, block, smem, st, a, TM, TP);
    else if (fused == 2)
        hipLaunchKernelGGL((k_gemm<2, NSTAGES>), grid, block, smem, st, a, TM, TP);
    else if (fused)
        hipLaunchKernelGGL((k_gemm<1, NSTAGES>), grid, block, smem, st, a, TM, TP);
    else
        hipLaunchKernelGGL((k_gemm<0, NSTAGES>), grid, block, smem, st, a, TM, TP);
    return hipGetLastError();
}

// One-time set-up of the current device: the chunk GEMM kernels need more dynamic LDS than the default limit.
hipError_t setup_gemm_kernels()
{
    const int smem = NSTAGES * STAGE_BYTES + EXP_BYTES;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm<0, NSTAGES>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm<1, NSTAGES>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm<2, NSTAGES>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm<3, NSTAGES>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, smem);
}

hipError_t launch_fill_zero_i32(int64_t count, int32_t* x, hipStream_t st)
{
    if (count <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_zero_i32, dim3((unsigned)((count + 1023) / 1024)), dim3(256), 0, st, count, x);
    return hipGetLastError();
}

hipError_t launch_fill_zero_i32_2d(int64_t m, int64_t p, int32_t* C, int64_t ldc, hipStream_t st)
{
    dim3 grid((unsigned)m, (unsigned)((p + 255) / 256));
    hipLaunchKernelGGL(k_zero_i32_2d, grid, dim3(256), 0, st, m, p, C, ldc);
    return hipGetLastError();
}

hipError_t launch_accumulate(int64_t m, int64_t p, const int32_t* C, int64_t ldc, const int32_t* eA,
                             const int32_t* eB, int shift, int first, double* D, int64_t ldd, hipStream_t st)
{
    dim3 grid((unsigned)((m + 7) / 8), (unsigned)((p + 255) / 256));
    hipLaunchKernelGGL(k_accumulate, grid, dim3(256), 0, st, m, p, C, ldc, eA, eB, shift, first, D, ldd);
    return hipGetLastError();
}

hipError_t launch_accumulate_tiles(const TileAccArgs& t_in, hipStream_t st)
{
    if (t_in.tile_count <= 0) return hipSuccess;
    TileAccArgs t = t_in;
    t.TM = (int)(ozl::rows_padded(t.m) / ozl::TILE_R);
    t.TP = (int)(ozl::rows_padded(t.p) / ozl::TILE_R);
    hipLaunchKernelGGL(k_accumulate_tiles, dim3((unsigned)t.tile_count * 32u), dim3(256), 0, st, t);
    return hipGetLastError();
}

hipError_t launch_accumulate_chunks(const TileAccArgs& t_in, int k, int r, int beta, hipStream_t st)
{
    if (t_in.tile_count <= 0) return hipSuccess;
    TileAccArgs t = t_in;
    t.TM = (int)(ozl::rows_padded(t.m) / ozl::TILE_R);
    t.TP = (int)(ozl::rows_padded(t.p) / ozl::TILE_R);
    hipLaunchKernelGGL(k_accumulate_chunks, dim3((unsigned)t.tile_count * 32u), dim3(256), 0, st, t, k, r, beta);
    return hipGetLastError();
}

hipError_t launch_axpby(int64_t m, int64_t p, double alpha, const double* D, int64_t ldd, double beta, double* C,
                        int64_t ldc, hipStream_t st)
{
    dim3 grid((unsigned)((m + 7) / 8), (unsigned)((p + 255) / 256));
    hipLaunchKernelGGL(k_axpby, grid, dim3(256), 0, st, m, p, alpha, D, ldd, beta, C, ldc);
    return hipGetLastError();
}

hipError_t launch_fill_zero_f64(int64_t m, int64_t p, double* D, int64_t ldd, hipStream_t st)
{
    dim3 grid((unsigned)m, (unsigned)((p + 255) / 256));
    hipLaunchKernelGGL(k_zero_f64, grid, dim3(256), 0, st, m, p, D, ldd);
    return hipGetLastError();
}

}  // namespace ozk
