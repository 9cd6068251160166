// Steps (i) and (ii) of the scheme: power-of-two scale exponents and INT8
// slices, written in the packed tile-major layout of ozimmu_layout.h.
//
// What is computed (Algorithm 8 of the paper, with its scale mu'' = 2^e * 2^(1-beta)):
//   e      = ceil(log2 max |x|) over a row of A / a column of B (0 if all zero)
//   slice s (s = 1..k) of x = the integer nearest (ties to even) to
//            remainder / 2^(e + 1 - s beta), remainder reduced accordingly.
// How: instead of the printed (x + sigma) - sigma trick the kernels scale once,
//   y_1 = x * 2^(beta - 1 - e)  (exact, |y_1| <= 2^(beta-1)),
//   q_s = rint(y_s)             (v_rndne_f64: round half to even),
//   y_{s+1} = (y_s - q_s) * 2^beta   (both exact),
// which yields the same integers: y_s is remainder / grid_s at every step.
// Both kernels are HBM-bound: 8 bytes read (A twice when its row does not stay
// in cache) and k bytes written per element.
// The bytes stored are q_s + c (c = offset of the stack, see ozimmu_layout.h;
// inner padding counts as a real zero, padding rows of A are all zero bytes); with them go the prefix sums over the slices
// of the row sums of the stored bytes, which the GEMM epilogue needs to take the
// offsets out again.
#include "ozimmu_kernels.h"
#include "ozimmu_layout.h"

namespace {

using namespace ozl;

constexpr int OZIMMU_MAX_SLICES_DEV = 20;  // OZIMMU_MAX_SLICES of the C ABI

// ceil(log2 x) key of a positive finite double given as its bit pattern,
// monotone in x so that maxima can be taken on keys:
// key = 2 * (t + 1100) + (f != 0.5) with x = f * 2^t, f in [0.5, 1); 0 for x == 0.
__device__ inline uint32_t exp_key(uint64_t absbits)
{
    if (absbits == 0) return 0u;
    double x = __longlong_as_double((long long)absbits);
    int t;
    double f = frexp(x, &t);
    return (uint32_t)(2 * (t + 1100) + (f != 0.5 ? 1 : 0));
}
// MASK = false: ceil(log2 x) (round-to-nearest split); MASK = true: floor(log2 x) = t - 1 (bit-mask split)
template <bool MASK>
__device__ inline int key_to_exp(uint32_t key)
{
    if (key == 0u) return 0;
    int t = (int)(key >> 1) - 1100;
    if (MASK) return t - 1;
    return (key & 1u) ? t : t - 1;
}
// digit of one slice: nearest integer, ties to even (Algorithm 8) or truncation toward zero (Algorithm 3)
template <bool MASK>
__device__ inline double digit(double y)
{
    return MASK ? __builtin_trunc(y) : __builtin_rint(y);
}

__device__ inline uint64_t abs_bits(double x)
{
    return (uint64_t)__double_as_longlong(x) & 0x7fffffffffffffffull;
}

__device__ inline uint64_t wave_max_u64(uint64_t v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        uint64_t o = __shfl_xor(v, off, 64);
        v = o > v ? o : v;
    }
    return v;
}

__device__ inline int wave_sum_i32(int v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// One slice of 4 consecutive inner elements: digits of y[], remainders updated in place, the 4 stored
// bytes (digit + c, c = the stack's offset) packed into a dword.  Returns the dword; *sum receives the sum
// of the 4 stored bytes.  Inner padding (l >= n) enters as y = 0 like a real zero and is stored as c.
template <bool MASK>
__device__ inline uint32_t slice_word4(double* y, int c, double two_beta, int* sum)
{
    uint32_t w = 0;
    int sm = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const double q = digit<MASK>(y[j]);
        const int b = (int)q + c;
        w |= ((uint32_t)b & 0xffu) << (8 * j);
        sm += b;
        y[j] = (y[j] - q) * two_beta;
    }
    *sum = sm;
    return w;
}

// ---------------------------------------------------------------------------
// A: one wave per padded row, four consecutive rows per workgroup (their 64-byte
// segments are adjacent in a packed tile, so the workgroup's stores fill whole
// 128-byte lines).  Pass 1 reduces max |a_ij| over the row inside the wave,
// pass 2 re-reads the row (from L2 / Infinity Cache when it is still there)
// and writes the k slices.  A lane handles 4 consecutive inner elements per
// 256-element sweep: the wave reads 2 KiB contiguous per sweep.
// ---------------------------------------------------------------------------
template <bool VEC, bool MASK>
__global__ __launch_bounds__(256) void k_split_A(int64_t m, int64_t n, const double* __restrict__ A, int64_t lda,
                                                 int k, int beta, int c, int8_t* __restrict__ SA,
                                                 int32_t* __restrict__ eA, int32_t* __restrict__ P,
                                                 int32_t* __restrict__ trailer, int64_t Npad, int64_t Rpad,
                                                 int64_t slice_stride)
{
    __shared__ int lsum[4][OZIMMU_MAX_SLICES_DEV][64];  // per-lane sums of the stored bytes, per slice
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t R = (int64_t)blockIdx.x * 4 + w;
    const int64_t KT = Npad / TILE_K;
    if (blockIdx.x == 0 && threadIdx.x == 0) trailer[0] = c;

    if (R >= m) {  // padding row: zeros in every slice, zero sums
        for (int64_t l = 4 * lane; l < Npad; l += 256)
            for (int s = 0; s < k; ++s)
                *reinterpret_cast<uint32_t*>(SA + s * slice_stride + packed_offset(R, l, KT)) = 0u;
        if (lane < k) P[(int64_t)lane * Rpad + R] = 0;
        return;
    }
    const double* row = A + R * lda;

    auto load4 = [&](int64_t l, double* v) {
        if (VEC && l + 3 < n) {
            double2 a = *reinterpret_cast<const double2*>(row + l);
            double2 b = *reinterpret_cast<const double2*>(row + l + 2);
            v[0] = a.x; v[1] = a.y; v[2] = b.x; v[3] = b.y;
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = (l + j < n) ? row[l + j] : 0.0;
        }
    };

    uint64_t mx = 0;
    for (int64_t l = 4 * lane; l < n; l += 256) {
        double v[4];
        load4(l, v);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint64_t b = abs_bits(v[j]);
            mx = b > mx ? b : mx;
        }
    }
    mx = wave_max_u64(mx);
    const int e = key_to_exp<MASK>(exp_key(mx));
    if (lane == 0) eA[R] = e;
    const int sc = beta - 1 - e;
    const double two_beta = (double)(1 << beta);
    for (int s = 0; s < k; ++s) lsum[w][s][lane] = 0;

    for (int64_t l = 4 * lane; l < Npad; l += 256) {
        double y[4];
        load4(l, y);
#pragma unroll
        for (int j = 0; j < 4; ++j) y[j] = ldexp(y[j], sc);
        int8_t* out = SA + packed_offset(R, l, KT);
        for (int s = 0; s < k; ++s) {
            int sm;
            *reinterpret_cast<uint32_t*>(out) = slice_word4<MASK>(y, c, two_beta, &sm);
            out += slice_stride;
            lsum[w][s][lane] += sm;
        }
    }
    int run = 0;
    for (int s = 0; s < k; ++s) {
        run += wave_sum_i32(lsum[w][s][lane]);
        if (lane == 0) P[(int64_t)s * Rpad + R] = run;
    }
}

// ---------------------------------------------------------------------------
// A, single pass (rows of at most 1024 * GROUPS padded elements; GROUPS = 4, 8 or 16): one workgroup
// per padded row keeps the whole row in registers (4 * GROUPS doubles per
// thread), reduces max |a_ij| through LDS and writes the k slices, so A is read
// from HBM exactly once.  Thread t holds elements 4t + 1024 g .. + 3.
// Workgroup b serves XCD b % 8 (hardware dispatch order); the row mapping below
// gives the four rows of a 4-row group (whose 64-byte segments share 256
// contiguous bytes of a packed tile) to four workgroups of the same XCD, so the
// partial lines meet in one L2.
// ---------------------------------------------------------------------------
template <int GROUPS, bool VEC, bool MASK>
__global__ __launch_bounds__(256) void k_split_A_row(int64_t m, int64_t n, const double* __restrict__ A, int64_t lda,
                                                     int k, int beta, int c, int8_t* __restrict__ SA,
                                                     int32_t* __restrict__ eA, int32_t* __restrict__ P,
                                                     int32_t* __restrict__ trailer, int64_t Npad, int64_t Rpad,
                                                     int64_t slice_stride)
{
    __shared__ uint64_t part[4];
    __shared__ int wsum[4][OZIMMU_MAX_SLICES_DEV];  // per-wave sums of the stored bytes, per slice
    const int t = threadIdx.x;
    // the grid has rows_padded(m) workgroups, a multiple of 256, so b / 8 and b % 8 cover whole groups of 32 rows
    const int64_t b = blockIdx.x, x = b % 8, j = b / 8;
    const int64_t R = ((j / 4) * 8 + x) * 4 + (j % 4);
    const int64_t KT = Npad / TILE_K;
    if (b == 0 && t == 0) trailer[0] = c;

    if (R >= m) {  // padding row: zeros in every slice, zero sums
        for (int64_t l = 4 * t; l < Npad; l += 1024)
            for (int s = 0; s < k; ++s)
                *reinterpret_cast<uint32_t*>(SA + s * slice_stride + packed_offset(R, l, KT)) = 0u;
        if (t < k) P[(int64_t)t * Rpad + R] = 0;
        return;
    }
    const double* row = A + R * lda;
    double v[GROUPS][4];
    uint64_t mx = 0;
#pragma unroll
    for (int g = 0; g < GROUPS; ++g) {
        const int64_t l = 4 * t + 1024 * g;
        if (VEC && l + 3 < n) {
            double2 a = *reinterpret_cast<const double2*>(row + l);
            double2 d = *reinterpret_cast<const double2*>(row + l + 2);
            v[g][0] = a.x; v[g][1] = a.y; v[g][2] = d.x; v[g][3] = d.y;
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) v[g][q] = (l + q < n) ? row[l + q] : 0.0;
        }
    }
#pragma unroll
    for (int g = 0; g < GROUPS; ++g)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint64_t ab = abs_bits(v[g][q]);
            mx = ab > mx ? ab : mx;
        }
    mx = wave_max_u64(mx);
    if ((t & 63) == 0) part[t >> 6] = mx;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < 4; ++w) mx = part[w] > mx ? part[w] : mx;
    const int e = key_to_exp<MASK>(exp_key(mx));
    if (t == 0) eA[R] = e;
    const int sc = beta - 1 - e;
    const double two_beta = (double)(1 << beta);
#pragma unroll
    for (int g = 0; g < GROUPS; ++g)
#pragma unroll
        for (int q = 0; q < 4; ++q) v[g][q] = ldexp(v[g][q], sc);
    // slice after slice over the whole row (the remainders stay in v), so that one sum per slice is reduced
    for (int s = 0; s < k; ++s) {
        int tsum = 0;
#pragma unroll
        for (int g = 0; g < GROUPS; ++g) {
            const int64_t l = 4 * t + 1024 * g;
            if (l < Npad) {
                int sm;
                *reinterpret_cast<uint32_t*>(SA + s * slice_stride + packed_offset(R, l, KT)) =
                    slice_word4<MASK>(v[g], c, two_beta, &sm);
                tsum += sm;
            }
        }
        tsum = wave_sum_i32(tsum);
        if ((t & 63) == 0) wsum[t >> 6][s] = tsum;
    }
    __syncthreads();
    if (t == 0) {
        int run = 0;
        for (int s = 0; s < k; ++s) {
            run += wsum[0][s] + wsum[1][s] + wsum[2][s] + wsum[3][s];
            P[(int64_t)s * Rpad + R] = run;
        }
    }
}

// ---------------------------------------------------------------------------
// B, pass 1: column maxima.  A workgroup covers 64 columns x LCH inner rows;
// lane = column, so each wave reads 512 contiguous bytes per inner row.  The
// per-column maximum is merged into keys[] with a 32-bit atomic max (order
// free, hence deterministic).
// ---------------------------------------------------------------------------
constexpr int LCH = 512;  // rows of B per workgroup of the column-maximum kernel (fewer for small B)
// Marks a column entry of eB that still holds the key of the column maximum rather than the exponent decoded
// from it (k_split_B decodes on the fly and stores the exponents): exponents are small, keys carry this bit.
constexpr uint32_t RAW_KEY_TAG = 0x40000000u;

__global__ __launch_bounds__(256) void k_colmax_B(int64_t n, int64_t p, const double* __restrict__ B, int64_t ldb,
                                                  uint32_t* __restrict__ keys, int lch, uint32_t tag)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t j = (int64_t)blockIdx.y * 64 + lane;
    const int64_t l0 = (int64_t)blockIdx.x * lch;
    const int64_t l1 = l0 + lch < n ? l0 + lch : n;
    __shared__ uint64_t part[4][64];
    uint64_t mx = 0;
    if (j < p) {
        for (int64_t l = l0 + w; l < l1; l += 4) {
            uint64_t b = abs_bits(B[l * ldb + j]);
            mx = b > mx ? b : mx;
        }
    }
    part[w][lane] = mx;
    __syncthreads();
    if (w == 0 && j < p) {
        for (int q = 1; q < 4; ++q) mx = part[q][lane] > mx ? part[q][lane] : mx;
        uint32_t key = exp_key(mx);
        if (key) atomicMax(keys + j, tag | key);
    }
}

// rows per workgroup of k_colmax_B: LCH, halved while that leaves the chip short of workgroups
inline int colmax_rows(int64_t n, int64_t p)
{
    int lch = LCH;
    while (lch > 16 && ((n + lch - 1) / lch) * ((p + 63) / 64) < 1024) lch /= 2;
    return lch;
}

// two fills in one launch: x[0, cx) = vx and y[0, cy) = vy, then z[0, cz) = 0 (any count may be 0)
__global__ void k_fill3_u32(int64_t cx, uint32_t* x, uint32_t vx, int64_t cy, uint32_t* y, uint32_t vy, int64_t cz,
                            uint32_t* z)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < cx) x[i] = vx;
    if (i < cy) y[i] = vy;
    if (i < cz) z[i] = 0u;
}

__global__ void k_fill_u32(int64_t count, uint32_t* x, uint32_t v)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) x[i] = v;
}

template <bool MASK>
__global__ void k_decode_keys(int64_t count, int32_t* e)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) e[i] = key_to_exp<MASK>((uint32_t)e[i]);
}

// per-slice sums of a stack (k arrays of Rpad entries) -> prefix sums over the slices, in place
__global__ void k_prefix_sums(int64_t Rpad, int k, int32_t* P)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= Rpad) return;
    int run = 0;
    for (int s = 0; s < k; ++s) {
        run += P[(int64_t)s * Rpad + i];
        P[(int64_t)s * Rpad + i] = run;
    }
}

// ---------------------------------------------------------------------------
// B, pass 2: slices, transposed so that the inner index becomes contiguous.
// A workgroup handles 128 inner rows x 64 columns.  Reads: lane = column
// (512 contiguous bytes per wave and inner row).  Each thread keeps its 32
// remainders in registers, emits slices in batches of SBATCH through LDS
// (row pitch 33 dwords: conflict-free column-wise dword stores), and the
// batch is written out with lane = 16-byte chunk along the inner index, i.e.
// full 128-byte lines (two adjacent rows of a tile) per slice.
// ---------------------------------------------------------------------------
constexpr int SBATCH = 4;
constexpr int PITCH = 33;  // dwords per column row in LDS (32 data + 1 pad)

template <bool MASK>
__global__ __launch_bounds__(256) void k_split_B(int64_t n, int64_t p, const double* __restrict__ B, int64_t ldb,
                                                 int k, int beta, int c, int8_t* __restrict__ SB,
                                                 int32_t* eB, int32_t* __restrict__ P,
                                                 int32_t* __restrict__ trailer, int64_t Npad, int64_t Rpad,
                                                 int64_t slice_stride, int blocks_per_wg)
{
    __shared__ uint32_t tile[SBATCH][64 * PITCH];
    __shared__ int colsum[OZIMMU_MAX_SLICES_DEV][64];  // sums of the stored bytes per slice and column
    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
    const int64_t j0 = (int64_t)blockIdx.y * 64;      // first column (= packed row)
    const int64_t j = j0 + lane;
    const int64_t KT = Npad / TILE_K;
    const double two_beta = (double)(1 << beta);
    const bool col_ok = j < p;
    // eB[j] holds the tagged key of the column maximum until the workgroups of the first inner block have
    // replaced it by the exponent; a workgroup that reads it meanwhile gets one or the other, and both give e
    int e = 0;
    if (col_ok) {
        const uint32_t v = __hip_atomic_load(reinterpret_cast<uint32_t*>(eB) + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        e = (v & 0xc0000000u) == RAW_KEY_TAG ? key_to_exp<MASK>(v - RAW_KEY_TAG) : (int)v;
        if (blockIdx.x == 0 && w == 0)
            __hip_atomic_store(reinterpret_cast<uint32_t*>(eB) + j, (uint32_t)e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    const int sc = beta - 1 - e;
    if (blockIdx.x == 0 && blockIdx.y == 0 && t == 0) trailer[0] = c;
    for (int i = t; i < k * 64; i += 256) colsum[i / 64][i % 64] = 0;
    // write-out mapping: 8 lanes per column row, 32 column rows per pass
    const int oc = t & 7, orow = t >> 3;
    __syncthreads();

    // blocks_per_wg consecutive blocks of 128 inner rows (fewer atomics on the sums than one block each)
    for (int blk = 0; blk < blocks_per_wg; ++blk) {
        const int64_t l0 = ((int64_t)blockIdx.x * blocks_per_wg + blk) * 128;  // inner offset of this block
        if (l0 >= Npad) break;
        double y[32];
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            const int64_t l = l0 + w * 32 + i;
            const double v = (col_ok && l < n) ? B[l * ldb + j] : 0.0;
            y[i] = ldexp(v, sc);
        }
        for (int sb = 0; sb < k; sb += SBATCH) {
            const int ns = (k - sb) < SBATCH ? (k - sb) : SBATCH;
            for (int s = 0; s < ns; ++s) {
                int tsum = 0;
#pragma unroll
                for (int ii = 0; ii < 8; ++ii) {
                    int sm;
                    tile[s][lane * PITCH + w * 8 + ii] = slice_word4<MASK>(&y[4 * ii], c, two_beta, &sm);
                    tsum += sm;
                }
                atomicAdd(&colsum[sb + s][lane], tsum);
            }
            __syncthreads();
            for (int s = 0; s < ns; ++s) {
#pragma unroll
                for (int pass = 0; pass < 2; ++pass) {
                    int jr = orow + 32 * pass;
                    const uint32_t* src = &tile[s][jr * PITCH + oc * 4];
                    uint4 v = make_uint4(src[0], src[1], src[2], src[3]);
                    int8_t* dst = SB + (int64_t)(sb + s) * slice_stride + packed_offset(j0 + jr, l0 + oc * CHUNK, KT);
                    // whole 128-byte lines that nobody reads before the GEMM: non-temporal (4 % on this kernel; the
                    // 64-byte row segments of the A kernels need the L2 to merge them and stay temporal)
                    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
                    const u32x4 vv = {v.x, v.y, v.z, v.w};
                    __builtin_nontemporal_store(vv, reinterpret_cast<u32x4*>(dst));
                }
            }
            __syncthreads();
        }
    }
    // integer sums: order-free, hence deterministic (P was zeroed; k_prefix_sums finishes)
    for (int i = t; i < k * 64; i += 256)
        if (colsum[i / 64][i % 64] != 0) atomicAdd(&P[(int64_t)(i / 64) * Rpad + j0 + (i % 64)], colsum[i / 64][i % 64]);
}

// ---------------------------------------------------------------------------
// Algorithm 5 (one scale per slice), A: one wave per padded row as in k_split_A.
// The scale of slice s+1 comes from the largest remainder after slice s, so the
// row is walked k times; what is left of it lives in `rem` (row pitch Npad) and
// every lane re-reads only the elements it wrote itself.  With
//   y = remainder * 2^(beta-1-e_s)  (exact),  q_s = rint(y),
//   remainder <- (y - q_s) * 2^(e_s+1-beta)  (both exact).
// HBM-bound: about 16 k bytes per element (remainder read and written per slice).
// ---------------------------------------------------------------------------
template <bool VEC>
__global__ __launch_bounds__(256) void k_split_A_ps(int64_t m, int64_t n, const double* __restrict__ A, int64_t lda,
                                                    int k, int beta, int8_t* __restrict__ SA,
                                                    int32_t* __restrict__ eA, double* __restrict__ rem,
                                                    int32_t* __restrict__ trailer, int64_t Npad,
                                                    int64_t slice_stride)
{
    const int lane = threadIdx.x & 63;
    const int64_t R = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t KT = Npad / TILE_K;
    if (blockIdx.x == 0 && threadIdx.x == 0) trailer[0] = 0;  // slices with a scale each are stored without offset

    if (R >= m) {  // padding row: zeros in every slice
        for (int64_t l = 4 * lane; l < Npad; l += 256)
            for (int s = 0; s < k; ++s)
                *reinterpret_cast<uint32_t*>(SA + s * slice_stride + packed_offset(R, l, KT)) = 0u;
        return;
    }
    const double* row = A + R * lda;
    double* rrow = rem + R * Npad;

    auto load4 = [&](int64_t l, double* v) {
        if (VEC && l + 3 < n) {
            double2 a = *reinterpret_cast<const double2*>(row + l);
            double2 b = *reinterpret_cast<const double2*>(row + l + 2);
            v[0] = a.x; v[1] = a.y; v[2] = b.x; v[3] = b.y;
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = (l + j < n) ? row[l + j] : 0.0;
        }
    };

    uint64_t mx = 0;
    for (int64_t l = 4 * lane; l < n; l += 256) {
        double v[4];
        load4(l, v);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint64_t b = abs_bits(v[j]);
            mx = b > mx ? b : mx;
        }
    }
    int e = key_to_exp<false>(exp_key(wave_max_u64(mx)));

    for (int s = 0; s < k; ++s) {
        if (lane == 0) eA[(int64_t)s * m + R] = e;
        const int sc = beta - 1 - e;
        const bool keep = s + 1 < k;
        mx = 0;
        for (int64_t l = 4 * lane; l < Npad; l += 256) {
            double v[4];
            if (s == 0) {
                load4(l, v);
            } else {
                double2 a = *reinterpret_cast<const double2*>(rrow + l);
                double2 b = *reinterpret_cast<const double2*>(rrow + l + 2);
                v[0] = a.x; v[1] = a.y; v[2] = b.x; v[3] = b.y;
            }
            uint32_t w = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const double y = ldexp(v[j], sc);
                const double q = __builtin_rint(y);
                w |= ((uint32_t)(int)q & 0xffu) << (8 * j);
                v[j] = ldexp(y - q, -sc);
                const uint64_t b = abs_bits(v[j]);
                mx = b > mx ? b : mx;
            }
            *reinterpret_cast<uint32_t*>(SA + s * slice_stride + packed_offset(R, l, KT)) = w;
            if (keep) {
                *reinterpret_cast<double2*>(rrow + l) = make_double2(v[0], v[1]);
                *reinterpret_cast<double2*>(rrow + l + 2) = make_double2(v[2], v[3]);
            }
        }
        e = key_to_exp<false>(exp_key(wave_max_u64(mx)));
    }
}

// ---------------------------------------------------------------------------
// Algorithm 5, B: one launch per slice (the column maxima of the remainder need
// a grid-wide reduction between slices).  Tiling and write-out as in k_split_B;
// src is B for the first slice and the remainder buffer (pitch p) afterwards.
// The maxima of the new remainder are merged into keys_next for the next launch.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_split_B_ps(int64_t n, int64_t p, const double* src, int64_t ld, int beta,
                                                    int8_t* __restrict__ SBs, const uint32_t* __restrict__ keys,
                                                    uint32_t* __restrict__ keys_next, double* rem, int64_t Npad)
{
    __shared__ uint32_t tile[64 * PITCH];
    __shared__ uint64_t part[4][64];
    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
    const int64_t l0 = (int64_t)blockIdx.x * 128;
    const int64_t j0 = (int64_t)blockIdx.y * 64;
    const int64_t j = j0 + lane;
    const int64_t KT = Npad / TILE_K;
    const bool col_ok = j < p;
    const int sc = beta - 1 - (col_ok ? key_to_exp<false>(keys[j]) : 0);

    double y[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) {
        const int64_t l = l0 + w * 32 + i;
        y[i] = (col_ok && l < n) ? src[l * ld + j] : 0.0;
    }
    uint64_t mx = 0;
#pragma unroll
    for (int ii = 0; ii < 8; ++ii) {
        uint32_t wv = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int i = 4 * ii + b;
            const double ys = ldexp(y[i], sc);
            const double q = __builtin_rint(ys);
            wv |= ((uint32_t)(int)q & 0xffu) << (8 * b);
            y[i] = ldexp(ys - q, -sc);
            const uint64_t ab = abs_bits(y[i]);
            mx = ab > mx ? ab : mx;
        }
        tile[lane * PITCH + w * 8 + ii] = wv;
    }
    if (keys_next) {
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            const int64_t l = l0 + w * 32 + i;
            if (col_ok && l < n) rem[l * p + j] = y[i];
        }
    }
    part[w][lane] = mx;
    __syncthreads();
    const int oc = t & 7, orow = t >> 3;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int jr = orow + 32 * pass;
        const uint32_t* sp = &tile[jr * PITCH + oc * 4];
        uint4 v = make_uint4(sp[0], sp[1], sp[2], sp[3]);
        *reinterpret_cast<uint4*>(SBs + packed_offset(j0 + jr, l0 + oc * CHUNK, KT)) = v;
    }
    if (keys_next && w == 0 && col_ok) {
        for (int q = 1; q < 4; ++q) mx = part[q][lane] > mx ? part[q][lane] : mx;
        const uint32_t key = exp_key(mx);
        if (key) atomicMax(keys_next + j, key);
    }
}

// Unpack: one thread per output byte, out[s][row][l].
__global__ __launch_bounds__(256) void k_export(int64_t rows, int64_t n, int k, const int8_t* __restrict__ packed,
                                                const int32_t* __restrict__ trailer, int8_t* __restrict__ out,
                                                int64_t KT, int64_t slice_stride)
{
    int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    int64_t total = (int64_t)k * rows * n;
    if (idx >= total) return;
    int64_t l = idx % n, R = (idx / n) % rows, s = idx / (n * rows);
    out[idx] = (int8_t)(packed[s * slice_stride + packed_offset(R, l, KT)] - trailer[0]);  // stored byte = q + c
}

}  // namespace

namespace ozk {

// k_set_i32: one INT32 (the offset in the trailer of a stack whose split kernels do not write it themselves)
}  // namespace ozk
namespace {
__global__ void k_set_i32(int32_t* x, int32_t v) { x[0] = v; }
}  // namespace
namespace ozk {

hipError_t launch_split_A(int64_t m, int64_t n, const double* A, int64_t lda, int k, int beta, int split_mode,
                          int offset, int8_t* SA, int32_t* eA, hipStream_t st)
{
    const int64_t Rpad = ozl::rows_padded(m), Npad = ozl::inner_padded(n);
    const int64_t stride = ozl::slice_bytes(m, n);
    int32_t* P = reinterpret_cast<int32_t*>(SA + ozl::sums_offset(m, n, k));
    int32_t* trailer = reinterpret_cast<int32_t*>(SA + ozl::trailer_offset(m, n, k));
    const bool vec = (reinterpret_cast<uintptr_t>(A) % 16 == 0) && (lda % 2 == 0);
    const bool mask = split_mode != 0;
    if (Npad <= 16384) {  // the row fits the registers of one workgroup: single pass over A
        dim3 grid((unsigned)Rpad), block(256);
#define OZ_LAUNCH_ROW(G, V, M)                                                                                    \
    hipLaunchKernelGGL((k_split_A_row<G, V, M>), grid, block, 0, st, m, n, A, lda, k, beta, offset, SA, eA, P, trailer, \
                       Npad, Rpad, stride)
#define OZ_PICK_ROW(G)                         \
    do {                                       \
        if (vec && !mask) OZ_LAUNCH_ROW(G, true, false);       \
        else if (!vec && !mask) OZ_LAUNCH_ROW(G, false, false); \
        else if (vec) OZ_LAUNCH_ROW(G, true, true);             \
        else OZ_LAUNCH_ROW(G, false, true);                     \
    } while (0)
        if (Npad <= 4096)
            OZ_PICK_ROW(4);
        else if (Npad <= 8192)
            OZ_PICK_ROW(8);
        else
            OZ_PICK_ROW(16);
#undef OZ_PICK_ROW
#undef OZ_LAUNCH_ROW
        return hipGetLastError();
    }
    dim3 grid((unsigned)(Rpad / 4)), block(256);
#define OZ_LAUNCH_A(V, M)                                                                                          \
    hipLaunchKernelGGL((k_split_A<V, M>), grid, block, 0, st, m, n, A, lda, k, beta, offset, SA, eA, P, trailer, Npad, \
                       Rpad, stride)
    if (vec && !mask)
        OZ_LAUNCH_A(true, false);
    else if (!vec && !mask)
        OZ_LAUNCH_A(false, false);
    else if (vec)
        OZ_LAUNCH_A(true, true);
    else
        OZ_LAUNCH_A(false, true);
#undef OZ_LAUNCH_A
    return hipGetLastError();
}

hipError_t launch_split_B(int64_t n, int64_t p, const double* B, int64_t ldb, int k, int beta, int split_mode,
                          int offset, int8_t* SB, int32_t* eB, hipStream_t st, uint32_t* also_zero,
                          int also_zero_count)
{
    const int64_t Rpad = ozl::rows_padded(p), Npad = ozl::inner_padded(n);
    const int64_t stride = ozl::slice_bytes(p, n);
    int32_t* P = reinterpret_cast<int32_t*>(SB + ozl::sums_offset(p, n, k));
    int32_t* trailer = reinterpret_cast<int32_t*>(SB + ozl::trailer_offset(p, n, k));
    const int64_t nsums = (int64_t)k * Rpad;
    const int64_t nfill = nsums > p ? (nsums > also_zero_count ? nsums : also_zero_count)
                                    : (p > also_zero_count ? p : also_zero_count);
    hipLaunchKernelGGL(k_fill3_u32, dim3((unsigned)((nfill + 255) / 256)), dim3(256), 0, st, p,
                       reinterpret_cast<uint32_t*>(eB), RAW_KEY_TAG, nsums, reinterpret_cast<uint32_t*>(P), 0u,
                       also_zero ? also_zero_count : 0, also_zero);
    const int lch = colmax_rows(n, p);
    dim3 gmax((unsigned)((n + lch - 1) / lch), (unsigned)((p + 63) / 64));
    hipLaunchKernelGGL(k_colmax_B, gmax, dim3(256), 0, st, n, p, B, ldb, reinterpret_cast<uint32_t*>(eB), lch,
                       RAW_KEY_TAG);
    // a workgroup takes 4 consecutive blocks of 128 inner rows once there are enough blocks to fill the chip anyway
    const int64_t blocks = Npad / 128;
    const int per_wg = blocks >= 32 ? 4 : 1;
    dim3 grid((unsigned)((blocks + per_wg - 1) / per_wg), (unsigned)(Rpad / 64));
    if (split_mode == 0) {
        hipLaunchKernelGGL(k_split_B<false>, grid, dim3(256), 0, st, n, p, B, ldb, k, beta, offset, SB, eB, P, trailer,
                           Npad, Rpad, stride, per_wg);
    } else {
        hipLaunchKernelGGL(k_split_B<true>, grid, dim3(256), 0, st, n, p, B, ldb, k, beta, offset, SB, eB, P, trailer,
                           Npad, Rpad, stride, per_wg);
    }
    hipLaunchKernelGGL(k_prefix_sums, dim3((unsigned)((Rpad + 255) / 256)), dim3(256), 0, st, Rpad, k, P);
    return hipGetLastError();
}

hipError_t launch_split_A_per_slice(int64_t m, int64_t n, const double* A, int64_t lda, int k, int beta, int8_t* SA,
                                    int32_t* eA, double* rem, hipStream_t st)
{
    const int64_t Rpad = ozl::rows_padded(m), Npad = ozl::inner_padded(n);
    const int64_t stride = ozl::slice_bytes(m, n);
    int32_t* trailer = reinterpret_cast<int32_t*>(SA + ozl::trailer_offset(m, n, k));
    const bool vec = (reinterpret_cast<uintptr_t>(A) % 16 == 0) && (lda % 2 == 0);
    dim3 grid((unsigned)(Rpad / 4)), block(256);
    if (vec)
        hipLaunchKernelGGL((k_split_A_ps<true>), grid, block, 0, st, m, n, A, lda, k, beta, SA, eA, rem, trailer, Npad,
                           stride);
    else
        hipLaunchKernelGGL((k_split_A_ps<false>), grid, block, 0, st, m, n, A, lda, k, beta, SA, eA, rem, trailer, Npad,
                           stride);
    return hipGetLastError();
}

hipError_t launch_split_B_per_slice(int64_t n, int64_t p, const double* B, int64_t ldb, int k, int beta, int8_t* SB,
                                    int32_t* eB, double* rem, hipStream_t st)
{
    const int64_t Rpad = ozl::rows_padded(p), Npad = ozl::inner_padded(n);
    const int64_t stride = ozl::slice_bytes(p, n);
    hipLaunchKernelGGL(k_set_i32, dim3(1), dim3(1), 0, st,
                       reinterpret_cast<int32_t*>(SB + ozl::trailer_offset(p, n, k)), 0);
    uint32_t* keys = reinterpret_cast<uint32_t*>(eB);  // k arrays of p keys, decoded in place at the end
    const int64_t nk = (int64_t)k * p;
    hipLaunchKernelGGL(k_fill_u32, dim3((unsigned)((nk + 255) / 256)), dim3(256), 0, st, nk, keys, 0u);
    dim3 gmax((unsigned)((n + LCH - 1) / LCH), (unsigned)((p + 63) / 64));
    hipLaunchKernelGGL(k_colmax_B, gmax, dim3(256), 0, st, n, p, B, ldb, keys, LCH, 0u);
    dim3 grid((unsigned)(Npad / 128), (unsigned)(Rpad / 64));
    for (int s = 0; s < k; ++s)
        hipLaunchKernelGGL(k_split_B_ps, grid, dim3(256), 0, st, n, p, s == 0 ? B : rem, s == 0 ? ldb : p, beta,
                           SB + (int64_t)s * stride, keys + (int64_t)s * p,
                           s + 1 < k ? keys + (int64_t)(s + 1) * p : nullptr, rem, Npad);
    hipLaunchKernelGGL(k_decode_keys<false>, dim3((unsigned)((nk + 255) / 256)), dim3(256), 0, st, nk, eB);
    return hipGetLastError();
}

hipError_t launch_export(int64_t rows, int64_t n, int k, const int8_t* packed, int8_t* out, hipStream_t st)
{
    const int64_t Npad = ozl::inner_padded(n);
    const int64_t total = (int64_t)k * rows * n;
    if (total == 0) return hipSuccess;
    hipLaunchKernelGGL(k_export, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, rows, n, k, packed,
                       reinterpret_cast<const int32_t*>(packed + ozl::trailer_offset(rows, n, k)), out,
                       Npad / ozl::TILE_K, ozl::slice_bytes(rows, n));
    return hipGetLastError();
}

}  // namespace ozk
