// Measurement aid of bench.py, not part of the library: what this chip sustains on the two INT8
// matrix-core instructions of gfx950 - v_mfma_i32_16x16x64_i8, which the GEMM phase is made of, and
// v_mfma_i32_32x32x32_i8 - when nothing else runs.
// One workgroup of 4 waves per compute unit; every wave runs `iters` rounds of independent MFMAs on register
// operands that fill its 256 accumulation registers (64 of 16 x 16 x 64 or 16 of 32 x 32 x 32; no LDS or memory
// traffic in the loop).  The operand bytes are pseudo-random and uniform in [lo, hi]: the clock the chip holds
// under this load depends on how much the operand bits toggle, so the rate for slice-like bytes is the ceiling
// the GEMM phase can be priced against next to the data-sheet peak.
//
//   int bench_mfma_rate_probe(int shape /* 16 or 32 */, int iters, int lo, int hi,
//                             int32_t* out /* device, >= 4 bytes */,
//                             double* ops /* host: integer operations of the launch */, void* stream)
// returns 0, -1 (null pointer), -2 (unknown shape, iters < 1 or range outside -128..127) or -5 (HIP error).
// The caller times the launch with events on `stream`.
#include <hip/hip_runtime.h>
#include <cstdint>
#include <type_traits>

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

template <int SHAPE>
__global__ __launch_bounds__(256) void k_mfma_rate_probe(int iters, int lo, int span, int32_t* out)
{
    // operand bytes from a linear congruential generator, one stream per thread
    uint32_t x = (uint32_t)(blockIdx.x * 256 + threadIdx.x) * 2654435761u + 12345u;
    auto next_byte = [&]() -> uint32_t {
        x = x * 1664525u + 1013904223u;
        return (uint32_t)(lo + (int)((x >> 16) % (uint32_t)span)) & 0xffu;
    };
    auto next_v4i = [&]() -> v4i {
        v4i v;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const uint32_t b0 = next_byte(), b1 = next_byte(), b2 = next_byte(), b3 = next_byte();
            v[d] = (int)(b0 | (b1 << 8) | (b2 << 16) | (b3 << 24));
        }
        return v;
    };
    constexpr int F = SHAPE == 32 ? 4 : 8;  // fragments per operand: F x F tiles fill the accumulation registers
    v4i fa[F], fb[F];
#pragma unroll
    for (int i = 0; i < F; ++i) {
        fa[i] = next_v4i();
        fb[i] = next_v4i();
    }
    typedef std::conditional_t<SHAPE == 32, v16i, v4i> acc_t;
    constexpr int R = SHAPE == 32 ? 16 : 4;
    acc_t acc[F][F];
#pragma unroll
    for (int i = 0; i < F; ++i)
#pragma unroll
        for (int j = 0; j < F; ++j)
#pragma unroll
            for (int r = 0; r < R; ++r) acc[i][j][r] = 0;
    for (int it = 0; it < iters; ++it) {
        // rotate one operand set so that consecutive rounds do not repeat the same products
        const v4i tmp = fa[0];
#pragma unroll
        for (int i = 0; i + 1 < F; ++i) fa[i] = fa[i + 1];
        fa[F - 1] = tmp;
#pragma unroll
        for (int i = 0; i < F; ++i)
#pragma unroll
            for (int j = 0; j < F; ++j) {
                if constexpr (SHAPE == 32)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
                else
                    acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
            }
    }
    int sum = 0;
#pragma unroll
    for (int i = 0; i < F; ++i)
#pragma unroll
        for (int j = 0; j < F; ++j)
#pragma unroll
            for (int r = 0; r < R; ++r) sum += acc[i][j][r];
    if (sum == 0x5a5a5a5a) out[0] = sum;  // practically never: keeps the loop alive without memory traffic
}

}  // namespace

extern "C" int bench_mfma_rate_probe(int shape, int iters, int lo, int hi, int32_t* out, double* ops, void* stream)
{
    if (!out || !ops) return -1;
    if ((shape != 16 && shape != 32) || iters < 1 || lo < -128 || hi > 127 || lo > hi) return -2;
    int dev = 0, ncu = 0;
    if (hipGetDevice(&dev) != hipSuccess) return -5;
    if (hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || ncu < 1) return -5;
    if (shape == 32)
        hipLaunchKernelGGL(k_mfma_rate_probe<32>, dim3((unsigned)ncu), dim3(256), 0, (hipStream_t)stream, iters, lo,
                           hi - lo + 1, out);
    else
        hipLaunchKernelGGL(k_mfma_rate_probe<16>, dim3((unsigned)ncu), dim3(256), 0, (hipStream_t)stream, iters, lo,
                           hi - lo + 1, out);
    // per wave and round: 16 MFMAs of 32 x 32 x 32 multiply-adds, or 64 of 16 x 16 x 64
    *ops = (double)ncu * 4.0 * (double)iters * (shape == 32 ? 16.0 * 2.0 * 32.0 * 32.0 * 32.0 : 64.0 * 2.0 * 16.0 * 16.0 * 64.0);
    return hipGetLastError() == hipSuccess ? 0 : -5;
}
