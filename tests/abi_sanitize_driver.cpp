// Drives the host side of the C-ABI library without a GPU, for a build whose host pass carries
// AddressSanitizer + UndefinedBehaviorSanitizer (tests/test_sanitizers.py): the parameter formulas, the size
// functions over the whole admissible range (64-bit products of sizes), and every argument check.  No call
// below reaches a kernel launch: each fails validation first or has nothing to do.
#include "../include/ozimmu.h"
#include <cstdio>
#include <cstdlib>

#define EXPECT(call, want)                                                                    \
    do {                                                                                      \
        const long long got_ = (long long)(call);                                             \
        if (got_ != (long long)(want)) {                                                      \
            std::printf("line %d: %s = %lld, expected %lld\n", __LINE__, #call, got_, (long long)(want)); \
            ++failures;                                                                       \
        }                                                                                     \
    } while (0)

int main()
{
    int failures = 0;
    const int64_t top = ((int64_t)1 << 22) - 256, inner_max = (int64_t)1 << 29;
    void* fake = reinterpret_cast<void*>(4096);  // never dereferenced
    double* fd = static_cast<double*>(fake);
    int8_t* f8 = static_cast<int8_t*>(fake);
    int32_t* f32 = static_cast<int32_t*>(fake);

    for (int64_t n = 1; n <= inner_max; n = n * 2 + ((n & 1) ? 0 : 1)) {
        int beta = 0;
        int64_t r = 0;
        EXPECT(ozimmu_params(n, &beta, &r), OZIMMU_OK);
        if (beta < 1 || beta > 7 || r < 1) ++failures;
        for (int k = 1; k <= OZIMMU_MAX_SLICES; ++k)
            if (ozimmu_num_chunks(n, k) < k) ++failures;
        if (ozimmu_r_wide(n) < r) ++failures;
    }
    EXPECT(ozimmu_params(0, nullptr, nullptr), OZIMMU_ERR_DIM);
    EXPECT(ozimmu_params(inner_max + 1, nullptr, nullptr), OZIMMU_ERR_DIM);
    // the size functions at the corners of the admissible range (no overflow in their 64-bit arithmetic)
    const int64_t sizes[] = {0, 1, 255, 256, 257, 65536, top};
    for (int64_t m : sizes)
        for (int64_t p : sizes)
            for (int64_t n : {(int64_t)0, (int64_t)1, (int64_t)300, inner_max})
                for (int k : {1, 8, OZIMMU_MAX_SLICES}) {
                    const size_t w = ozimmu_workspace_bytes(m, n, p, k);
                    if (ozimmu_workspace_bytes_ex(m, n, p, k) < w) ++failures;
                    for (int mode = 0; mode < 3; ++mode)
                        if (ozimmu_workspace_bytes_variant(m, n, p, k, mode) < (mode == 2 ? 0 : w)) ++failures;
                    (void)ozimmu_slices_bytes(m, n, k);
                    (void)ozimmu_remainder_bytes(m, n, 0);
                    (void)ozimmu_remainder_bytes(p, n, 1);
                }
    EXPECT(ozimmu_workspace_bytes(-1, 1, 1, 1), 0);
    for (int s = 1; s >= -6; --s)
        if (!ozimmu_status_string(s)) ++failures;

    // argument checks of every entry point
    EXPECT(ozimmu_dgemm(-1, 4, 4, fd, 4, fd, 4, fd, 4, 8, fake, 1 << 30, nullptr), OZIMMU_ERR_DIM);
    EXPECT(ozimmu_dgemm(4, 4, 4, fd, 3, fd, 4, fd, 4, 8, fake, 1 << 30, nullptr), OZIMMU_ERR_DIM);
    EXPECT(ozimmu_dgemm(4, 4, 4, fd, (int64_t)1 << 30, fd, 4, fd, 4, 8, fake, 1 << 30, nullptr), OZIMMU_ERR_DIM);
    EXPECT(ozimmu_dgemm(top + 1, 4, 4, fd, 4, fd, 4, fd, 4, 8, fake, 1 << 30, nullptr), OZIMMU_ERR_DIM);
    EXPECT(ozimmu_dgemm(4, inner_max + 1, 4, fd, inner_max + 1, fd, 4, fd, 4, 8, fake, 1 << 30, nullptr), OZIMMU_ERR_DIM);
    EXPECT(ozimmu_dgemm(4, 4, 4, fd, 4, fd, 4, fd, 4, 0, fake, 1 << 30, nullptr), OZIMMU_ERR_SLICES);
    EXPECT(ozimmu_dgemm(4, 4, 4, fd, 4, fd, 4, fd, 4, 21, fake, 1 << 30, nullptr), OZIMMU_ERR_SLICES);
    EXPECT(ozimmu_dgemm(4, 4, 4, nullptr, 4, fd, 4, fd, 4, 8, fake, 1 << 30, nullptr), OZIMMU_ERR_NULL);
    EXPECT(ozimmu_dgemm(4, 4, 4, fd, 4, fd, 4, fd, 4, 8, fake, 16, nullptr), OZIMMU_ERR_WORKSPACE);
    EXPECT(ozimmu_dgemm(4, 4, 4, fd, 4, fd, 4, fd, 4, 8, reinterpret_cast<void*>(4097), (size_t)1 << 30, nullptr),
           OZIMMU_ERR_WORKSPACE);
    EXPECT(ozimmu_dgemm(0, 4, 4, nullptr, 4, nullptr, 4, nullptr, 4, 8, nullptr, 0, nullptr), OZIMMU_OK);
    EXPECT(ozimmu_dgemm(top, inner_max, top, fd, inner_max, fd, top, fd, top, 20, fake, 16, nullptr), OZIMMU_ERR_WORKSPACE);
    EXPECT(ozimmu_dgemm_variant(4, 4, 4, fd, 4, fd, 4, fd, 4, 8, 3, 0, fake, 1 << 30, nullptr), OZIMMU_ERR_SLICES);
    EXPECT(ozimmu_dgemm_variant(4, 4, 4, fd, 4, fd, 4, fd, 4, 8, 0, 3, fake, 1 << 30, nullptr), OZIMMU_ERR_SLICES);
    EXPECT(ozimmu_dgemm_variant(4, 4, 4, fd, 4, fd, 4, fd, 4, 8, 1, OZIMMU_ACCUM_WIDE, fake, 1 << 30, nullptr),
           OZIMMU_ERR_SLICES);
    EXPECT(ozimmu_dgemm_variant(4, 4, 4, fd, 4, fd, 4, fd, 4, 8, 2, OZIMMU_ACCUM_GROUPED, fake, 1 << 30, nullptr),
           OZIMMU_ERR_SLICES);
    EXPECT(ozimmu_dgemm_variant(4, 4, 4, fd, 4, fd, 4, fd, 4, 8, 0, 0x300, fake, 1 << 30, nullptr), OZIMMU_ERR_SLICES);
    EXPECT(ozimmu_gemm_ex(0, 0, 4, 4, 4, 1.0, fd, 3, fd, 4, 0.0, fd, 4, 8, fake, 1 << 30, nullptr), OZIMMU_ERR_DIM);
    EXPECT(ozimmu_gemm_ex(1, 0, 5, 4, 4, 1.0, fd, 4, fd, 4, 0.0, fd, 4, 8, fake, 1 << 30, nullptr), OZIMMU_ERR_DIM);
    EXPECT(ozimmu_gemm_ex(0, 1, 4, 5, 4, 1.0, fd, 5, fd, 4, 0.0, fd, 4, 8, fake, 1 << 30, nullptr), OZIMMU_ERR_DIM);
    EXPECT(ozimmu_gemm_ex(0, 0, 4, 4, 4, 1.0, fd, 4, fd, 4, 0.0, nullptr, 4, 8, fake, 1 << 30, nullptr), OZIMMU_ERR_NULL);
    EXPECT(ozimmu_gemm_ex(0, 0, 4, 4, 4, 1.0, fd, 4, fd, 4, 0.5, fd, 4, 8, fake, 16, nullptr), OZIMMU_ERR_WORKSPACE);
    EXPECT(ozimmu_split_A(4, 4, fd, 3, 8, f8, f32, nullptr), OZIMMU_ERR_DIM);
    EXPECT(ozimmu_split_A(4, 4, fd, 4, 8, reinterpret_cast<int8_t*>(4097), f32, nullptr), OZIMMU_ERR_WORKSPACE);
    EXPECT(ozimmu_split_A(4, 4, nullptr, 4, 8, f8, f32, nullptr), OZIMMU_ERR_NULL);
    EXPECT(ozimmu_split_B(4, top + 1, fd, top + 1, 8, f8, f32, nullptr), OZIMMU_ERR_DIM);
    EXPECT(ozimmu_split_B(4, 4, fd, 4, 0, f8, f32, nullptr), OZIMMU_ERR_SLICES);
    EXPECT(ozimmu_split_A_variant(4, 4, fd, 4, 8, 2, f8, f32, nullptr), OZIMMU_ERR_SLICES);
    EXPECT(ozimmu_split_B_variant(4, 4, fd, 4, 8, -1, f8, f32, nullptr), OZIMMU_ERR_SLICES);
    EXPECT(ozimmu_split_A_per_slice(4, 4, fd, 4, 8, f8, f32, nullptr, nullptr), OZIMMU_ERR_NULL);
    EXPECT(ozimmu_split_B_per_slice(4, 4, fd, 4, 8, f8, f32, reinterpret_cast<double*>(4104), nullptr),
           OZIMMU_ERR_WORKSPACE);
    EXPECT(ozimmu_gemm_group(4, 4, 4, f8, 2, f8, 2, 5, 1, 1, f32, 4, fake, nullptr), OZIMMU_ERR_SLICES);
    EXPECT(ozimmu_gemm_group(4, 4, 4, f8, 2, f8, 2, 3, 2, 1, f32, 4, fake, nullptr), OZIMMU_ERR_SLICES);
    EXPECT(ozimmu_gemm_group(4, 4, 4, f8, 2, f8, 2, 3, 1, 2, f32, 3, fake, nullptr), OZIMMU_ERR_DIM);
    EXPECT(ozimmu_gemm_group(4, 4, 4, f8, 2, f8, 2, 3, 1, 2, nullptr, 4, fake, nullptr), OZIMMU_ERR_NULL);
    EXPECT(ozimmu_gemm_group(4, 4, 4, f8, 2, f8, 2, 3, 1, 2, f32, 4, reinterpret_cast<void*>(4098), nullptr),
           OZIMMU_ERR_WORKSPACE);
    EXPECT(ozimmu_gemm_group_accumulate(4, 4, 4, f8, 2, f8, 2, 3, 1, 2, f32, f32, 1, fd, 3, fake, nullptr), OZIMMU_ERR_DIM);
    EXPECT(ozimmu_gemm_group_accumulate(4, 4, 4, f8, 2, f8, 2, 3, 1, 2, nullptr, f32, 1, fd, 4, fake, nullptr),
           OZIMMU_ERR_NULL);
    EXPECT(ozimmu_accumulate(4, 4, f32, 4, f32, f32, 0, 2, 1, fd, 4, nullptr), OZIMMU_ERR_SLICES);
    EXPECT(ozimmu_accumulate(4, 4, f32, 4, f32, f32, 7, 1, 1, fd, 4, nullptr), OZIMMU_ERR_SLICES);
    EXPECT(ozimmu_accumulate(4, 4, nullptr, 4, f32, f32, 7, 2, 1, fd, 4, nullptr), OZIMMU_ERR_NULL);
    EXPECT(ozimmu_export_slices(4, 4, 0, f8, f8, nullptr), OZIMMU_ERR_SLICES);
    EXPECT(ozimmu_export_slices(4, 4, 2, nullptr, f8, nullptr), OZIMMU_ERR_NULL);
    EXPECT(ozimmu_dgemm_static(4096, 4096, 4096, fd, 4096, fd, 4096, fd, 4096, 8, nullptr), OZIMMU_ERR_WORKSPACE);
    EXPECT(ozimmu_dgemm_static(4, 4, 4, fd, 4, fd, 4, fd, 4, 21, nullptr), OZIMMU_ERR_SLICES);
    EXPECT(ozimmu_dgemm_static(0, 4, 4, nullptr, 4, nullptr, 4, nullptr, 4, 8, nullptr), OZIMMU_OK);

    if (failures) {
        std::printf("abi sanitize driver: %d failure(s)\n", failures);
        return 1;
    }
    std::printf("abi sanitize driver ok\n");
    return 0;
}
