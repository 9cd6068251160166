/*
 * ozimmu.h - C ABI of the gfx950 (MI355X) library that emulates FP64 matrix
 * multiplication D = A B on the INT8 matrix cores with the Ozaki scheme in its
 * "ozIMMU_H" form: round-to-nearest INT8 slices with one power-of-two scale
 * per row of A / column of B (Algorithm 8 of the paper), INT8 x INT8 -> INT32
 * products of the slice pairs (s, t) with s + t <= k + 1, products that share
 * a shift summed in INT32 in chunks of at most r (Algorithm 6 and the
 * definition of r in Section 3.2), and one shifted FP64 addition per chunk.
 *
 * Conventions
 *   - A is m x n, B is n x p, D is m x p: n is the INNER dimension (paper's
 *     notation, Section 1).  All three are row-major with leading dimensions
 *     lda >= n, ldb >= p, ldd >= p counted in elements.
 *   - Every pointer marked "device" is memory of the current HIP device,
 *     owned by the caller; the library allocates nothing.  A and B are never
 *     modified.  The only state kept between calls is the one-time set-up of a
 *     device (see ozimmu_init), guarded by a mutex: calls from several host
 *     threads are safe as long as they do not share a workspace or scratch area.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*); no
 *     call synchronises with the host.  Buffers must stay alive until the
 *     stream has run the work.
 *   - Every function returns OZIMMU_OK (0) or a negative status; nothing is
 *     enqueued when an argument check fails.  Inputs are assumed finite with
 *     no overflow / underflow in the scaling (the paper's standing assumption,
 *     Section 5); NaN / Inf inputs give unspecified numbers, never a fault.
 */
#ifndef OZIMMU_H
#define OZIMMU_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define OZIMMU_MAX_SLICES 20
/* Bytes of device scratch the chunk GEMM entry points need (scheduling counters
 * of the persistent kernel; contents on entry are irrelevant).  Calls that may
 * run at the same time must not share a scratch area. */
#define OZIMMU_SCRATCH_BYTES 512

enum {
    OZIMMU_OK = 0,
    OZIMMU_ERR_NULL = -1,       /* a required pointer is NULL */
    OZIMMU_ERR_DIM = -2,        /* negative size; m or p > 2^22 - 256; n > 2^29 (beta < 1); a leading dimension
                                   smaller than the row length or >= 2^30 */
    OZIMMU_ERR_SLICES = -3,     /* k outside 1..OZIMMU_MAX_SLICES, or g / s range invalid */
    OZIMMU_ERR_WORKSPACE = -4,  /* workspace too small or misaligned (needs 256-byte alignment) */
    OZIMMU_ERR_HIP = -5         /* a kernel launch reported a HIP error */
};

/* Human-readable text for a status code (static storage, host). */
const char *ozimmu_status_string(int status);

/* One-time set-up of the current HIP device: raises the dynamic-LDS limit of the chunk GEMM kernels,
 * reads the number of compute units and resolves the device address of the static workspace of
 * ozimmu_dgemm_static.  Every entry point that launches the chunk GEMM does this by itself on its first
 * call on a device; the set-up calls are not legal inside a HIP stream capture, so call ozimmu_init (or
 * any such entry point) once per device BEFORE capturing a graph that contains library calls.  Host;
 * idempotent; thread-safe.  Returns OZIMMU_OK or OZIMMU_ERR_HIP. */
int ozimmu_init(void);

/* beta = min(7, floor((31 - log2 n)/2))   [Section 2, the bound n 2^(2 beta) <= 2^31]  and
 * r = max(1, 2^(31 - 2 beta - ceil(log2 n)))   [Section 3.2, definition of r], host, pure.
 * Returns OZIMMU_ERR_DIM for n < 1 or n > 2^29. */
int ozimmu_params(int64_t n, int *beta, int64_t *r);

/* Number of FP64 additions per element of D (= number of INT32 chunks the
 * schedule of Algorithm 6 produces) for inner dimension n and k slices; host. */
int64_t ozimmu_num_chunks(int64_t n, int k);

/* Bytes of the packed INT8 slice stack of a matrix with `rows` scaled vectors
 * (m for A, p for B) of inner length n and k slices; host.  The packed layout
 * is private to the library (tile-major slices stored with an offset, followed
 * by the row sums that take the offset out again and a trailer naming it; use
 * ozimmu_export_slices to read the slice integers).  A stack is only ever
 * valid for the k it was made with: pass that k as kA / kB below. */
size_t ozimmu_slices_bytes(int64_t rows, int64_t n, int k);

/* Bytes of device workspace ozimmu_dgemm makes the best use of (scheduling scratch, exponents, the two slice
 * stacks and INT32 blocks of 256 x 256: one per output tile for up to 128 tiles; for outputs of fewer than 96
 * tiles one per chunk and tile, at most 4096 = 1 GiB; for larger outputs what the queue schedule takes,
 * min(ceil(tiles / 256), 3) x chunks x min(tiles, 256) blocks and a block of counters -- 1.5 GiB at k = 8 with one chunk
 * per group, more where the inner dimension makes the chunks shorter than the groups); host.  Not monotone in k (the per-chunk blocks
 * are only counted while they stay within those limits). */
size_t ozimmu_workspace_bytes(int64_t m, int64_t n, int64_t p, int k);

/* The least ozimmu_dgemm accepts (one block per output tile, at most 128): with less than
 * ozimmu_workspace_bytes the call gives the same D, but small outputs cannot take the chunk-parallel
 * schedule (see OZIMMU_SCHEDULE_CHUNK_PARALLEL below).  Monotone in m, n, p and k.  Host. */
size_t ozimmu_workspace_bytes_min(int64_t m, int64_t n, int64_t p, int k);

/* D <- A B with k slices: steps (i)-(iv) of the scheme (Section 1) as
 * Algorithm 8 (split) followed by Algorithm 6 (grouped accumulation).
 *   A, B, D      device, FP64, row-major (see above); D is overwritten.
 *   k            number of slices, 1..OZIMMU_MAX_SLICES.
 *   workspace    device, 256-byte aligned, >= ozimmu_workspace_bytes_min(m,n,p,k) bytes
 *                (ozimmu_workspace_bytes(m,n,p,k) to let small outputs run their fastest schedule).
 * m, n or p equal to 0 is valid: nothing is computed, and for n == 0 (m, p > 0)
 * D is set to +0. */
int ozimmu_dgemm(int64_t m, int64_t n, int64_t p,
                 const double *A, int64_t lda,
                 const double *B, int64_t ldb,
                 double *D, int64_t ldd,
                 int k, void *workspace, size_t workspace_bytes, void *stream);

/* ozimmu_dgemm with phase markers for profiling: caller-created HIP events
 * (hipEvent_t passed as void*, any may be NULL) are recorded on `stream`
 * before the first kernel (events[0]), after the split kernels of steps (i),
 * (ii) (events[1]) and after the last chunk kernel of steps (iii), (iv)
 * (events[2]).  events == NULL behaves exactly like ozimmu_dgemm. */
int ozimmu_dgemm_profiled(int64_t m, int64_t n, int64_t p,
                          const double *A, int64_t lda,
                          const double *B, int64_t ldb,
                          double *D, int64_t ldd,
                          int k, void *workspace, size_t workspace_bytes, void *stream,
                          void *const *events);

/* The variants the paper compares (Section 4), through the same kernels:
 *   split_mode       OZIMMU_SPLIT_NEAREST  round-to-nearest slices, ceil exponent     [Algorithm 8]
 *                    OZIMMU_SPLIT_BITMASK  bit-mask digits (truncation), floor exponent [Algorithm 3]
 *   accumulate_mode  OZIMMU_ACCUM_GROUPED  chunks of r products (Section 3.2)          [Algorithm 6]
 *                    OZIMMU_ACCUM_PER_PAIR one FP64 addition per slice pair            [Algorithm 4]
 *                    OZIMMU_ACCUM_WIDE     chunks of ozimmu_r_wide(n) products; needs OZIMMU_SPLIT_NEAREST.
 *                                          Not in the paper: its r is derived for |A''| <= 2^beta - 1, while
 *                                          round-to-nearest slices obey |A''| <= 2^(beta-1).
 *   split_mode       OZIMMU_SPLIT_NEAREST_PER_SLICE  round-to-nearest slices, each slice with a scale of
 *                    its own taken from what the earlier slices left; needs OZIMMU_ACCUM_PER_PAIR (slices
 *                    of one group no longer share a shift)                              [Algorithm 5]
 * (NEAREST, GROUPED) is ozimmu_dgemm (ozIMMU_H); (BITMASK, GROUPED) is ozIMMU_EF; (BITMASK, PER_PAIR) is the
 * earlier ozIMMU; (NEAREST_PER_SLICE, PER_PAIR) is ozIMMU_RN.  Other arguments as for ozimmu_dgemm, except
 * that the workspace holds ozimmu_workspace_bytes_variant(m,n,p,k,split_mode) bytes; an invalid mode or
 * combination returns OZIMMU_ERR_SLICES. */
enum { OZIMMU_SPLIT_NEAREST = 0, OZIMMU_SPLIT_BITMASK = 1, OZIMMU_SPLIT_NEAREST_PER_SLICE = 2 };
enum { OZIMMU_ACCUM_GROUPED = 0, OZIMMU_ACCUM_PER_PAIR = 1, OZIMMU_ACCUM_WIDE = 2 };
/* How the schedule is run; OR one of these into accumulate_mode (default: the library chooses).  The result
 * does not depend on it, bit for bit.
 *   OZIMMU_SCHEDULE_ONE_LAUNCH   the whole schedule in one persistent kernel with the FP64 accumulation
 *                                fused into the GEMM epilogue (what large outputs get when the workspace
 *                                has no room for the blocks of the queue);
 *   OZIMMU_SCHEDULE_SPLIT_INNER  for the tiles (256 x 256) that would leave most compute units idle -- an
 *                                output of at most 128 tiles, or the last, partly filled round of at most
 *                                128 tiles of a larger output: per chunk, the inner dimension is cut into
 *                                parts that run on different workgroups and add their INT32 partial sums
 *                                with integer atomics, then one accumulation kernel.  Chosen by default when
 *                                the inner dimension is long enough to pay for the extra launches; the flag
 *                                forces it wherever the inner dimension can be cut at all. */
/*   OZIMMU_SCHEDULE_CHUNK_PARALLEL  for outputs of at most 256 tiles, or the tiles of the last, partly filled round of
 *                                256 of a larger one (tiles x chunks <= 4096): one launch whose workgroups
 *                                take (chunk, inner part, tile) work items, every chunk leaving its INT32 sums in
 *                                a block of its own, and one kernel that adds the chunks of each element in the
 *                                order of Algorithm 6.  All chunks run side by side (a 1024^3 product occupies
 *                                128 compute units instead of 16).  Chosen by default for outputs of one round of
 *                                tiles (at most one per compute unit) when the
 *                                workspace has room for the blocks (ozimmu_workspace_bytes includes them,
 *                                ozimmu_workspace_bytes_min does not); the flag forces it wherever it fits and
 *                                is ignored elsewhere. */
/*   OZIMMU_SCHEDULE_QUEUE          every (chunk, tile) is a work item of one launch, handed out round by round
 *                                (256 tiles, all their chunks, longest chunks first) through a counter; an item
 *                                leaves its INT32 sums in a block, and the workgroup that completes a tile's last
 *                                block adds the tile's chunks up in the order of Algorithm 6.  The blocks are
 *                                recycled every few rounds.  The default for outputs of more tiles than compute
 *                                units; ignored where the workspace has no room for it. */
enum { OZIMMU_SCHEDULE_ONE_LAUNCH = 0x100, OZIMMU_SCHEDULE_SPLIT_INNER = 0x200, OZIMMU_SCHEDULE_CHUNK_PARALLEL = 0x400,
       OZIMMU_SCHEDULE_QUEUE = 0x800 };
int ozimmu_dgemm_variant(int64_t m, int64_t n, int64_t p,
                         const double *A, int64_t lda, const double *B, int64_t ldb,
                         double *D, int64_t ldd, int k, int split_mode, int accumulate_mode,
                         void *workspace, size_t workspace_bytes, void *stream);

/* Workspace of ozimmu_dgemm_variant: ozimmu_workspace_bytes for the shared-scale splits; for
 * OZIMMU_SPLIT_NEAREST_PER_SLICE also k exponents per row / column and the FP64 remainders of A and B
 * (8 (m inner_padded + n p) bytes more).  0 for an invalid mode.  Host. */
size_t ozimmu_workspace_bytes_variant(int64_t m, int64_t n, int64_t p, int k, int split_mode);

/* Largest power of two r_w with r_w * n * (2^(beta-1))^2 <= 2^31 - 1 (0 for n outside 1..2^29); host. */
int64_t ozimmu_r_wide(int64_t n);

/* Steps (i)-(v): C <- alpha * op(A) op(B) + beta * C, the GEMM-routine form of the scheme (Section 1,
 * step (v)), with op(X) = X (trans == 0) or X^T (trans != 0).
 *   op(A) is m x n: A is stored row-major m x n (lda >= n) or, transposed, n x m (lda >= m).
 *   op(B) is n x p: B is stored row-major n x p (ldb >= p) or, transposed, p x n (ldb >= n).
 *   C       device, m x p row-major, ldc >= p; read unless beta == 0, then overwritten.
 *   workspace  device, 256-byte aligned; at least ozimmu_workspace_bytes_min(m,n,p,k) bytes when beta == 0
 *              (the sum is then formed in C itself), plus 8 m p bytes (rounded up to 256) when beta != 0;
 *              ozimmu_workspace_bytes_ex(m,n,p,k) covers both and the fastest schedule.
 * The product D is formed exactly as by ozimmu_dgemm; then, per element, t1 = fl(alpha d),
 * t2 = fl(beta c), c = fl(t1 + t2) (three rounded FP64 operations, no fused multiply-add); with
 * beta == 0 the old C is not read and c = fl(alpha d).  Step (v) costs no pass of its own: the last
 * chunk of every output tile applies it in its epilogue.  Transposition costs nothing either: a
 * transposed operand is split by the kernel that otherwise handles the other operand.
 * m == 0 or p == 0: nothing to do; n == 0: C <- beta C (or +0 when beta == 0). */
int ozimmu_gemm_ex(int transA, int transB, int64_t m, int64_t n, int64_t p,
                   double alpha, const double *A, int64_t lda, const double *B, int64_t ldb,
                   double beta, double *C, int64_t ldc,
                   int k, void *workspace, size_t workspace_bytes, void *stream);

/* Bytes of device workspace ozimmu_gemm_ex needs when beta != 0 (ozimmu_dgemm's plus an m x p FP64 buffer for
 * the running sum, because the old C is needed until the very end); host. */
size_t ozimmu_workspace_bytes_ex(int64_t m, int64_t n, int64_t p, int k);

/* ---- phase-level entry points (the same kernels ozimmu_dgemm runs) ---- */

/* Steps (i): eA[i] = ceil(log2 max_j |a_ij|) (0 for an all-zero row) and the k
 * INT8 slices of A on the grids 2^(eA[i] + 1 - s beta), s = 1..k, rounded to
 * nearest-even   [Algorithm 8].
 *   A       device, m x n row-major, lda >= n.
 *   SA      device, ozimmu_slices_bytes(m, n, k) bytes, 256-byte aligned, packed.
 *   eA      device, int32[m].
 * beta is derived from n. */
int ozimmu_split_A(int64_t m, int64_t n, const double *A, int64_t lda, int k,
                   int8_t *SA, int32_t *eA, void *stream);

/* Step (ii): the same for the COLUMNS of B (B is split as the transpose of
 * the split of B^T, Section 2): eB[j] = ceil(log2 max_i |b_ij|), slices packed
 * with the inner index contiguous.
 *   B       device, n x p row-major, ldb >= p.
 *   SB      device, ozimmu_slices_bytes(p, n, k) bytes, 256-byte aligned, packed.
 *   eB      device, int32[p]. */
int ozimmu_split_B(int64_t n, int64_t p, const double *B, int64_t ldb, int k,
                   int8_t *SB, int32_t *eB, void *stream);

/* ozimmu_split_A / ozimmu_split_B with the split mode of ozimmu_dgemm_variant. */
int ozimmu_split_A_variant(int64_t m, int64_t n, const double *A, int64_t lda, int k, int split_mode,
                           int8_t *SA, int32_t *eA, void *stream);
int ozimmu_split_B_variant(int64_t n, int64_t p, const double *B, int64_t ldb, int k, int split_mode,
                           int8_t *SB, int32_t *eB, void *stream);

/* Steps (i) / (ii) with one scale per slice                                    [Algorithm 5]
 * For s = 1..k: e_s = ceil(log2 max |remainder|) over the row of A (column of B), 0 when nothing is
 * left; slice s = RNE(remainder / 2^(e_s + 1 - beta)); remainder reduced accordingly.
 *   eA / eB  device, k arrays of m / p exponents, slice-major: e_s of row i at eA[(s-1) m + i].
 *   rem      device scratch for the remainders, ozimmu_remainder_bytes(m, n, 0) bytes for A
 *            (m rows of the padded inner length) and ozimmu_remainder_bytes(p, n, 1) for B (n x p),
 *            16-byte aligned; contents undefined afterwards.
 * Other arguments as for ozimmu_split_A / ozimmu_split_B.  The pair product of slices s and t enters
 * D with the factor 2^(eA_s[i] + eB_t[j] + 2 - 2 beta), which ozimmu_accumulate applies when given
 * those two exponent arrays and g = 2. */
size_t ozimmu_remainder_bytes(int64_t rows, int64_t n, int by_col);
int ozimmu_split_A_per_slice(int64_t m, int64_t n, const double *A, int64_t lda, int k,
                             int8_t *SA, int32_t *eA, double *rem, void *stream);
int ozimmu_split_B_per_slice(int64_t n, int64_t p, const double *B, int64_t ldb, int k,
                             int8_t *SB, int32_t *eB, double *rem, void *stream);

/* Step (iii) for one chunk: C'' <- sum_{s = s0..s1} A''_s B''_{g-s} in INT32
 *                                              [Algorithm 6, the inner loop over s].
 * s0 == s1 gives the single pair product A''_s B''_{g-s} of Algorithm 4.
 *   SA, SB  device, packed slice stacks made with kA / kB slices.
 *   C       device, int32 m x p row-major, ldc >= p, overwritten (with zeros when n == 0).
 *   scratch device, OZIMMU_SCRATCH_BYTES bytes, 4-byte aligned.
 * Requires 1 <= s0 <= s1 <= kA and 1 <= g - s1, g - s0 <= kB.  The caller is
 * responsible for s1 - s0 + 1 <= r (no INT32 overflow, Section 5.2). */
int ozimmu_gemm_group(int64_t m, int64_t n, int64_t p,
                      const int8_t *SA, int kA, const int8_t *SB, int kB,
                      int g, int s0, int s1,
                      int32_t *C, int64_t ldc, void *scratch, void *stream);

/* Step (iv) for one chunk: D <- D + 2^(2 - beta g) diag(2^eA) FP64(C'') diag(2^eB)
 *                                              [Algorithm 6, the accumulation step].
 * first != 0: D is taken to be zero and is overwritten (the initialisation D = O of Algorithm 6).
 * beta is passed explicitly (it depends on n, which this call does not see). */
int ozimmu_accumulate(int64_t m, int64_t p, const int32_t *C, int64_t ldc,
                      const int32_t *eA, const int32_t *eB, int beta, int g, int first,
                      double *D, int64_t ldd, void *stream);

/* Steps (iii)+(iv) for one chunk in one kernel: the INT32 chunk sum stays in
 * registers and is converted, scaled and added to D in the GEMM epilogue
 * (ozimmu_dgemm runs the same kernel once, over every chunk of the schedule).  n == 0: the chunk sum is
 * zero, so D is set to +0 when first != 0 and left as it is otherwise. */
int ozimmu_gemm_group_accumulate(int64_t m, int64_t n, int64_t p,
                                 const int8_t *SA, int kA, const int8_t *SB, int kB,
                                 int g, int s0, int s1,
                                 const int32_t *eA, const int32_t *eB, int first,
                                 double *D, int64_t ldd, void *scratch, void *stream);

/* Unpack a packed slice stack into the canonical order out[s][row][l]
 * (int8, k x rows x n, dense): for A that is A''_s[i][l]; for B it is
 * B''_s[l][j] stored at out[s][j][l].  Debug / test helper. */
int ozimmu_export_slices(int64_t rows, int64_t n, int k, const int8_t *packed,
                         int8_t *out, void *stream);

/* ozimmu_dgemm for callers that cannot allocate device memory and have no workspace to hand over
 * (code under HIP graph capture, tight serving loops, harnesses that forbid allocation): the workspace is
 * a static device array of OZIMMU_STATIC_WORKSPACE_BYTES inside the library, one copy on every GPU the
 * library is loaded on, held until the process ends.  The call allocates nothing and frees nothing.
 * Arguments and results as for ozimmu_dgemm (bit-identical D).
 *   Returns OZIMMU_ERR_WORKSPACE when the call does not fit the array: the two slice stacks
 *   (ozimmu_slices_bytes), 4 (m + p) bytes of exponents and one 256 KiB block per output tile (at most 128)
 *   must stay within OZIMMU_STATIC_WORKSPACE_BYTES (1024^3 with k <= 20 and 2048^3 with k <= 5 fit).
 *   The schedules that need more room than that are simply not chosen.
 * All calls on one GPU share that GPU's array: two calls that may run at the same time on one GPU (different
 * streams, or different host threads) race and give undefined results; calls on one stream are ordered and
 * safe.  What a call needs cleared it clears itself; nothing carries over from the previous call.  Before
 * the first use inside a stream capture, call ozimmu_init on that device. */
#define OZIMMU_STATIC_WORKSPACE_BYTES ((size_t)64 << 20)
int ozimmu_dgemm_static(int64_t m, int64_t n, int64_t p,
                        const double *A, int64_t lda,
                        const double *B, int64_t ldb,
                        double *D, int64_t ldd,
                        int k, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* OZIMMU_H */
