// C ABI of the library (declared in include/ozimmu.h): argument checks, the
// host-side schedule of Algorithm 6 (groups g = 2..k+1, chunks of at most r
// consecutive s), workspace carving and kernel launches.  No allocation, no
// host synchronisation.  The only state kept between calls is what the one-time
// set-up of a device leaves behind (ozimmu_init).
#include "../../include/ozimmu.h"
#include "ozimmu_kernels.h"
#include "ozimmu_layout.h"
#include <mutex>

namespace {

// m, p <= 2^22 - 256: every grid dimension stays within the HIP limits (the column split launches
// rows_padded(p) / 64 <= 65535 workgroups along y)
constexpr int64_t MAX_OUTER = ((int64_t)1 << 22) - 256;
constexpr int64_t MAX_INNER = (int64_t)1 << 29;   // beta >= 1 (Section 2)
constexpr int64_t MAX_LD = ((int64_t)1 << 30) - 1;  // the kernels form 4 * ld in 32 bits

// Workspace of ozimmu_dgemm_static: device memory of the library itself, one copy on every GPU the library
// is loaded on.  In host code this name is only a handle for hipGetSymbolAddress; the address kernels and
// launchers get is DeviceState::static_ws.
static __device__ __align__(256) unsigned char scratch[OZIMMU_STATIC_WORKSPACE_BYTES];

constexpr int MAX_DEVICES = 64;
struct DeviceState {
    bool ready;
    int num_cu;       // compute units: size of the persistent grid
    void* static_ws;  // device address of `scratch` on this device
};
std::mutex g_state_mutex;
DeviceState g_state[MAX_DEVICES];

// State of the current device, set up on first use.
int device_state(DeviceState* out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return OZIMMU_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_state_mutex);
    DeviceState& s = g_state[dev];
    if (!s.ready) {
        if (ozk::setup_gemm_kernels() != hipSuccess) return OZIMMU_ERR_HIP;
        int ncu = 0;
        if (hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || ncu < 1)
            return OZIMMU_ERR_HIP;
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return OZIMMU_ERR_HIP;
        s.num_cu = ncu;
        s.static_ws = ptr;
        s.ready = true;
    }
    *out = s;
    return OZIMMU_OK;
}

inline int64_t align256(int64_t x) { return (x + 255) / 256 * 256; }

int beta_of(int64_t n)
{
    // floor((31 - log2 n)/2) >= b  <=>  n * 4^b <= 2^31
    int beta = 0;
    while (beta < 7 && (n << (2 * (beta + 1))) <= ((int64_t)1 << 31)) ++beta;
    return beta;
}

int64_t r_of(int64_t n, int beta)
{
    int L = 0;  // ceil(log2 n)
    while (((int64_t)1 << L) < n) ++L;
    const int ex = 31 - 2 * beta - L;
    return ex > 0 ? ((int64_t)1 << ex) : 1;
}

// largest power of two r_w with r_w * n * (2^(beta-1))^2 <= 2^31 - 1 (round-to-nearest slices obey |q| <= 2^(beta-1))
int64_t r_wide_of(int64_t n, int beta)
{
    int64_t r = 1;
    const int64_t lim = ((int64_t)1 << 31) - 1;
    while (2 * r * n * ((int64_t)1 << (2 * beta - 2)) <= lim) r *= 2;
    return r;
}

int dgemm_impl(int64_t m, int64_t n, int64_t p, const double* A, int64_t lda, const double* B, int64_t ldb,
               double* D, int64_t ldd, int k, int split_mode, int accumulate_mode, void* workspace,
               size_t workspace_bytes, void* stream, void* const* events);

// The split-inner way of running the schedule (see run_schedule) works on at most this many 256 x 256 tiles
// at a time: outputs that small as a whole, or the last, partly filled round of tiles of a larger output
// (half the 256 compute units of the chip this is written for: every tile can then be cut at least in two).
// A constant, so that the workspace size does not depend on the device.
constexpr int64_t SPLIT_INNER_MAX_TILES = 128;
inline int64_t output_tiles(int64_t m, int64_t p)
{
    return (ozl::rows_padded(m) / ozl::TILE_R) * (ozl::rows_padded(p) / ozl::TILE_R);
}
// The chunk-parallel way (see run_schedule) keeps one block per (chunk, tile): used for outputs of fewer tiles than
// the chip has compute units whose tiles times chunks stay within this many blocks (1 GiB).
constexpr int64_t CHUNK_PARALLEL_MAX_BLOCKS = 4096;
// Inner dimensions above this make the persistent kernel wait for the whole grid at chunk starts.
constexpr int64_t GRID_WAIT_MIN_INNER = 8192 + 512;
// Sets of blocks the rounds of the queue schedule take in turn (see run_schedule).
constexpr int64_t QUEUE_SETS = 3;
// Outputs of at least this many tiles take the queue by default, unless they are one round of tiles (one per compute
// unit at most) whose blocks fit the chunk-parallel way.
constexpr int64_t QUEUE_MIN_TILES = 96;
constexpr int64_t QUEUE_XCD_WORDS = 8 * 40;  // per-XCD ticket batches of the queue (see k_gemm)
constexpr int64_t BLOCK_BYTES = 4 * 256 * 256;
inline int64_t chunks_of(int k, int64_t r)
{
    int64_t w = 0;
    for (int g = 2; g <= k + 1; ++g) w += ((g - 1) + r - 1) / r;
    return w;
}
// INT32 blocks of 256 x 256 behind the slice stacks: what the split-inner way needs at least ...
inline int64_t min_partial_blocks(int64_t m, int64_t p)
{
    const int64_t T = output_tiles(m, p);
    return T < SPLIT_INNER_MAX_TILES ? T : SPLIT_INNER_MAX_TILES;
}
// ... and what ozimmu_workspace_bytes asks for, so that the chunk-parallel way can be used where it applies
inline int64_t partial_blocks(int64_t m, int64_t n, int64_t p, int k)
{
    const int64_t base = min_partial_blocks(m, p);
    if (n < 1 || n > MAX_INNER || k < 1) return base;
    // (the chunk-parallel way takes the tiles that do not fill a round of the 256 compute units of the chip this is
    // written for; the queue, which takes outputs of QUEUE_MIN_TILES tiles and more, wants up to QUEUE_SETS sets of chunks x 256
    // blocks and a counter per tile and round)
    const int64_t T = output_tiles(m, p);
    const int64_t w = chunks_of(k, r_of(n, beta_of(n)));
    const int64_t items = (T <= 256 ? T : T % 256) * w;
    int64_t blocks = (items <= CHUNK_PARALLEL_MAX_BLOCKS && items > base) ? items : base;
    if (T >= QUEUE_MIN_TILES && w * 256 * BLOCK_BYTES < ((int64_t)1 << 31) && T * w < ((int64_t)1 << 30)) {
        const int64_t rounds = (T + 255) / 256;
        const int64_t queue = (rounds < QUEUE_SETS ? rounds : QUEUE_SETS) * w * (T < 256 ? T : 256) +
                              (4 * (T + rounds + 2 + QUEUE_XCD_WORDS) + BLOCK_BYTES - 1) / BLOCK_BYTES;
        if (queue > blocks) blocks = queue;
    }
    return blocks;
}
// the least a call of ozimmu_dgemm can run in (no room for the chunk-parallel blocks)
inline size_t min_workspace_bytes(int64_t m, int64_t n, int64_t p, int k)
{
    return (size_t)(align256(OZIMMU_SCRATCH_BYTES) + align256(4 * m) + align256(4 * p)) +
           (size_t)ozl::stack_bytes(m, n, k) + (size_t)ozl::stack_bytes(p, n, k) +
           (size_t)(min_partial_blocks(m, p) * BLOCK_BYTES);
}

inline int hip_status(hipError_t e) { return e == hipSuccess ? OZIMMU_OK : OZIMMU_ERR_HIP; }

int check_gemm_args(int64_t m, int64_t n, int64_t p, const void* SA, int kA, const void* SB, int kB, int g, int s0,
                    int s1)
{
    if (m < 0 || n < 0 || p < 0 || m > MAX_OUTER || p > MAX_OUTER || n > MAX_INNER) return OZIMMU_ERR_DIM;
    if (kA < 1 || kA > OZIMMU_MAX_SLICES || kB < 1 || kB > OZIMMU_MAX_SLICES) return OZIMMU_ERR_SLICES;
    if (s0 < 1 || s1 < s0 || s1 > kA || g - s1 < 1 || g - s0 > kB) return OZIMMU_ERR_SLICES;
    if (m == 0 || n == 0 || p == 0) return OZIMMU_OK;
    if (!SA || !SB) return OZIMMU_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(SA) % 256 || reinterpret_cast<uintptr_t>(SB) % 256) return OZIMMU_ERR_WORKSPACE;
    return OZIMMU_OK;
}

// Offset of the stored bytes (see ozimmu_layout.h): round-to-nearest slices obey |q| <= 2^(beta-1), so the offset
// 2^(beta-1) - 1 (63 for beta = 7) moves them into [-1, 2^beta - 1]: inside the magnitude 2^beta - 1 for which the
// paper derives the chunk length r, so no INT32 sum of a chunk can overflow with the stored bytes either.  Bit-mask
// slices (|q| <= 2^beta - 1) have no room for an offset, and neither have the wide chunks, whose length is derived
// from |q| <= 2^(beta-1).
inline int rn_offset(int beta) { return (1 << (beta - 1)) - 1; }

// single chunk (s0 > 0): g, s = s0..s1; full schedule (s0 == 0): g = g_lo..g_hi, chunks of r.
// SA / SB are whole stacks of kA / kB slices (slices, prefix row sums, trailer).
ozk::GemmArgs make_args(int64_t m, int64_t n, int64_t p, const int8_t* SA, int kA, const int8_t* SB, int kB, int g_lo,
                        int g_hi, int r, int s0, int s1, void* scratch, int num_cu)
{
    ozk::GemmArgs a{};
    a.num_cu = num_cu;
    a.SA = SA;
    a.SB = SB;
    a.PA = reinterpret_cast<const int32_t*>(SA + ozl::sums_offset(m, n, kA));
    a.PB = reinterpret_cast<const int32_t*>(SB + ozl::sums_offset(p, n, kB));
    a.pstrideA = ozl::rows_padded(m);
    a.pstrideB = ozl::rows_padded(p);
    a.cA = reinterpret_cast<const int32_t*>(SA + ozl::trailer_offset(m, n, kA));
    a.cB = reinterpret_cast<const int32_t*>(SB + ozl::trailer_offset(p, n, kB));
    a.strideA = ozl::slice_bytes(m, n);
    a.strideB = ozl::slice_bytes(p, n);
    a.KT = (int)(ozl::inner_padded(n) / ozl::TILE_K);
    a.g_lo = g_lo;
    a.g_hi = g_hi;
    a.r = r;
    a.s0 = s0;
    a.s1 = s1;
    a.m = m;
    a.p = p;
    a.beta = beta_of(n);
    a.tile_begin = 0;
    a.tile_count = (int)((ozl::rows_padded(m) / ozl::TILE_R) * (ozl::rows_padded(p) / ozl::TILE_R));
    a.zsplit = 1;
    a.sync = static_cast<unsigned*>(scratch);
    a.spin_limit = 64;  // polls (about 0.1 us each) before a workgroup stops waiting for its team
    // the grid-wide wait pays only when the operand panels are long (see arrive_and_wait2)
    a.grid_spin_limit = n > GRID_WAIT_MIN_INNER ? 64 : 0;
    a.sync_epoch = 0;
    a.alpha = 1.0;
    return a;
}

// Step (v) applied by the last chunk of every tile: out = fl(fl(alpha d) + fl(cbeta c_old)).
struct Finish {
    bool on;
    double alpha, cbeta;
    double* Cout;   // == D when cbeta == 0 (the sum is formed in C itself)
    int64_t ldco;
};

// Steps (iii) + (iv) (+ (v), see Finish) for the whole schedule of Algorithm 6 (groups g = 2..k+1 ascending, chunks
// of at most r consecutive s), into D.  Four ways to run it, with bit-identical results (details where each is
// decided below):
//  * the queue: one launch whose work items are the (chunk, tile) pairs, an INT32 block per item, the tile's chunks
//    added up by the workgroup that completes it -- the default for outputs of more tiles than compute units (and
//    from QUEUE_MIN_TILES tiles on where the chunk-parallel way has no room) when the workspace holds the blocks;
//  * one persistent launch with the accumulation fused into the GEMM epilogue (mode 1, or 2 for per-slice
//    scales): one workgroup per compute unit takes tile after tile, all chunks of a tile in turn -- needs no
//    blocks;
//  * chunk-parallel, for outputs of few tiles or the last, partly filled round after a persistent launch: one
//    launch whose work items are (chunk, inner part, tile), a block per chunk and tile, then one accumulation
//    kernel over those tiles;
//  * split-inner, for the same tiles when there is room for one block per tile only: per chunk, the chunk GEMM
//    with its inner range cut into Z parts on Z workgroups per tile, which add their partial sums to zeroed
//    per-tile INT32 blocks with integer atomics, then the accumulation kernel over those tiles, which also clears
//    the blocks again.
// schedule: 0 = choose, or one of the OZIMMU_SCHEDULE_* flags (honoured when possible).
int run_schedule(int64_t m, int64_t n, int64_t p, const int8_t* SA, const int8_t* SB, const int32_t* eA,
                 const int32_t* eB, int k, int64_t r, bool per_slice, int schedule, double* D, int64_t ldd,
                 const Finish& fin, int32_t* partial, int64_t partial_capacity, void* scratch, int num_cu, hipStream_t st,
                 bool sync_clean = false)
{
    // sync_clean: the caller has already zeroed the soft-barrier counters in `scratch` (the first GEMM launch
    // then need not; later ones of the same call find them used and do)
    auto take_clean = [&]() -> int {
        const int c = sync_clean ? 1 : 0;
        sync_clean = false;
        return c;
    };
    const int beta = beta_of(n);
    const int r_eff = (int)(r < k ? r : k);
    const int KT = (int)(ozl::inner_padded(n) / ozl::TILE_K);
    const int64_t T = output_tiles(m, p);
    const int64_t w = chunks_of(k, r_eff);

    // Fourth way ("queue"), for the tiles [0, tiles) of the band order: one launch whose work items are all
    // (chunk, tile) pairs, handed out round by round (256 tiles) through a counter; an item leaves its INT32 sums
    // in a block, and the workgroup that stores the last block of a tile adds the tile's chunks up (steps (iv),
    // (v)).  Needs sets x chunks x min(tiles, 256) blocks (the rounds take the sets in turn) and a counter per
    // tile and round.  Against the persistent launch with the fused epilogue it moves 4 + 4 bytes per element
    // and chunk instead of 16, and no workgroup ever waits for another (measured 3 to 4 % faster at 16384^3,
    // 2 % at 8192^3, k = 8).  queue_sets: how many sets fit (0: the way cannot be used for that many tiles).
    auto queue_sets = [&](int64_t tiles) -> int64_t {
        if (per_slice || !partial || tiles < 1 || tiles * w >= ((int64_t)1 << 30)) return 0;
        const int64_t stride = tiles < ozk::QUEUE_ROUND_TILES ? tiles : ozk::QUEUE_ROUND_TILES;
        if (w * stride * BLOCK_BYTES >= ((int64_t)1 << 31)) return 0;  // 32-bit byte offsets inside a set of blocks
        const int64_t rounds = (tiles + ozk::QUEUE_ROUND_TILES - 1) / ozk::QUEUE_ROUND_TILES;
        const int64_t counter_blocks = (4 * (tiles + rounds + 2 + QUEUE_XCD_WORDS) + BLOCK_BYTES - 1) / BLOCK_BYTES;
        int64_t sets = rounds < QUEUE_SETS ? rounds : QUEUE_SETS;
        while (sets > 1 && sets * w * stride + counter_blocks > partial_capacity) --sets;
        if (sets * w * stride + counter_blocks > partial_capacity) return 0;
        return (sets >= 2 || rounds == 1) ? sets : 0;
    };
    auto launch_queue = [&](int64_t tiles, int64_t sets) -> int {
        const int64_t stride = tiles < ozk::QUEUE_ROUND_TILES ? tiles : ozk::QUEUE_ROUND_TILES;
        const int64_t rounds = (tiles + ozk::QUEUE_ROUND_TILES - 1) / ozk::QUEUE_ROUND_TILES;
        int32_t* const ctr = partial + sets * w * stride * (BLOCK_BYTES / 4);
        // counters: one per tile, one per round, the flag; then, 8-byte aligned, the per-XCD ticket batches
        const int64_t xq_at = (tiles + rounds + 2) & ~(int64_t)1;
        hipError_t e = ozk::launch_fill_zero_i32(xq_at + QUEUE_XCD_WORDS, ctr, st);
        if (e != hipSuccess) return OZIMMU_ERR_HIP;
        ozk::GemmArgs a = make_args(m, n, p, SA, k, SB, k, 2, k + 1, r_eff, 0, 0, scratch, num_cu);
        a.tile_count = (int)tiles;
        a.C = partial;
        a.zsplit = 1;
        a.nchunks = (int)w;
        a.queue_sets = (int)sets;
        a.queue_stride = (int)stride;
        const int64_t TM = ozl::rows_padded(m) / ozl::TILE_R, TP = ozl::rows_padded(p) / ozl::TILE_R;
        a.queue_block_rounds = (tiles == T && TM % 16 == 0 && TP % 16 == 0) ? 1 : 0;
        a.done = reinterpret_cast<unsigned*>(ctr);
        // batches of 32 tickets per XCD when every compute unit of the 8-XCD chip this is written for has a workgroup
        a.xq = (tiles >= num_cu && num_cu == 256) ? reinterpret_cast<unsigned*>(ctr) + xq_at : nullptr;
        a.D = D;
        a.ldd = ldd;
        a.eA = eA;
        a.eB = eB;
        a.finish = fin.on ? 1 : 0;
        a.alpha = fin.alpha;
        a.cbeta = fin.cbeta;
        a.Cout = fin.Cout;
        a.ldco = fin.ldco;
        a.spin_limit = 0;  // the items of a team are different chunks: nothing to line up
        a.grid_spin_limit = 0;
        a.sync_zeroed = take_clean();
        return hip_status(ozk::launch_gemm(a, 3, st));
    };
    // Asked for, or the output has more tiles than compute units (measured against queue for the full rounds +
    // one of the other ways for a short last round: equal or better with everything in the queue), or at least
    // QUEUE_MIN_TILES and no room for the chunk-parallel way.  An output of one round of tiles whose blocks fit
    // goes the chunk-parallel way further down: every compute unit gets items from the first moment, and the one
    // accumulation kernel at the end costs less than the queue's ramp (k = 8, chunk-parallel against queue:
    // 2560^3, 100 tiles, 0.53 against 0.58 ms; 3072^3 0.87 against 0.92; 4096^3, 256 tiles, 1.87 against 1.89;
    // 5120^3, 400 tiles, with the queue for the full round only: 3.60 against 3.43).
    const bool one_round_fits = !per_slice && partial && T <= num_cu && T * w <= CHUNK_PARALLEL_MAX_BLOCKS &&
                                T * w <= partial_capacity;
    if (schedule == OZIMMU_SCHEDULE_QUEUE || (schedule == 0 && T >= QUEUE_MIN_TILES && !one_round_fits)) {
        const int64_t sets = queue_sets(T);
        if (sets > 0) return launch_queue(T, sets);
    }

    // Third way, for outputs of few tiles, or the tiles of a partly filled last round (`cand`, the last ones in band
    // order): ONE launch whose work items are (chunk, inner part, tile), every chunk writing (or, when cut,
    // atomically adding) its INT32 sums to a block of its own per tile, and one kernel that adds the chunks of every
    // element in the order of Algorithm 6.  All chunks of all those tiles run side by side, so a 1024^3 product
    // occupies 128 compute units instead of 16; the price is 4 bytes of workspace per element and chunk.
    const int64_t cand = num_cu > 0 ? (T <= num_cu ? T : T % num_cu) : 0;  // tiles of the last round, if not full or the only one
    int64_t cp_tail = 0;  // tiles that go this way
    int cp_z = 1;
    if (!per_slice && partial && cand >= 1 && cand * w <= CHUNK_PARALLEL_MAX_BLOCKS && cand * w <= partial_capacity &&
        schedule != OZIMMU_SCHEDULE_ONE_LAUNCH && schedule != OZIMMU_SCHEDULE_SPLIT_INNER) {
        // (measured on MI355X: a stage 0.58 us; prologue + epilogue of an item 12 us, 19 us when the epilogue adds
        // with atomics; clearing the blocks 5 us + 0.065 us per block; the accumulation kernel 15 us + 0.058 us
        // per block)
        const double stage_us = 0.58;
        const double pairs = (double)k * (k + 1) / 2;
        const int longest = r_eff < k ? r_eff : k;  // pairs of the longest chunk
        const double blocks = (double)(cand * w);
        // one more round of the persistent launch: every tile at once, chunks in sequence, each with a fused
        // epilogue in which all workgroups update D at the same time (measured 2.0 ms at 4096^3, k = 8)
        const double one_launch_us = 0.60 * pairs * KT + 50.0 * (double)w;
        double best = 0.0;
        int best_z = 0;
        const int zmax = KT / 4 > 0 ? KT / 4 : 1;
        for (int z = 1; z <= zmax; z *= 2) {
            const double item_us = z > 1 ? 19.0 : 12.0;
            const double total = (double)cand * (stage_us * pairs * KT + item_us * (double)w * z);
            const double longest_item = stage_us * longest * KT / z + item_us;
            // items are handed out longest first to whichever workgroup is free: the last ones end unevenly
            double t = total / (double)num_cu + 0.25 * longest_item;
            if (t < longest_item) t = longest_item;
            t += 15.0 + 0.058 * blocks;               // the accumulation kernel
            if (z > 1) t += 5.0 + 0.065 * blocks;     // clearing the blocks for the atomic adds
            if (best_z == 0 || t < best) {
                best = t;
                best_z = z;
            }
        }
        if (schedule == OZIMMU_SCHEDULE_CHUNK_PARALLEL || best < 0.97 * one_launch_us) {
            cp_tail = cand;
            cp_z = best_z;
        }
    }
    if (cp_tail == 0 && one_round_fits && schedule == 0 && T >= QUEUE_MIN_TILES) {
        // (the model preferred the persistent launch to the chunk-parallel way: the queue beats that one)
        const int64_t sets = queue_sets(T);
        if (sets > 0) return launch_queue(T, sets);
    }

    // tiles [0, T - tail) go to the persistent launch, the last `tail` tiles (band order) are cut Z ways
    int64_t tail = 0;
    int Z = 1;
    if (!per_slice && partial && cp_tail == 0 && schedule != OZIMMU_SCHEDULE_ONE_LAUNCH &&
        schedule != OZIMMU_SCHEDULE_CHUNK_PARALLEL) {
        const int64_t ncu = num_cu;
        const int64_t zmax = KT / 4;  // every part gets at least one group of 4 stages of the shortest chunk
        if (cand >= 1 && cand <= SPLIT_INNER_MAX_TILES && zmax >= 2) {
            // Time per chunk in microseconds, from measurements on MI355X: a stage of the main loop takes
            // 0.58 us; the fused path pays about 35 us per chunk and tile for epilogue and prologue, a part of
            // the cut path about 15 us (atomic epilogue, prologue), and every chunk of the cut path about 15 us
            // of launches plus the accumulation pass over the tail tiles (20 bytes per element at 4.5 TB/s).
            const double chunk_us = 0.58 * (double)k * (k + 1) / 2 * KT / (double)w;  // average chunk of one tile
            const double fused_us = chunk_us + 35.0;  // one more round of the persistent launch
            const double fixed_us = 15.0 + 0.29 * (double)cand;
            double best = 0.0;
            int64_t best_z = 0;
            // one round only: cutting finer and running the parts in several rounds measured slower than the
            // fused path even where this model favours it (3072 x 16384 x 3072: 8.0 against 6.0 ms)
            for (int64_t z = 2; z <= zmax && cand * z <= ncu; ++z) {
                const double t = chunk_us / (double)z + 15.0 + fixed_us;
                if (best_z == 0 || t < best) {
                    best = t;
                    best_z = z;
                }
            }
            if (best_z && (schedule == OZIMMU_SCHEDULE_SPLIT_INNER || best < 0.9 * fused_us)) {
                tail = cand;
                Z = (int)best_z;
            }
        }
    }
    if (T - tail - cp_tail > 0) {
        ozk::GemmArgs a = make_args(m, n, p, SA, k, SB, k, 2, k + 1, r_eff, 0, 0, scratch, num_cu);
        a.tile_count = (int)(T - tail - cp_tail);
        a.D = D;
        a.ldd = ldd;
        a.eA = eA;
        a.eB = eB;
        a.estrideA = m;
        a.estrideB = p;
        a.first = 1;
        a.finish = fin.on ? 1 : 0;
        a.alpha = fin.alpha;
        a.cbeta = fin.cbeta;
        a.Cout = fin.Cout;
        a.ldco = fin.ldco;
        a.sync_zeroed = take_clean();
        const hipError_t e = ozk::launch_gemm(a, per_slice ? 2 : 1, st);
        if (e != hipSuccess) return OZIMMU_ERR_HIP;
    }
    if (cp_tail > 0) {
        hipError_t e = hipSuccess;
        if (cp_z > 1) e = ozk::launch_fill_zero_i32(cp_tail * w * 256 * 256, partial, st);
        if (e != hipSuccess) return OZIMMU_ERR_HIP;
        ozk::GemmArgs a = make_args(m, n, p, SA, k, SB, k, 2, k + 1, r_eff, 0, 0, scratch, num_cu);
        a.tile_begin = (int)(T - cp_tail);
        a.tile_count = (int)cp_tail;
        a.C = partial;
        a.zsplit = cp_z;
        a.nchunks = (int)w;
        a.spin_limit = 0;  // the items of a team are different chunks: nothing to line up
        a.grid_spin_limit = 0;
        a.sync_zeroed = take_clean();
        e = ozk::launch_gemm(a, 3, st);
        if (e != hipSuccess) return OZIMMU_ERR_HIP;
        ozk::TileAccArgs t{};
        t.tile_begin = (int)(T - cp_tail);
        t.tile_count = (int)cp_tail;
        t.m = m;
        t.p = p;
        t.Ct = partial;
        t.parts = cp_z;
        t.eA = eA;
        t.eB = eB;
        t.D = D;
        t.ldd = ldd;
        t.finish = fin.on ? 1 : 0;
        t.alpha = fin.alpha;
        t.cbeta = fin.cbeta;
        t.Cout = fin.Cout;
        t.ldco = fin.ldco;
        return hip_status(ozk::launch_accumulate_chunks(t, k, r_eff, beta, st));
    }
    if (tail == 0) return OZIMMU_OK;
    int first = 1;
    int epoch = 0;
    hipError_t e = ozk::launch_fill_zero_i32(tail * 256 * 256, partial, st);  // later chunks find it cleared
    if (e != hipSuccess) return OZIMMU_ERR_HIP;
    for (int g = 2; g <= k + 1; ++g)
        for (int s0 = 1; s0 <= g - 1; s0 += r_eff) {
            const int s1 = s0 + r_eff - 1 < g - 1 ? s0 + r_eff - 1 : g - 1;
            ozk::GemmArgs a = make_args(m, n, p, SA, k, SB, k, g, g, s1 - s0 + 1, s0, s1, scratch, num_cu);
            a.tile_begin = (int)(T - tail);
            a.tile_count = (int)tail;
            a.C = partial;
            a.zsplit = Z;
            a.sync_epoch = epoch++;
            a.sync_zeroed = take_clean();
            e = ozk::launch_gemm(a, 3, st);
            if (e != hipSuccess) return OZIMMU_ERR_HIP;
            ozk::TileAccArgs t{};
            t.tile_begin = (int)(T - tail);
            t.tile_count = (int)tail;
            t.m = m;
            t.p = p;
            t.Ct = partial;
            t.parts = Z;
            t.eA = eA;
            t.eB = eB;
            t.shift = 2 - beta * g;
            t.first = first;
            t.D = D;
            t.ldd = ldd;
            const bool last = (g == k + 1 && s1 == g - 1);
            t.finish = (fin.on && last) ? 1 : 0;
            t.alpha = fin.alpha;
            t.cbeta = fin.cbeta;
            t.Cout = fin.Cout;
            t.ldco = fin.ldco;
            e = ozk::launch_accumulate_tiles(t, st);
            if (e != hipSuccess) return OZIMMU_ERR_HIP;
            first = 0;
        }
    return OZIMMU_OK;
}

}  // namespace

extern "C" {

const char* ozimmu_status_string(int status)
{
    switch (status) {
        case OZIMMU_OK: return "ok";
        case OZIMMU_ERR_NULL: return "null pointer argument";
        case OZIMMU_ERR_DIM: return "invalid dimension or leading dimension";
        case OZIMMU_ERR_SLICES: return "invalid slice count or slice range";
        case OZIMMU_ERR_WORKSPACE: return "workspace too small or misaligned";
        case OZIMMU_ERR_HIP: return "HIP launch error";
        default: return "unknown status";
    }
}

int ozimmu_params(int64_t n, int* beta, int64_t* r)
{
    if (n < 1 || n > MAX_INNER) return OZIMMU_ERR_DIM;
    const int b = beta_of(n);
    if (beta) *beta = b;
    if (r) *r = r_of(n, b);
    return OZIMMU_OK;
}

int64_t ozimmu_num_chunks(int64_t n, int k)
{
    if (n < 1 || n > MAX_INNER || k < 1) return 0;
    const int64_t r = r_of(n, beta_of(n));
    int64_t w = 0;
    for (int g = 2; g <= k + 1; ++g) w += ((g - 1) + r - 1) / r;
    return w;
}

size_t ozimmu_slices_bytes(int64_t rows, int64_t n, int k)
{
    if (rows < 0 || n < 0 || k < 0) return 0;
    return (size_t)ozl::stack_bytes(rows, n, k);
}

size_t ozimmu_workspace_bytes(int64_t m, int64_t n, int64_t p, int k)
{
    if (m < 0 || n < 0 || p < 0 || k < 0) return 0;
    return (size_t)(align256(OZIMMU_SCRATCH_BYTES) + align256(4 * m) + align256(4 * p)) +
           ozimmu_slices_bytes(m, n, k) + ozimmu_slices_bytes(p, n, k) + (size_t)(partial_blocks(m, n, p, k) * BLOCK_BYTES);
}

size_t ozimmu_workspace_bytes_min(int64_t m, int64_t n, int64_t p, int k)
{
    if (m < 0 || n < 0 || p < 0 || k < 0) return 0;
    return min_workspace_bytes(m, n, p, k);
}

int ozimmu_split_A(int64_t m, int64_t n, const double* A, int64_t lda, int k, int8_t* SA, int32_t* eA, void* stream)
{
    if (m < 0 || n < 0 || m > MAX_OUTER || n > MAX_INNER || lda < n || lda > MAX_LD) return OZIMMU_ERR_DIM;
    if (k < 1 || k > OZIMMU_MAX_SLICES) return OZIMMU_ERR_SLICES;
    if (m == 0 || n == 0) return OZIMMU_OK;
    if (!A || !SA || !eA) return OZIMMU_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(SA) % 256) return OZIMMU_ERR_WORKSPACE;
    return hip_status(ozk::launch_split_A(m, n, A, lda, k, beta_of(n), 0, rn_offset(beta_of(n)), SA, eA, (hipStream_t)stream));
}

int ozimmu_split_B(int64_t n, int64_t p, const double* B, int64_t ldb, int k, int8_t* SB, int32_t* eB, void* stream)
{
    if (p < 0 || n < 0 || p > MAX_OUTER || n > MAX_INNER || ldb < p || ldb > MAX_LD) return OZIMMU_ERR_DIM;
    if (k < 1 || k > OZIMMU_MAX_SLICES) return OZIMMU_ERR_SLICES;
    if (p == 0 || n == 0) return OZIMMU_OK;
    if (!B || !SB || !eB) return OZIMMU_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(SB) % 256) return OZIMMU_ERR_WORKSPACE;
    return hip_status(ozk::launch_split_B(n, p, B, ldb, k, beta_of(n), 0, rn_offset(beta_of(n)), SB, eB, (hipStream_t)stream));
}

int ozimmu_gemm_group(int64_t m, int64_t n, int64_t p, const int8_t* SA, int kA, const int8_t* SB, int kB, int g,
                      int s0, int s1, int32_t* C, int64_t ldc, void* scratch, void* stream)
{
    int st = check_gemm_args(m, n, p, SA, kA, SB, kB, g, s0, s1);
    if (st != OZIMMU_OK) return st;
    if (ldc < p || ldc > MAX_LD) return OZIMMU_ERR_DIM;
    if (m == 0 || p == 0) return OZIMMU_OK;
    if (!C) return OZIMMU_ERR_NULL;
    if (n == 0) return hip_status(ozk::launch_fill_zero_i32_2d(m, p, C, ldc, (hipStream_t)stream));  // empty sum
    if (!scratch) return OZIMMU_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(scratch) % 4) return OZIMMU_ERR_WORKSPACE;
    DeviceState ds;
    st = device_state(&ds);
    if (st != OZIMMU_OK) return st;
    const int num_cu = ds.num_cu;
    ozk::GemmArgs a = make_args(m, n, p, SA, kA, SB, kB, g, g, s1 - s0 + 1, s0, s1, scratch, num_cu);
    a.C = C;
    a.ldc = ldc;
    return hip_status(ozk::launch_gemm(a, 0, (hipStream_t)stream));
}

int ozimmu_accumulate(int64_t m, int64_t p, const int32_t* C, int64_t ldc, const int32_t* eA, const int32_t* eB,
                      int beta, int g, int first, double* D, int64_t ldd, void* stream)
{
    if (m < 0 || p < 0 || m > MAX_OUTER || p > MAX_OUTER || ldc < p || ldd < p || ldc > MAX_LD || ldd > MAX_LD)
        return OZIMMU_ERR_DIM;
    if (beta < 1 || beta > 7 || g < 2 || g > 2 * OZIMMU_MAX_SLICES) return OZIMMU_ERR_SLICES;
    if (m == 0 || p == 0) return OZIMMU_OK;
    if (!C || !eA || !eB || !D) return OZIMMU_ERR_NULL;
    return hip_status(
        ozk::launch_accumulate(m, p, C, ldc, eA, eB, 2 - beta * g, first, D, ldd, (hipStream_t)stream));
}

int ozimmu_gemm_group_accumulate(int64_t m, int64_t n, int64_t p, const int8_t* SA, int kA, const int8_t* SB, int kB,
                                 int g, int s0, int s1, const int32_t* eA, const int32_t* eB, int first, double* D,
                                 int64_t ldd, void* scratch, void* stream)
{
    int st = check_gemm_args(m, n, p, SA, kA, SB, kB, g, s0, s1);
    if (st != OZIMMU_OK) return st;
    if (ldd < p || ldd > MAX_LD) return OZIMMU_ERR_DIM;
    if (m == 0 || p == 0) return OZIMMU_OK;
    if (!D) return OZIMMU_ERR_NULL;
    if (n == 0)  // empty sum: D <- D + 0, or D <- +0 when D is taken to be zero
        return first ? hip_status(ozk::launch_fill_zero_f64(m, p, D, ldd, (hipStream_t)stream)) : OZIMMU_OK;
    if (!eA || !eB || !scratch) return OZIMMU_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(scratch) % 4) return OZIMMU_ERR_WORKSPACE;
    DeviceState ds;
    st = device_state(&ds);
    if (st != OZIMMU_OK) return st;
    const int num_cu = ds.num_cu;
    ozk::GemmArgs a = make_args(m, n, p, SA, kA, SB, kB, g, g, s1 - s0 + 1, s0, s1, scratch, num_cu);
    a.D = D;
    a.ldd = ldd;
    a.eA = eA;
    a.eB = eB;
    a.first = first;
    return hip_status(ozk::launch_gemm(a, 1, (hipStream_t)stream));
}

int ozimmu_export_slices(int64_t rows, int64_t n, int k, const int8_t* packed, int8_t* out, void* stream)
{
    if (rows < 0 || n < 0 || rows > MAX_OUTER || n > MAX_INNER) return OZIMMU_ERR_DIM;
    if (k < 1 || k > OZIMMU_MAX_SLICES) return OZIMMU_ERR_SLICES;
    if (rows == 0 || n == 0) return OZIMMU_OK;
    if (!packed || !out) return OZIMMU_ERR_NULL;
    return hip_status(ozk::launch_export(rows, n, k, packed, out, (hipStream_t)stream));
}

size_t ozimmu_workspace_bytes_ex(int64_t m, int64_t n, int64_t p, int k)
{
    if (m < 0 || n < 0 || p < 0 || k < 0) return 0;
    return ozimmu_workspace_bytes(m, n, p, k) + (size_t)align256(8 * m * p);
}

int ozimmu_gemm_ex(int transA, int transB, int64_t m, int64_t n, int64_t p, double alpha, const double* A,
                   int64_t lda, const double* B, int64_t ldb, double beta, double* C, int64_t ldc, int k,
                   void* workspace, size_t workspace_bytes, void* stream)
{
    if (m < 0 || n < 0 || p < 0 || m > MAX_OUTER || p > MAX_OUTER || n > MAX_INNER) return OZIMMU_ERR_DIM;
    if (lda < (transA ? m : n) || ldb < (transB ? n : p) || ldc < p) return OZIMMU_ERR_DIM;
    if (lda > MAX_LD || ldb > MAX_LD || ldc > MAX_LD) return OZIMMU_ERR_DIM;
    if (k < 1 || k > OZIMMU_MAX_SLICES) return OZIMMU_ERR_SLICES;
    if (m == 0 || p == 0) return OZIMMU_OK;
    if (!C) return OZIMMU_ERR_NULL;
    hipStream_t st = (hipStream_t)stream;
    if (n == 0) {  // empty product: C <- beta C
        if (beta == 0.0) return hip_status(ozk::launch_fill_zero_f64(m, p, C, ldc, st));
        return hip_status(ozk::launch_axpby(m, p, 0.0, nullptr, 0, beta, C, ldc, st));
    }
    if (!A || !B || !workspace) return OZIMMU_ERR_NULL;
    // beta == 0: the sum is formed in C itself, no m x p buffer
    const size_t need = min_workspace_bytes(m, n, p, k) + (beta == 0.0 ? (size_t)0 : (size_t)align256(8 * m * p));
    if (reinterpret_cast<uintptr_t>(workspace) % 256 || workspace_bytes < need) return OZIMMU_ERR_WORKSPACE;

    DeviceState ds;
    const int drc = device_state(&ds);
    if (drc != OZIMMU_OK) return drc;
    const int bt = beta_of(n);
    const int64_t r = r_of(n, bt);
    char* ws = static_cast<char*>(workspace);
    void* scratch = ws;
    ws += align256(OZIMMU_SCRATCH_BYTES);
    int32_t* eA = reinterpret_cast<int32_t*>(ws);
    ws += align256(4 * m);
    int32_t* eB = reinterpret_cast<int32_t*>(ws);
    ws += align256(4 * p);
    int8_t* SA = reinterpret_cast<int8_t*>(ws);
    ws += ozimmu_slices_bytes(m, n, k);
    int8_t* SB = reinterpret_cast<int8_t*>(ws);
    ws += ozimmu_slices_bytes(p, n, k);
    double* Dw = reinterpret_cast<double*>(ws);  // beta != 0 only
    if (beta != 0.0) ws += align256(8 * m * p);
    int32_t* partial = reinterpret_cast<int32_t*>(ws);  // the rest: INT32 blocks, as many as there is room for
    const int64_t blocks = (int64_t)((static_cast<char*>(workspace) + workspace_bytes - ws) / BLOCK_BYTES);

    // op(A): one scale per row of op(A).  Stored transposed (n x m), those rows are the columns of the
    // stored matrix, which is what the column-wise split kernel handles; likewise for op(B).
    hipError_t e = transA ? ozk::launch_split_B(n, m, A, lda, k, bt, 0, rn_offset(bt), SA, eA, st)
                          : ozk::launch_split_A(m, n, A, lda, k, bt, 0, rn_offset(bt), SA, eA, st);
    if (e != hipSuccess) return OZIMMU_ERR_HIP;
    e = transB ? ozk::launch_split_A(p, n, B, ldb, k, bt, 0, rn_offset(bt), SB, eB, st)
               : ozk::launch_split_B(n, p, B, ldb, k, bt, 0, rn_offset(bt), SB, eB, st, static_cast<uint32_t*>(scratch),
                                     ozk::SYNC_WORDS);
    if (e != hipSuccess) return OZIMMU_ERR_HIP;

    // Step (v) rides on the epilogue of every tile's last chunk.  beta == 0: the running sum lives in C and the
    // last chunk stores fl(alpha d) there.  Otherwise the running sum lives in the workspace buffer and the last
    // chunk reads the old C and writes the new one.
    const bool in_place = beta == 0.0;
    const Finish fin = {!(alpha == 1.0 && beta == 0.0), alpha, beta, C, ldc};
    return run_schedule(m, n, p, SA, SB, eA, eB, k, r, false, 0, in_place ? C : Dw, in_place ? ldc : p, fin, partial,
                        blocks, scratch, ds.num_cu, st, !transB);
}

int ozimmu_dgemm(int64_t m, int64_t n, int64_t p, const double* A, int64_t lda, const double* B, int64_t ldb,
                 double* D, int64_t ldd, int k, void* workspace, size_t workspace_bytes, void* stream)
{
    return ozimmu_dgemm_profiled(m, n, p, A, lda, B, ldb, D, ldd, k, workspace, workspace_bytes, stream, nullptr);
}

int ozimmu_dgemm_profiled(int64_t m, int64_t n, int64_t p, const double* A, int64_t lda, const double* B,
                          int64_t ldb, double* D, int64_t ldd, int k, void* workspace, size_t workspace_bytes,
                          void* stream, void* const* events)
{
    return dgemm_impl(m, n, p, A, lda, B, ldb, D, ldd, k, OZIMMU_SPLIT_NEAREST, OZIMMU_ACCUM_GROUPED, workspace,
                      workspace_bytes, stream, events);
}

size_t ozimmu_remainder_bytes(int64_t rows, int64_t n, int by_col)
{
    if (rows < 0 || n < 0) return 0;
    return (size_t)8 * (size_t)rows * (size_t)(by_col ? n : ozl::inner_padded(n));
}

size_t ozimmu_workspace_bytes_variant(int64_t m, int64_t n, int64_t p, int k, int split_mode)
{
    if (m < 0 || n < 0 || p < 0 || k < 0) return 0;
    if (split_mode == OZIMMU_SPLIT_NEAREST || split_mode == OZIMMU_SPLIT_BITMASK)
        return ozimmu_workspace_bytes(m, n, p, k);
    if (split_mode != OZIMMU_SPLIT_NEAREST_PER_SLICE) return 0;
    return (size_t)(align256(OZIMMU_SCRATCH_BYTES) + align256(4 * (int64_t)k * m) + align256(4 * (int64_t)k * p)) +
           ozimmu_slices_bytes(m, n, k) + ozimmu_slices_bytes(p, n, k) +
           (size_t)align256((int64_t)ozimmu_remainder_bytes(m, n, 0)) +
           (size_t)align256((int64_t)ozimmu_remainder_bytes(p, n, 1));
}

int ozimmu_split_A_per_slice(int64_t m, int64_t n, const double* A, int64_t lda, int k, int8_t* SA, int32_t* eA,
                             double* rem, void* stream)
{
    if (m < 0 || n < 0 || m > MAX_OUTER || n > MAX_INNER || lda < n || lda > MAX_LD) return OZIMMU_ERR_DIM;
    if (k < 1 || k > OZIMMU_MAX_SLICES) return OZIMMU_ERR_SLICES;
    if (m == 0 || n == 0) return OZIMMU_OK;
    if (!A || !SA || !eA || !rem) return OZIMMU_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(SA) % 256 || reinterpret_cast<uintptr_t>(rem) % 16) return OZIMMU_ERR_WORKSPACE;
    return hip_status(ozk::launch_split_A_per_slice(m, n, A, lda, k, beta_of(n), SA, eA, rem, (hipStream_t)stream));
}

int ozimmu_split_B_per_slice(int64_t n, int64_t p, const double* B, int64_t ldb, int k, int8_t* SB, int32_t* eB,
                             double* rem, void* stream)
{
    if (p < 0 || n < 0 || p > MAX_OUTER || n > MAX_INNER || ldb < p || ldb > MAX_LD) return OZIMMU_ERR_DIM;
    if (k < 1 || k > OZIMMU_MAX_SLICES) return OZIMMU_ERR_SLICES;
    if (p == 0 || n == 0) return OZIMMU_OK;
    if (!B || !SB || !eB || !rem) return OZIMMU_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(SB) % 256 || reinterpret_cast<uintptr_t>(rem) % 16) return OZIMMU_ERR_WORKSPACE;
    return hip_status(ozk::launch_split_B_per_slice(n, p, B, ldb, k, beta_of(n), SB, eB, rem, (hipStream_t)stream));
}

int ozimmu_dgemm_variant(int64_t m, int64_t n, int64_t p, const double* A, int64_t lda, const double* B, int64_t ldb,
                         double* D, int64_t ldd, int k, int split_mode, int accumulate_mode, void* workspace,
                         size_t workspace_bytes, void* stream)
{
    const int flags = accumulate_mode & ~0xff, amode = accumulate_mode & 0xff;
    if (split_mode < OZIMMU_SPLIT_NEAREST || split_mode > OZIMMU_SPLIT_NEAREST_PER_SLICE) return OZIMMU_ERR_SLICES;
    if (amode < OZIMMU_ACCUM_GROUPED || amode > OZIMMU_ACCUM_WIDE) return OZIMMU_ERR_SLICES;
    if (flags != 0 && flags != OZIMMU_SCHEDULE_ONE_LAUNCH && flags != OZIMMU_SCHEDULE_SPLIT_INNER &&
        flags != OZIMMU_SCHEDULE_CHUNK_PARALLEL && flags != OZIMMU_SCHEDULE_QUEUE)
        return OZIMMU_ERR_SLICES;
    if (amode == OZIMMU_ACCUM_WIDE && split_mode != OZIMMU_SPLIT_NEAREST) return OZIMMU_ERR_SLICES;
    if (split_mode == OZIMMU_SPLIT_NEAREST_PER_SLICE && amode != OZIMMU_ACCUM_PER_PAIR) return OZIMMU_ERR_SLICES;
    return dgemm_impl(m, n, p, A, lda, B, ldb, D, ldd, k, split_mode, accumulate_mode, workspace, workspace_bytes,
                      stream, nullptr);
}

int ozimmu_split_A_variant(int64_t m, int64_t n, const double* A, int64_t lda, int k, int split_mode, int8_t* SA,
                           int32_t* eA, void* stream)
{
    if (m < 0 || n < 0 || m > MAX_OUTER || n > MAX_INNER || lda < n || lda > MAX_LD) return OZIMMU_ERR_DIM;
    if (k < 1 || k > OZIMMU_MAX_SLICES || (split_mode != 0 && split_mode != 1)) return OZIMMU_ERR_SLICES;
    if (m == 0 || n == 0) return OZIMMU_OK;
    if (!A || !SA || !eA) return OZIMMU_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(SA) % 256) return OZIMMU_ERR_WORKSPACE;
    return hip_status(ozk::launch_split_A(m, n, A, lda, k, beta_of(n), split_mode, split_mode == 0 ? rn_offset(beta_of(n)) : 0, SA, eA,
                                          (hipStream_t)stream));
}

int ozimmu_split_B_variant(int64_t n, int64_t p, const double* B, int64_t ldb, int k, int split_mode, int8_t* SB,
                           int32_t* eB, void* stream)
{
    if (p < 0 || n < 0 || p > MAX_OUTER || n > MAX_INNER || ldb < p || ldb > MAX_LD) return OZIMMU_ERR_DIM;
    if (k < 1 || k > OZIMMU_MAX_SLICES || (split_mode != 0 && split_mode != 1)) return OZIMMU_ERR_SLICES;
    if (p == 0 || n == 0) return OZIMMU_OK;
    if (!B || !SB || !eB) return OZIMMU_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(SB) % 256) return OZIMMU_ERR_WORKSPACE;
    return hip_status(ozk::launch_split_B(n, p, B, ldb, k, beta_of(n), split_mode, split_mode == 0 ? rn_offset(beta_of(n)) : 0, SB, eB,
                                          (hipStream_t)stream));
}

int ozimmu_init(void)
{
    DeviceState ds;
    return device_state(&ds);
}

int ozimmu_dgemm_static(int64_t m, int64_t n, int64_t p, const double* A, int64_t lda, const double* B, int64_t ldb,
                        double* D, int64_t ldd, int k, void* stream)
{
    if (m < 0 || n < 0 || p < 0 || m > MAX_OUTER || p > MAX_OUTER || n > MAX_INNER) return OZIMMU_ERR_DIM;
    if (k < 1 || k > OZIMMU_MAX_SLICES) return OZIMMU_ERR_SLICES;
    if (min_workspace_bytes(m, n, p, k) > (size_t)OZIMMU_STATIC_WORKSPACE_BYTES) return OZIMMU_ERR_WORKSPACE;
    if (m == 0 || p == 0) return OZIMMU_OK;
    DeviceState ds;
    const int rc = device_state(&ds);
    if (rc != OZIMMU_OK) return rc;
    return dgemm_impl(m, n, p, A, lda, B, ldb, D, ldd, k, OZIMMU_SPLIT_NEAREST, OZIMMU_ACCUM_GROUPED, ds.static_ws,
                      (size_t)OZIMMU_STATIC_WORKSPACE_BYTES, stream, nullptr);
}

int64_t ozimmu_r_wide(int64_t n)
{
    if (n < 1 || n > MAX_INNER) return 0;
    return r_wide_of(n, beta_of(n));
}

}  // extern "C"

namespace {

int dgemm_impl(int64_t m, int64_t n, int64_t p, const double* A, int64_t lda, const double* B, int64_t ldb,
               double* D, int64_t ldd, int k, int split_mode, int accumulate_mode, void* workspace,
               size_t workspace_bytes, void* stream, void* const* events)
{
    if (m < 0 || n < 0 || p < 0 || m > MAX_OUTER || p > MAX_OUTER || n > MAX_INNER) return OZIMMU_ERR_DIM;
    if (lda < n || ldb < p || ldd < p || lda > MAX_LD || ldb > MAX_LD || ldd > MAX_LD) return OZIMMU_ERR_DIM;
    if (k < 1 || k > OZIMMU_MAX_SLICES) return OZIMMU_ERR_SLICES;
    if (m == 0 || p == 0) return OZIMMU_OK;
    if (!D) return OZIMMU_ERR_NULL;
    hipStream_t st = (hipStream_t)stream;
    if (n == 0) return hip_status(ozk::launch_fill_zero_f64(m, p, D, ldd, st));
    if (!A || !B || !workspace) return OZIMMU_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(workspace) % 256 ||
        workspace_bytes < (split_mode == OZIMMU_SPLIT_NEAREST_PER_SLICE
                               ? ozimmu_workspace_bytes_variant(m, n, p, k, split_mode)
                               : min_workspace_bytes(m, n, p, k)))
        return OZIMMU_ERR_WORKSPACE;
    DeviceState ds;
    const int drc = device_state(&ds);
    if (drc != OZIMMU_OK) return drc;

    const int schedule =
        accumulate_mode & (OZIMMU_SCHEDULE_ONE_LAUNCH | OZIMMU_SCHEDULE_SPLIT_INNER | OZIMMU_SCHEDULE_CHUNK_PARALLEL |
                           OZIMMU_SCHEDULE_QUEUE);
    accumulate_mode &= 0xff;
    const int beta = beta_of(n);
    const bool per_slice = split_mode == OZIMMU_SPLIT_NEAREST_PER_SLICE;
    const int64_t ne = per_slice ? k : 1;  // exponent arrays per operand
    const int64_t r = accumulate_mode == OZIMMU_ACCUM_PER_PAIR
                          ? 1
                          : (accumulate_mode == OZIMMU_ACCUM_WIDE ? r_wide_of(n, beta) : r_of(n, beta));
    char* ws = static_cast<char*>(workspace);
    void* scratch = ws;
    ws += align256(OZIMMU_SCRATCH_BYTES);
    int32_t* eA = reinterpret_cast<int32_t*>(ws);
    ws += align256(4 * ne * m);
    int32_t* eB = reinterpret_cast<int32_t*>(ws);
    ws += align256(4 * ne * p);
    int8_t* SA = reinterpret_cast<int8_t*>(ws);
    ws += ozimmu_slices_bytes(m, n, k);
    int8_t* SB = reinterpret_cast<int8_t*>(ws);
    ws += ozimmu_slices_bytes(p, n, k);
    double* remA = reinterpret_cast<double*>(ws);  // per-slice split only
    double* remB = reinterpret_cast<double*>(ws + align256((int64_t)ozimmu_remainder_bytes(m, n, 0)));

    auto mark = [&](int i) -> hipError_t {
        return (events && events[i]) ? hipEventRecord((hipEvent_t)events[i], st) : hipSuccess;
    };
    hipError_t e = mark(0);
    if (e != hipSuccess) return OZIMMU_ERR_HIP;
    const int offset = (split_mode == OZIMMU_SPLIT_NEAREST && accumulate_mode != OZIMMU_ACCUM_WIDE) ? rn_offset(beta) : 0;
    e = per_slice ? ozk::launch_split_A_per_slice(m, n, A, lda, k, beta, SA, eA, remA, st)
                  : ozk::launch_split_A(m, n, A, lda, k, beta, split_mode, offset, SA, eA, st);
    if (e != hipSuccess) return OZIMMU_ERR_HIP;
    e = per_slice ? ozk::launch_split_B_per_slice(n, p, B, ldb, k, beta, SB, eB, remB, st)
                  : ozk::launch_split_B(n, p, B, ldb, k, beta, split_mode, offset, SB, eB, st,
                                        static_cast<uint32_t*>(scratch), ozk::SYNC_WORDS);
    if (e != hipSuccess) return OZIMMU_ERR_HIP;
    e = mark(1);
    if (e != hipSuccess) return OZIMMU_ERR_HIP;

    int32_t* partial = nullptr;  // INT32 partial sums of few-tile outputs, behind the slices
    if (!per_slice) partial = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(SB) + ozimmu_slices_bytes(p, n, k));
    const Finish no_finish = {false, 1.0, 0.0, D, ldd};
    // blocks of 256 x 256 INT32 the rest of the workspace holds (decides whether the chunk-parallel way fits)
    int64_t capacity = 0;
    if (partial)
        capacity = (int64_t)((static_cast<char*>(workspace) + workspace_bytes - reinterpret_cast<char*>(partial)) /
                             BLOCK_BYTES);
    const int rc = run_schedule(m, n, p, SA, SB, eA, eB, k, r, per_slice, schedule, D, ldd, no_finish, partial,
                                capacity, scratch, ds.num_cu, st, !per_slice);
    if (rc != OZIMMU_OK) return rc;
    return hip_status(mark(2));
}

}  // namespace
