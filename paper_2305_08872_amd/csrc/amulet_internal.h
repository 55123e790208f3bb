// Declarations shared by the library's own translation units (not part of the
// C ABI and not used by the CPU oracle).
#ifndef AMULET_INTERNAL_H
#define AMULET_INTERNAL_H

#include <hip/hip_runtime.h>
#include <atomic>
#include <stdint.h>
#include <stdlib.h>

namespace amulet {

enum { TASK_IDENTITY = 0, TASK_DISCOUNT = 1, TASK_BOOST = 2, TASK_COUNT_GT = 3 };
// form of the threshold operand (paper Sec. 6.3): thres[j], thres[i], a constant, thres[i][j]
enum { THRES_COL = 0, THRES_ROW = 1, THRES_CONST = 2, THRES_ELEM = 3 };

// XCD-aware tile order, shared by every tiled kernel.  Workgroups are handed to the 8 XCDs
// round-robin (workgroup b runs on XCD b % 8) and each XCD has its own L2.  The tile grid of R
// is cut into 8 rectangular parts, px column parts by 8 / px row parts, and XCD x walks its
// part row tile by row tile: the workgroups resident on an XCD at any moment form a compact
// block of R that shares A rows and B columns through that L2.  px is the one of 8, 4, 2, 1
// whose largest part is smallest (ties go to more column parts), so that narrow grids and
// column counts that are not multiples of 8 still give every XCD a part.  (Used as the tile order
// when the parts cover the grid exactly, see below.)
struct XcdParts {
    int px;   // column parts
    int cw;   // column tiles per part
    int rh;   // row tiles per part
};
__host__ __device__ inline XcdParts xcd_parts(int64_t tiles_m, int64_t tiles_n)
{
    XcdParts best = {8, 0, 0};
    int64_t best_size = -1;
    for (int px = 8; px >= 1; px >>= 1) {
        const int py = 8 / px;
        const int64_t cw = (tiles_n + px - 1) / px, rh = (tiles_m + py - 1) / py;
        if (best_size < 0 || cw * rh < best_size) {
            best_size = cw * rh;
            best.px = px;
            best.cw = (int)cw;
            best.rh = (int)rh;
        }
    }
    return best;
}
// The parts cover the grid exactly (no padding) when both tile counts divide.  Otherwise some
// XCDs would get less than others, up to nothing (33 column tiles in 8 parts of 5: the last XCD
// idle, the one before it at 3 / 5), and the launch takes as long as its fullest XCD.  Then the
// tiles are put in one order instead -- column panels as wide as a part would be, row tile by
// row tile inside a panel -- and that order is cut into 8 runs of equal length (to within one
// tile): XCD x takes run x, still a compact block of R, and every XCD has the same number of tiles.
__host__ __device__ inline bool xcd_parts_exact(const XcdParts &g, int64_t tiles_m, int64_t tiles_n)
{
    return 8LL * g.cw * g.rh == tiles_m * tiles_n;
}
// places of one XCD's share of the order (the last of them may hold no tile)
__host__ __device__ inline int64_t xcd_places(int64_t tiles_m, int64_t tiles_n)
{
    const XcdParts g = xcd_parts(tiles_m, tiles_n);
    if (xcd_parts_exact(g, tiles_m, tiles_n)) return (int64_t)g.cw * g.rh;
    return (tiles_m * tiles_n + 7) / 8;
}
// workgroups to launch for a tile grid
inline int64_t xcd_grid(int64_t tiles_m, int64_t tiles_n) { return 8 * xcd_places(tiles_m, tiles_n); }
// tile of workgroup `block`; false when the workgroup is padding
__host__ __device__ inline bool xcd_tile(int block, int tiles_m, int tiles_n, int &tm, int &tn)
{
    const XcdParts g = xcd_parts(tiles_m, tiles_n);
    const int xcd = block & 7, slot = block >> 3;
    if (xcd_parts_exact(g, tiles_m, tiles_n)) {
        tn = (xcd % g.px) * g.cw + slot % g.cw;
        tm = (xcd / g.px) * g.rh + slot / g.cw;
        return tn < tiles_n && tm < tiles_m;
    }
    const int64_t tiles = (int64_t)tiles_m * tiles_n;
    const int64_t first = tiles * xcd / 8, next = tiles * (xcd + 1) / 8;   // XCD x: places [first, next)
    tm = 0;
    tn = 0;
    if (slot >= next - first) return false;
    const int64_t idx = first + slot;
    const int pw = (tiles_n + 7) / 8;                      // panel width, column tiles
    const int64_t per_panel = (int64_t)pw * tiles_m;
    const int full = tiles_n / pw;                         // panels of that width; one narrower may follow
    const int64_t p = idx / per_panel;
    if (p < full) {
        const int64_t rem = idx - p * per_panel;
        tm = (int)(rem / pw);
        tn = (int)(p * pw + rem % pw);
    } else {
        const int wl = tiles_n - full * pw;
        const int64_t rem = idx - (int64_t)full * per_panel;
        tm = (int)(rem / wl);
        tn = (int)(full * pw + rem % wl);
    }
    return true;
}

// Compute units of the current device (256 on MI355X), asked once per device.
inline int compute_units()
{
    static std::atomic<int> cached[16];   // zero-initialised; several host threads may ask at once
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) return 256;
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

// Rows `ld` elements of `elem_bytes` apart collide in the memory system (same L2 sets, same
// channel) when their pitch is a multiple of 32 KiB of at least 64 KiB (measured on the vector-ALU
// kernels; the exported amulet_pitch_collides is this rule).
inline bool pitch_collides(int64_t ld, int elem_bytes)
{
    const int64_t pitch = ld * elem_bytes;
    return ld > 0 && pitch >= 65536 && pitch % 32768 == 0;
}

// A grid dimension holds at most 2^32 - 1 work-items (workgroups x threads), fewer than the
// 2^31 - 1 workgroups a tile order can have: a longer row of workgroups goes out as several
// launches, each told in `args.block_base` where in the row it starts (the kernels add it to
// blockIdx.x).  `launch(n)` enqueues n workgroups with the current args.  Returns the first
// launch error (later parts are then not sent).
// Test seam (amulet_debug_fail_launches): while positive, each launch attempt is refused on the
// host, counted down, and reported as hipErrorLaunchFailure; nothing reaches the device.
inline std::atomic<int> g_forced_launch_failures{0};
inline bool forced_launch_failure()
{
    int n = g_forced_launch_failures.load(std::memory_order_relaxed);
    while (n > 0)
        if (g_forced_launch_failures.compare_exchange_weak(n, n - 1, std::memory_order_relaxed)) return true;
    return false;
}

template <typename Args, typename Launch>
inline hipError_t launch_row_of_blocks(Args &args, int64_t blocks, int threads, Launch launch)
{
    const int64_t max_blocks = 0xFFFFFFFFLL / threads;
    for (int64_t base = 0; base < blocks; base += max_blocks) {
        if (forced_launch_failure()) return hipErrorLaunchFailure;
        args.block_base = (int)base;
        launch((unsigned)(blocks - base < max_blocks ? blocks - base : max_blocks));
        // a refused launch (bad grid, LDS not granted, a stream in error) ends the row: the error is
        // read, and so reset, exactly once, here, and handed up as the call's status
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// Reproducible floating-point results (amulet_set_deterministic, or AMULET_DETERMINISTIC=1 in the
// environment when the library is first used): no launch splits K, so no tile is summed by
// several workgroups through float atomics, whose order of arrival differs from run to run.
inline std::atomic<int> g_deterministic{-1};   // -1: not asked yet, read the environment
inline bool k_split_allowed()
{
    int d = g_deterministic.load(std::memory_order_relaxed);
    if (d < 0) {
        const char *e = getenv("AMULET_DETERMINISTIC");
        d = (e && e[0] && e[0] != '0') ? 1 : 0;
        g_deterministic.store(d, std::memory_order_relaxed);
    }
    return d == 0;
}

// Tail split of the vector-ALU launchers.  The chip holds `round` workgroups at once (4 waves
// per SIMD) and workgroups take equally long, so a launch runs in rounds, and a last round with
// few workgroups leaves most of the chip idle for a whole K loop.  The tiles of the last round
// (or of the last two, or all of them when there is less than one round) are therefore launched
// once per k range, s ranges, when that shortens the launch: x rounds' worth of tiles then take
// ceil(x s) / s rounds.  They add their parts to R with hardware atomics and follow the whole
// tiles in the same grid, so they start as the last whole tiles finish.  Counted in real tiles:
// the blocks that pad the XCD parts to equal length come last in launch order and leave at once.
// A k range per workgroup for the streamed identity kernels: `chunk` (a multiple of the stage,
// `gran` k) made longer until the last range, K mod chunk, is empty or holds a whole stage too: the
// kernels multiply the k past a range's last whole stage from values fetched per lane, after
// streaming at least one stage.
inline int64_t chunk_with_a_whole_last_stage(int64_t K, int64_t chunk, int gran)
{
    while (chunk < K && K % chunk != 0 && K % chunk < gran) chunk += gran;
    return chunk;
}

struct TailSplit {
    int64_t base;     // first block (place in the tile order) of the split region
    int64_t blocks;   // places from there to the end of the padded order
    int splits;       // k ranges per tile
    int chunk;        // k per range, a multiple of k_align
    int64_t grid;     // blocks to launch: base + blocks * splits
};
inline bool choose_tail_split(int64_t real, int64_t wgs, int64_t round, int64_t K, int k_align, TailSplit &t)
{
    if (K < 512 || round <= 0 || real % round == 0 || !k_split_allowed()) return false;
    const int64_t tail = real % round;
    const int max_s = K / 256 < 8 ? (int)(K / 256) : 8;
    double best_cost = (double)((real + round - 1) / round);   // rounds of the plain launch
    int64_t best_region = 0;
    int best_s = 1;
    for (int two = 0; two < 2; ++two) {
        const int64_t region = tail + (two ? round : 0);
        if (region > real) break;
        for (int sp = 2; sp <= max_s; ++sp) {
            const int64_t parts = (region * sp + round - 1) / round;      // ceil(x s)
            // a k range costs a little more than its share of the K loop (set-up, atomics)
            const double cost = (double)((real - region) / round) + (double)parts / sp * (1.0 + 0.01 * sp);
            if (cost < best_cost - 0.03) { best_cost = cost; best_region = region; best_s = sp; }
        }
    }
    if (best_s <= 1) return false;
    const int64_t chunk = ((K + best_s - 1) / best_s + k_align - 1) / k_align * k_align;
    t.splits = (int)((K + chunk - 1) / chunk);
    t.chunk = (int)chunk;
    t.base = real - best_region;
    t.blocks = wgs - t.base;
    t.grid = t.base + t.blocks * t.splits;
    return t.splits > 1 && t.grid <= 0x7fffffffLL;
}

// K split of every tile for the matrix-core kernels when the tiles are few (at most four per
// compute unit).  One workgroup does not keep a compute unit's matrix cores busy: measured on
// the fp32 kernel, a unit with 1 / 2 / 3+ resident workgroups runs at 0.72 / 0.81 / 1.0 of its
// full rate (fp64, 8 waves per workgroup: 0.86 / 1.0).  With every tile launched once per k
// range, s ranges, the busiest unit of the busiest XCD (each XCD walks its own part of the tile
// grid, `part_tiles` places, on its own `units_per_xcd` units) gets n = ceil(part_tiles s /
// units_per_xcd) workgroups of 1/s of a tile each.  The estimate (n / s) / rate(n), plus 1 %
// per range for set-up and the atomic adds into R (mostly hidden behind other workgroups'
// K loops), is minimised over s <= 8 with at least 256 k per range.  Returns s (1: do not
// split).  Checked against sweeps of s = 1..8 at 144 ... 1024 tiles (fp32, K = 2048 ... 8192):
// the chosen s is within 4 % of the best one measured.
inline int choose_full_split(int64_t part_tiles, int64_t units_per_xcd, int64_t K, const double *rate,
                             int n_rates)
{
    if (!k_split_allowed()) return 1;
    const int max_s = K / 256 < 8 ? (int)(K / 256) : 8;
    int best_s = 1;
    double best = 0.0;
    for (int sp = 1; sp <= max_s; ++sp) {
        const int64_t n = (part_tiles * sp + units_per_xcd - 1) / units_per_xcd;
        const double r = rate[(n < n_rates ? n : n_rates) - 1];
        const double cost = (double)n / sp / r * (sp > 1 ? 1.0 + 0.01 * sp : 1.0);
        if (sp == 1 || cost < best - 0.02) { best = cost; best_s = sp; }
    }
    return best_s;
}

// K split of every tile for the streamed identity kernels (identity_mfma_dma.hip,
// identity_mfma_f64_dma.hip), whose workgroups hold `cap` to a compute unit and run at
// rate[c - 1] of the unit's full rate with c of them resident (fp32, measured: 0.92 / 0.985 /
// 1.0).  An XCD's `part_tiles` tiles, each launched once per k range, s ranges, are W =
// part_tiles s workgroups of K / s k each on S = units cap slots.  They run in W / S full rounds
// of cap K / s each, and the remainder either is the whole launch (spread evenly, c = ceil(W /
// units) per unit: c (K / s) / rate(c)) or follows full rounds, where the dispatcher refills the
// units that free first, so that a remainder piles up on a few units instead of spreading: after
// one full round it costs at least two workgroups' time, after two or more (the units have
// drifted apart by then) a whole round's (fp32, 1280 tiles: unsplit 123, in 3 ranges = five full
// rounds 142 TFLOP/s).  Costs are in units of one k of a tile at full rate (fp32 57.5 ns, fp64
// 115 ns).  A workgroup's set-up and write-back add `ovh_alone` (3 us: 50 / 30); a split launch
// adds its atomic adds, which the L2s retire at about 0.42 T per second for the whole chip:
// `atom_per_tile` (16384 adds: 0.68 / 0.34) x tiles x s (measured: 256 tiles in 2 ranges + 20 us,
// 64 tiles in 8 ranges + 23 us).  The s <= 1024 with at least 128 k per range and the lowest
// estimate is returned (1: do not split).  Checked against sweeps of s = 1..8 at 64 ... 1536 tiles
// (K = 512 ... 4096): the chosen s is the best or within 3 % of the best one measured.
inline int choose_stream_split(int64_t part_tiles, int64_t units, int64_t K, int cap, const double *rate,
                               double ovh_alone = 50.0, double atom_per_tile = 0.68)
{
    if (!k_split_allowed() || part_tiles <= 0 || units <= 0) return 1;
    const int max_s = K / 128 < 1024 ? (int)(K / 128) : 1024;
    int best_s = 1;
    double best = 0.0;
    // every s up to 16, then a coarser ladder (problems of a tile or two with a very long K)
    for (int sp = 1; sp <= max_s; sp = sp < 16 ? sp + 1 : sp < 64 ? sp + 8 : sp < 256 ? sp + 32 : sp + 128) {
        const int64_t W = part_tiles * sp, S = units * cap;
        const int64_t q = W / S, r = W % S;
        const double work = (double)K / sp;
        double cost = (double)q * cap * work;
        if (r > 0) {
            const int64_t c = (r + units - 1) / units;
            double left = (double)c / rate[c - 1];
            if (q == 1 && left < 2.0) left = 2.0;
            if (q >= 2) left = (double)cap;
            cost += left * work;
        }
        cost += ovh_alone;
        if (sp > 1) cost += atom_per_tile * (double)(part_tiles * 8) * sp;
        if (sp == 1 || cost < best * 0.99) { best = cost; best_s = sp; }
    }
    return best_s;
}

// Arguments of an fp32 task launch, already validated on the host.
struct MmlikeArgs {
    const float *A;
    const float *B;
    const float *thres;  // indexed as the launch's threshold form says; unused by the identity task
    const float *dis;    // dis[0..N), discount task only
    float *R;
    int64_t lda, ldb, ldr, ldt;   // ldt: row pitch of thres[i][j]
    int M, N, K;
    int transA, transB;  // operand stored transposed: a(i,k) = A[k*lda+i], b(k,j) = B[j*ldb+k]
    int vec;   // 1 when B, R and their row pitches allow 16-byte vector accesses
    int vecA;  // 1 when A and its row pitch do
    int kchunk;  // k range of one workgroup when a launch splits K (set by the launcher)
    // Tail split: blocks from tail_base on are the launch's last `tail_blocks` places of the tile
    // order, each present tail_splits times, once per k range (tail_splits <= 1: no such blocks).
    int tail_base, tail_blocks, tail_splits;
    int block_base;   // added to blockIdx.x (launch_row_of_blocks)
    int force_splits; // > 1: every tile's K in this many parts (a k-axis point of the shape grid); 0: the launcher's rule
};

// Tile shapes of the VALU kernels, laid out as the two-axis grid the greedy parameter search
// walks (paper Sec. 4.4-4.6).  Axis 0 is the k axis, the analogue of the paper's k_c (how much
// of K one unit of work covers): the depth BK of the B tile staged per barrier, and then how
// much of K one workgroup sums, K itself or K / 2, K / 4, K / 8 (the paper's sequence K,
// ceil(K / 2), ceil(K / 4), ...; the parts reach R through atomic adds).  Axis 1 is the
// workgroup's R tile from narrow to wide (the n_c analogue).
// shape id = k-axis index * VALU_TILES + tile.
//   k axis 0: BK 8    1: BK 16 (K split only where the launcher's own rule asks for it)
//          2, 3, 4: BK 16, every tile's K in 2, 4, 8 parts
//   tile 0: 4x4 per lane, 4 waves  -> 16 x 256      tile 1: 4x4, 8 waves -> 32 x 256
//   tile 2: 8x4 per lane, 8 waves  -> 64 x 256      tile 3: 4x8, 8 waves -> 32 x 512
// The identity task keeps the first two k-axis points (ids 0-7) and adds its matrix-core
// shapes (ids 8 to 12); the predicate tasks have all VALU_SHAPE_COUNT ids.
enum { VALU_DEPTHS = 2, VALU_KAXIS = 5, VALU_TILES = 4, VALU_SHAPE_COUNT = VALU_KAXIS * VALU_TILES };

struct ValuShapeDesc {
    int TM, NG, NW, BK;
    int splits;   // 0: the launcher's rule; else every tile's K in this many parts
    const char *name;
};
extern const ValuShapeDesc kValuShapes[VALU_SHAPE_COUNT];

// Arguments of an int8 join-count launch, already validated on the host.
struct CountArgs {
    const int8_t *A;
    const int8_t *B;
    int32_t *R;
    int64_t lda, ldb, ldr;
    int M, N, K;
    int Mload, Nload;  // rows of A / columns of B that exist in memory (>= M, N): a tile inside them loads without guards
    int vecA, vecB;  // 1 when the operand and its row pitch allow 16-byte loads
    int vecR;        // 1 when R and its row pitch allow 16-byte accesses
    int kchunk;      // k range of one workgroup when a launch splits K (set by the launcher)
    int block_base;  // added to blockIdx.x (launch_row_of_blocks)
    // persistent streamed kernel, where in its first tile's k range a workgroup starts: the slots
    // of an XCD in pers_groups groups, pers_group_stages stages (of 64 k) apart, and XCD x another
    // (x % pers_xcds) * pers_xcd_span / pers_xcds sixteenths of the range
    int pers_groups, pers_group_stages, pers_xcds, pers_xcd_span;
    // 1: R = the counts instead of R += (amulet_count_i8_assign): a workgroup that owns its tile
    // alone stores its sums without reading R; a launch that splits K clears R first and adds
    int assign = 0;
};
// shape 0: plain per-output loop; MFMA tiles 1: 128 x 128 (4 waves), 2: 256 x 256 (8 waves),
// 3: 128 x 256 (8 waves)
enum { COUNT_SHAPE_COUNT = 9 };
hipError_t launch_count_i8(int shape, const CountArgs &a, hipStream_t s);
// R[0..M) x [0..N) = 0 (a fill kernel: usable under graph capture)
hipError_t launch_zero_r_i32(const CountArgs &a, hipStream_t s);
// direct HBM -> LDS kernels: tile (64 * wr) x 256, wr = 2 or 4
bool count_i8_dma_eligible(const CountArgs &a, int wr);
hipError_t launch_count_i8_dma(const CountArgs &a, int wr, hipStream_t s, bool persistent = false);

// Identity task on the fp32 matrix cores; its five shape ids follow its eight VALU shapes: a
// 128 x 128 tile (4 waves, register staged), a 256 x 256 tile (16 waves), the 128 x 128 tile
// with its operands streamed HBM -> LDS through a ring of 3 or 4 stages, and a streamed 64 x 64
// tile for problems of few tiles.
enum { IDENTITY_MFMA_SHAPE = VALU_DEPTHS * VALU_TILES, IDENTITY_MFMA_BIG_SHAPE = VALU_DEPTHS * VALU_TILES + 1,
       IDENTITY_MFMA_DMA3_SHAPE = VALU_DEPTHS * VALU_TILES + 2, IDENTITY_MFMA_DMA4_SHAPE = VALU_DEPTHS * VALU_TILES + 3,
       IDENTITY_MFMA_SMALL_SHAPE = VALU_DEPTHS * VALU_TILES + 4, IDENTITY_SHAPE_COUNT = VALU_DEPTHS * VALU_TILES + 5 };
// variant = shape id - IDENTITY_MFMA_SHAPE
hipError_t launch_identity_mfma(const MmlikeArgs &a, int variant, hipStream_t s);
// the streamed kernel (identity_mfma_dma.hip)
bool identity_dma_eligible(const MmlikeArgs &a);
constexpr int ID_SMALL_STAGES = 4;   // ring depth of the streamed 64 x 64 tiles (fp32 and fp64)
hipError_t enqueue_identity_dma(const MmlikeArgs &a, int tile, int nstage, unsigned grid_x, unsigned grid_y, hipStream_t s);

template <int TASK, int TF>
hipError_t launch_mmlike_valu_task(int shape, const MmlikeArgs &a, hipStream_t s);

// Arguments of an fp64 task launch (row-major operands), already validated on the host.
struct MmlikeArgsF64 {
    const double *A;
    const double *B;
    const double *thres;
    const double *dis;
    double *R;
    int64_t lda, ldb, ldr, ldt;
    int M, N, K;
    int vec;   // 1 when B, R and their row pitches allow 16-byte vector accesses
    int vecA;  // 1 when A and its row pitch do
    int transA, transB;  // operand stored transposed: a(i,k) = A[k*lda+i], b(k,j) = B[j*ldb+k]
    int vecBt; // transposed B: 1 when B and its row pitch allow 16-byte loads along k
    int kchunk;  // k range of one workgroup when a launch splits K (set by the launcher)
    int tail_base, tail_blocks, tail_splits;   // as in MmlikeArgs
    int block_base;   // added to blockIdx.x (launch_row_of_blocks)
};
// predicate tasks: vector-ALU kernel; identity task: fp64 matrix-core kernel
// fp64 shapes of the predicate tasks: a small grid of the same two axes as the fp32 one
// (k axis: K whole, in 2, in 4 parts per tile; tile: 16 x 128 with 4 waves, 32 x 128 with 8).
enum { F64_KAXIS = 3, F64_TILES = 2, F64_SHAPE_COUNT = F64_KAXIS * F64_TILES };
hipError_t launch_mmlike_f64(int task, int form, int shape, const MmlikeArgsF64 &a, hipStream_t s);
hipError_t launch_identity_mfma_f64(const MmlikeArgsF64 &a, int tile, hipStream_t s);
// the streamed fp64 identity kernel (identity_mfma_f64_dma.hip)
bool identity_f64_dma_eligible(const MmlikeArgsF64 &a);
hipError_t enqueue_identity_f64_dma(const MmlikeArgsF64 &a, int tile, unsigned grid_x, unsigned grid_y, hipStream_t s);

// dst (cols x rows, pitch ld_dst) = transpose of src (rows x cols, pitch ld_src), bytes (pack.hip)
hipError_t launch_pack_pad_i8(int64_t rows, int64_t cols, const int8_t *src, int64_t ld_src, int8_t *dst,
                              int64_t ld_dst, int64_t rows_p, int64_t cols_p, hipStream_t s);
hipError_t launch_zero_block_i8(int8_t *dst, int64_t ld, int64_t row0, int64_t nrows, int64_t col0, int64_t ncols,
                                hipStream_t s);
hipError_t launch_transpose_i8(int64_t rows, int64_t cols, const int8_t *src, int64_t ld_src, int8_t *dst,
                               int64_t ld_dst, hipStream_t s);
// strided 2-D copy of rows x cols elements of 1, 4 or 8 bytes (pack.hip)
hipError_t launch_pack(int elem_bytes, int64_t rows, int64_t cols, const void *src, int64_t ld_src,
                       void *dst, int64_t ld_dst, hipStream_t s);

}  // namespace amulet
#endif
