// moe_expert_ffn: grouped expert FFN  y = act(x W1^T + b1) W2^T + b2  over expert-contiguous rows.
//
// Two launches of one grouped "NT" GEMM kernel  C[rows of e, N] = A[rows, K] * B_e[N, K]^T
// (both operands have the reduction dimension contiguous): the first with the bias+GELU
// epilogue writing the hidden activations of the A rows to the workspace (bf16: in a layout of their
// own that the accumulators can be stored to without a transposition, see RowMap), the second writing y.
// The per-expert row ranges are read from expert_offsets ON THE DEVICE: the grid is sized for
// the worst case (ceil(A/MT) + E_local row tiles) and every workgroup locates its own
// (expert, row tile, column tile) with a wavefront scan; surplus workgroups exit at once.
//
// bf16 kernel (gfx950 matrix cores)
//   - macro tile MT x NT x KT, WM x WN wavefronts, each owning (MT/WM) x (NT/WN) as 32x32 MFMA
//     tiles (v_mfma_f32_32x32x16_bf16, fp32 accumulators).
//   - global -> LDS with direct-to-LDS 16-byte loads (no staging registers), STAGES-deep ring,
//     one workgroup barrier per K tile, placed in the middle of a K step so that MFMAs are in
//     flight on both sides of it.  A direct-to-LDS load writes 64 lanes x 16 B contiguously, so
//     the LDS layout is fixed; bank conflicts on the MFMA operand reads are avoided by choosing
//     WHICH 16-byte chunk of a row each lane fetches (XOR swizzle applied on the global side).
//   - the weight tile feeds the MFMA row axis and the activation tile the column axis, so a lane
//     ends up with 4 consecutive output columns of one row; the epilogue transposes through LDS
//     and stores 16-byte chunks of contiguous row segments.
//   - workgroup -> tile order: consecutive ids go round-robin to the 8 XCDs, so id%8 selects the
//     XCD and every XCD walks contiguous ranges of tiles ordered (expert, column tile, row tile):
//     the workgroups resident on one XCD share an expert's activation rows and a few weight
//     panels in that XCD's L2.  When that would leave an XCD much more work than the others (a
//     short launch of tiles of different heights), every kind of tile is split evenly instead.
//   - remainder ("tail") tiles of the second contraction are cut into K slices when there are few of
//     them, and a small kernel adds the slices (see TileSchedule).
// fp32 kernel: LDS-tiled 64x64x16, 4x4 outputs per thread (tiny configuration; latency bound).
#include <math.h>

#include "common.hpp"

namespace exf {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

constexpr int kXcdCount = 8;

// ---------------------------------------------------------------------------- activations
__device__ __forceinline__ float gelu_erf_exact(float z) { return 0.5f * z * (1.0f + erff(z * 0.70710678118654752440f)); }
__device__ __forceinline__ float gelu_tanh_exact(float z)
{
    return 0.5f * z * (1.0f + tanhf(0.79788456080286535588f * (z + 0.044715f * z * z * z)));
}

// bf16 path: z * Phi(z) with the normal CDF evaluated as a logistic function of an odd
// polynomial,  Phi(z) ~ 1 / (1 + exp(-z (c0 + c1 z^2 + c2 z^4))),  coefficients fitted (minimax
// on [-10,10]) to the exact erf form: max |error| of the GELU value is 2.6e-5, two orders of
// magnitude below the bf16 rounding the result receives next.  z^2 is clamped where the logistic
// has long saturated, so that the quartic term cannot turn the polynomial around.
__device__ __forceinline__ float gelu_erf_fast(float z)
{
    const float t = fminf(z * z, 60.0f);
    // coefficients carry the factor -log2(e): exp(-z p(t)) = 2^(z q(t)), one v_exp_f32
    float q = fmaf(1.01407394e-3f, t, -1.06774916e-1f);
    q = fmaf(q, t, -2.30112032f);
    const float e = __builtin_amdgcn_exp2f(z * q);
    return z * __builtin_amdgcn_rcpf(1.0f + e);  // v_rcp_f32: 1 ulp
}
// z/2 (1 + tanh u) = z / (1 + exp(-2u))
__device__ __forceinline__ float gelu_tanh_fast(float z)
{
    const float u = 0.79788456080286535588f * (z + 0.044715f * z * z * z);
    return z * __builtin_amdgcn_rcpf(1.0f + __expf(-2.0f * u));
}

enum Epilogue { kEpiNone = 0, kEpiGeluErf = 1, kEpiGeluTanh = 2 };


// ---------------------------------------------------------------------------- tile lookup
// Rows of expert e are cut into "full" row tiles of MT rows.  A remainder of at most MT/2 rows is
// cut into "tail" row tiles of kTailRows rows, so that a small remainder costs in proportion to
// its size instead of a whole tile; a larger remainder becomes one more full tile whose missing
// rows are masked (a tail tile does a quarter of the MFMA work of a 256-row tile but loads the
// same weight panel, so three or four of them cost more than the one masked tile).  Both kinds are
// numbered (expert, column tile, row tile); locate_tile() says which kind a launch runs first.
constexpr int kTailRows = 64;
constexpr int kHiddenRowBlock = 32;  // rows whose 16-byte pieces are contiguous in the hidden layout
constexpr uint32_t kHiddenPieceStride = kHiddenRowBlock * 16;  // bytes from piece c to piece c+1 of a row
// byte offset of the 16-byte piece `piece` (8 columns) of hidden row h; pieces = pieces per row.  (A larger
// distance between the pieces of a row - 4, 8, 32 KiB - measured the same.)
__host__ __device__ inline size_t hidden_offset(uint32_t h, uint32_t piece, uint32_t pieces)
{
    return (static_cast<size_t>(h / kHiddenRowBlock) * pieces + piece) * kHiddenPieceStride + (h % kHiddenRowBlock) * 16;
}
__host__ __device__ constexpr int max_tail_tiles(int mt) { return mt / 2 >= kTailRows ? (mt / 2 + kTailRows - 1) / kTailRows : 1; }
constexpr int kXcdChunk = 32;  // consecutive tiles handed to one XCD at a time: one per compute unit of the XCD
constexpr int kLdsBytes = 160 * 1024;  // LDS of a compute unit
// A tile configuration can run tall tiles (MT + kTailRows rows) if its wavefront rows still split into
// 32-row MFMA tiles and the taller stages still fit the LDS.
__host__ __device__ constexpr bool tall_tiles_supported(int mt, int nt, int kt, int stages, int wm)
{
    return mt > kTailRows && ((mt + kTailRows) / wm) % 32 == 0 && (mt + kTailRows) % wm == 0 &&
           stages * (mt + kTailRows + nt) * kt * 2 <= kLdsBytes;
}

// Optional row indirections of the bf16 grouped GEMM; all members null / zero = sorted rows on both sides.
// They let the contraction read the tokens where they lie (no sorted copy of the activations) and
// let the second contraction of a top-1 layer write the gate-weighted result straight to the
// token's own row (no sorted copy of the outputs, no separate combine pass).
struct RowMap {
    const int32_t* a_row;     // operand row of sorted row s is a_row[s] / a_div        (null: row s)
    int a_div;
    const int32_t* out_row;   // output row of sorted row s is out_row[s]; every output row is the
    const float* out_scale;   //   target of at most one s and is scaled by out_scale[out_row[s]] in
                              //   fp32 before the single rounding to bf16              (null: row s, no scale)
    const int32_t* unrouted;  // [n_unrouted]: output row t with unrouted[t] < 0 is set to zero
    int n_unrouted;
    // The hidden activations between the two contractions live in a layout of their own (nobody else
    // reads them): 16-byte pieces (8 columns) of 32 consecutive rows are contiguous,
    //   byte address of (row h, column n) = ((h / 32) * (N / 8) + n / 8) * 512 + (h % 32) * 16 + (n % 8) * 2,
    // and every expert starts on a 32-row boundary: sorted row m of expert e is hidden row
    // m + 32 e - (first row of e) % 32.  The first contraction can then store its accumulators as they
    // lie in the registers (a lane holds 4 consecutive columns of a row; one swap between the two halves
    // of the wavefront makes that 8), 1 KiB per store instruction, without the transposition through
    // LDS, and the second contraction's direct-to-LDS loads fetch whole 128-byte lines as before.
    int hidden_out;           // != 0: `out` is the hidden buffer in that layout (first contraction)
    int hidden_act;           // != 0: `act` is the hidden buffer in that layout (second contraction)
    // Measurement only (exf_probe_ffn_timeline; null in every other call): workgroup b < timeline_cap
    // writes eight 64-bit words - [0] start, [1] tile located, [2] first K tile landed, [3] K loop done,
    // [4] end (all on the constant 100 MHz clock), [5] hardware id, [6] tile kind / expert / column tile /
    // rows / K tiles, [7] the experts' row ranges have arrived (between [0] and [1]).
    unsigned long long* timeline;
    int timeline_cap;
};

__device__ __forceinline__ void timeline_stamp(const RowMap& map, int slot)
{
    if (map.timeline != nullptr && threadIdx.x == 0 && static_cast<int>(blockIdx.x) < map.timeline_cap)
        map.timeline[static_cast<size_t>(blockIdx.x) * 8 + slot] = wall_clock64();
}

// LDS of a launch: the ring of STAGES stages of the tallest tile, and behind it (two-stage rings, if it
// still fits) a scratch area for the row ids of gathered activation rows: 256 bytes per wavefront-wide
// load of the tallest tile.
__host__ __device__ constexpr int ring_bytes(int mt, int nt, int kt, int stages, int wm)
{
    return stages * (mt + (tall_tiles_supported(mt, nt, kt, stages, wm) ? kTailRows : 0) + nt) * kt * 2;
}
__host__ __device__ constexpr int row_id_scratch_bytes(int mt, int nt, int kt, int stages, int wm, int waves)
{
    const int rows = mt + (tall_tiles_supported(mt, nt, kt, stages, wm) ? kTailRows : 0);
    const int bytes = rows / (1024 / (kt * 2)) * 256;  // one 256-byte line per load of 1024/(2 kt) rows
    return (stages == 2 && rows % (1024 / (kt * 2) * waves) == 0 && ring_bytes(mt, nt, kt, stages, wm) + bytes <= kLdsBytes) ? bytes : 0;
}

struct Tile2D {
    int expert;
    int row_begin, row_end;
    int n_tile;
    bool tail;
    bool tall;             // a full tile extended by kTailRows rows (see TileSchedule)
    int kt_begin, kt_end;  // K tiles [kt_begin, kt_end) of the reduction this workgroup sums
    int slot;              // >= 0: the sum goes to partial-sum slot `slot` (a K slice of a tail tile)
    int hid_shift;         // hidden row of sorted row m of this expert: m + hid_shift (see RowMap)
};

// Tail tiles hold a quarter of the rows of a full tile but walk the same reduction: one takes nearly
// half as long as a full tile (28 against 62 us in the second contraction of 8192 tokens) while only
// a few compute units have one.
// When there are few of them, each is therefore cut into `split` K slices that run side by side as
// workgroups of their own; a slice writes its fp32 partial sums to a slot of the workspace and a
// small second kernel adds the slices and applies the epilogue.  split * (number of tail tiles)
// never exceeds kSplitUnits, which bounds the slots.
constexpr int kSplitUnits = 256;    // one slice per compute unit
constexpr int kSplitMaxCols = 256;  // widest tile a partial-sum slot is sized for
constexpr size_t kSplitBytes = static_cast<size_t>(kSplitUnits) * kTailRows * kSplitMaxCols * sizeof(float);
constexpr int kSplitMinKTiles = 4;  // shortest K slice worth a workgroup (2 and 8 measured the same)
constexpr int kSplitMax = 8;        // most K slices per tail tile
// Only the second contraction slices: its reduction is the long one, and in the first contraction the
// kernel that adds the slices (and applies GELU) cost more than the slices saved.
constexpr bool kSplitFirstContraction = false;

// Workgroup id -> work item.  Consecutive workgroup ids are dealt round-robin to the 8 XCDs, so id % 8
// is the XCD and id / 8 the position in that XCD's queue; an XCD only ever runs its own queue.  Two
// ways to fill the queues from the launch's list of work items (see locate_tile for its order):
//   chunked : chunks of kXcdChunk consecutive items go to one XCD after the other.  The 32 compute
//             units of an XCD then walk one block of tiles in step and meet its few activation and
//             weight panels in their L2 - the faster way per tile (3 % at ten rounds of tiles).
//   balanced: every kind of item (tall, full and tail tiles differ several-fold in duration) is split
//             evenly over the XCDs: of the n items of a kind, XCD x takes a contiguous share of n/8,
//             and the n%8 left over go one each to consecutive XCDs, continuing where the previous
//             kind stopped.  With chunks, a launch of two or three rounds leaves some XCDs a whole
//             chunk of long tiles more than others (700 against 580 us for the second contraction of
//             a skewed 32-expert batch), and a one-round launch of 8 experts x 32 tiles puts halves of
//             two experts on an XCD instead of one expert (L2 hit rate 0.71 against 0.78).
// A launch of at most kBalancedMaxRounds rounds of work items, or of items of one kind only (contiguous shares
// then cost nothing: all tiles take the same time), is balanced, a longer mixed one chunked: same-run
// timings of the whole call (chunked / balanced, us): 8192 tokens (two rounds per launch) 157.2 / 153.8;
// 256 tokens x 64 experts (two to four rounds of remainder tiles) 2997 / 2894; skewed 32 experts (ten and
// 2.5 rounds) 1313 / 1225 with both launches balanced and as good with only the short one; 32768 tokens on
// 8 experts (eight and two rounds) 549 / 564 on one box and equal on another.
constexpr int kBalancedMaxRounds = 5;
__device__ __forceinline__ int chunked_item_of_workgroup(int wg)
{
    const unsigned xcd = static_cast<unsigned>(wg) % kXcdCount, slot = static_cast<unsigned>(wg) / kXcdCount;
    return static_cast<int>(((slot / kXcdChunk) * kXcdCount + xcd) * kXcdChunk + slot % kXcdChunk);
}
// Size of XCD `xcd`'s share of n items of one kind; `begin` receives its first item.
__device__ __forceinline__ int xcd_share(int n, int xcd, int& rot, int& begin)
{
    const int b = static_cast<int>(static_cast<unsigned>(n) / kXcdCount), r = static_cast<int>(static_cast<unsigned>(n) % kXcdCount);
    const int xr = (xcd - rot) & (kXcdCount - 1);
    begin = xr * b + min(xr, r);
    rot = (rot + r) & (kXcdCount - 1);
    return b + (xr < r ? 1 : 0);
}

// Per-expert tile counts (lane e = expert e) and their running sums; the same in every workgroup.
//
// "Tall" tiles.  A remainder of r <= MT/2 rows costs far more as tail tiles than its share of the work:
// a tail tile does a quarter of the MFMA work of a full tile but loads the same weight panel, pays
// the same tile start-up, and takes half as long as a full tile.  When the launch runs at least
// kTallMinRounds rounds of full tiles (every compute unit gets several tiles, so one longer tile
// does not decide the end of the launch), the remainder is instead folded into the expert's last full
// tiles: ceil(r/64) of them become MT + 64 rows tall (same weight panel, same start-up, same K loop
// with one more 32-row MFMA tile per wavefront).  Tall tiles are numbered first: longest work first.
constexpr int kTallMinRounds = 2;
struct TileSchedule {
    int lo, hi;              // this lane's expert: clamped row range
    int full_rt, tail_rt;    //   its full and tail row tiles
    int tall_rt;             //   its tall row tiles (they follow the full ones in the row order)
    int full_incl, tail_incl, tall_incl;
    int total_full, total_tail, total_tall;
    int split;               // K slices per tail tile
};

__device__ __forceinline__ TileSchedule scan_experts(const int32_t* __restrict__ offsets, int E_local, int mt, int n_tiles,
                                                     int max_rows, int nk, bool may_split, bool allow_tall,
                                                     const RowMap* probe = nullptr)
{
    TileSchedule sc;
    const int lane = lane_id();
    sc.lo = 0;
    sc.hi = 0;
    if (lane < E_local) {  // clamped so that a corrupt offsets array can never index past the buffers
        sc.lo = min(max(offsets[lane], 0), max_rows);
        sc.hi = min(max(offsets[lane + 1], sc.lo), max_rows);
    }
    const int cnt = sc.hi - sc.lo;
    if (probe != nullptr && probe->timeline != nullptr) {  // measurement only: when did the row ranges arrive?
        if (__ballot(cnt >= 0) != 0ull) timeline_stamp(*probe, 7);
    }
    const int q = cnt / mt;
    const int need = (cnt - q * mt + kTailRows - 1) / kTailRows;  // 64-row blocks of the remainder
    bool use_tall = false;
    if (allow_tall)  // rounds of the launch, counted in row tiles of mt rows (a ragged last one included)
        use_tall = wave_read_lane(wave_inclusive_scan((cnt + mt - 1) / mt * n_tiles), kWave - 1) >= kTallMinRounds * kSplitUnits;
    sc.tall_rt = (use_tall && need > 0 && need <= max_tail_tiles(mt) && need <= q) ? need : 0;
    sc.full_rt = q - sc.tall_rt;
    sc.tail_rt = sc.tall_rt > 0 ? 0 : need;
    if (sc.tail_rt > max_tail_tiles(mt)) {
        sc.full_rt += 1;
        sc.tail_rt = 0;
    }
    sc.full_incl = wave_inclusive_scan(sc.full_rt * n_tiles);
    sc.tail_incl = wave_inclusive_scan(sc.tail_rt * n_tiles);
    sc.total_full = wave_read_lane(sc.full_incl, kWave - 1);
    sc.total_tail = wave_read_lane(sc.tail_incl, kWave - 1);
    sc.tall_incl = 0;
    sc.total_tall = 0;
    if (use_tall) {
        sc.tall_incl = wave_inclusive_scan(sc.tall_rt * n_tiles);
        sc.total_tall = wave_read_lane(sc.tall_incl, kWave - 1);
    }
    int split = 1;
    if (may_split && sc.total_tail > 0) {  // the largest s <= kSplitMax with s * total_tail <= kSplitUnits and s * kSplitMinKTiles <= nk
#pragma unroll
        for (int c = 2; c <= kSplitMax; ++c)
            if (c * sc.total_tail <= kSplitUnits && c * kSplitMinKTiles <= nk) split = c;
    }
    sc.split = __builtin_amdgcn_readfirstlane(split);
    return sc;
}

// Quotient of two wavefront-uniform non-negative numbers.  A division by a run-time value costs a
// reciprocal sequence of some twenty dependent instructions, and the lookup ran ten of them per tile;
// the divisors here are powers of two in the common shapes (column tiles per row, rows left over).
__device__ __forceinline__ unsigned uniform_udiv(unsigned a, unsigned d)
{
    if ((d & (d - 1u)) == 0u) return a >> (31 - __builtin_clz(d | 1u));  // d = 2^k (d = 0 never occurs)
    return a / d;
}
// a / d for 1 <= d <= 8 and a < 8192: multiplication by ceil(2^16 / d), exact in that range.
__device__ __forceinline__ unsigned udiv_small(unsigned a, unsigned d)
{
    const unsigned long long lo = (32768ull << 16) | (21846ull << 32) | (16384ull << 48);              // d = 2..4 (d = 1 is handled apart)
    const unsigned long long hi = 13108ull | (10923ull << 16) | (9363ull << 32) | (8192ull << 48);     // d = 5..8
    if (d <= 1u) return a;
    const unsigned recip = static_cast<unsigned>(((d <= 4u ? lo : hi) >> (16u * ((d - 1u) & 3u))) & 0xffffull);
    return (a * recip) >> 16;
}

// Tile j of one kind (kTileFull, kTileTail, kTileTall) -> expert, rows, column tile.
enum TileKind { kTileFull = 0, kTileTail = 1, kTileTall = 2 };
__device__ __forceinline__ bool decode_tile(const TileSchedule& sc, int E_local, int mt, int n_tiles, int kind, int j, Tile2D& out)
{
    const int lane = lane_id();
    const bool tail = kind == kTileTail, tall = kind == kTileTall;
    const int incl = tail ? sc.tail_incl : (tall ? sc.tall_incl : sc.full_incl);
    const int rt = tail ? sc.tail_rt : (tall ? sc.tall_rt : sc.full_rt);
    const int excl = incl - rt * n_tiles;
    const unsigned long long m = __ballot(lane < E_local && j >= excl && j < incl);
    if (m == 0ull) return false;
    const int src = __ffsll(static_cast<long long>(m)) - 1;
    const int e_lo = wave_read_lane(sc.lo, src);
    const int e_hi = wave_read_lane(sc.hi, src);
    const int e_rt = wave_read_lane(rt, src);
    const int e_full = wave_read_lane(sc.full_rt, src);
    const int r = j - wave_read_lane(excl, src);
    // Order of the expert's tiles.  With many row tiles, consecutive tiles form blocks of kBlockRows
    // row tiles x kBlockCols column tiles (one XCD chunk): the 32 workgroups of a block share 4
    // activation and 8 weight panels in their L2, against 16 and 2 when the rows of a column simply
    // follow each other.  Remaining row tiles (and small experts) run row tile fastest.
    constexpr int kBlockRows = 4, kBlockCols = kXcdChunk / kBlockRows;
    int row_tile, col_tile;
    const int blocked_rows = (kind == kTileFull && (n_tiles & (kBlockCols - 1)) == 0) ? (e_rt & ~(kBlockRows - 1)) : 0;
    if (r < blocked_rows * n_tiles) {
        const unsigned per_row_block = static_cast<unsigned>(kBlockRows * n_tiles);
        const unsigned rbk = uniform_udiv(static_cast<unsigned>(r), per_row_block), in_rb = static_cast<unsigned>(r) - rbk * per_row_block;
        const unsigned cb = in_rb / (kBlockRows * kBlockCols), in_b = in_rb % (kBlockRows * kBlockCols);
        col_tile = static_cast<int>(cb * kBlockCols + in_b / kBlockRows);
        row_tile = static_cast<int>(rbk * kBlockRows + in_b % kBlockRows);
    } else {
        const unsigned rr = static_cast<unsigned>(r - blocked_rows * n_tiles), rows_left = static_cast<unsigned>(e_rt - blocked_rows);
        const unsigned c = uniform_udiv(rr, rows_left);
        col_tile = static_cast<int>(c);
        row_tile = blocked_rows + static_cast<int>(rr - c * rows_left);
    }
    // rows of an expert: its full tiles, then its tall tiles (or its tail tiles)
    const int begin = tail ? e_lo + e_full * mt + row_tile * kTailRows
                           : (tall ? e_lo + e_full * mt + row_tile * (mt + kTailRows) : e_lo + row_tile * mt);
    const int height = tail ? kTailRows : (tall ? mt + kTailRows : mt);
    // every lane holds the same values; readfirstlane tells the compiler so (scalar registers)
    out.expert = __builtin_amdgcn_readfirstlane(src);
    out.n_tile = __builtin_amdgcn_readfirstlane(col_tile);
    out.row_begin = __builtin_amdgcn_readfirstlane(begin);
    out.row_end = __builtin_amdgcn_readfirstlane(min(begin + height, e_hi));
    out.hid_shift = __builtin_amdgcn_readfirstlane(kHiddenRowBlock * src - (e_lo & (kHiddenRowBlock - 1)));
    out.tail = tail;
    out.tall = tall;
    return true;
}

// Work item of workgroup `wg`.  Order of the list (of every XCD's queue, when balanced): the tall
// tiles (longest work first); then - few tail items (at most one per compute unit, K slices counted) -
// the tail items, slice fastest, so that the launch ends with whole rounds of full tiles (behind the
// full tiles the few compute units that get a tail tile at the very end would decide when the launch
// is over); then the full tiles; many tail items go last instead and fill the ragged end of the last round.
__device__ __forceinline__ bool locate_tile(const int32_t* __restrict__ offsets, int E_local, int mt, int n_tiles, int max_rows,
                                            int nk, bool may_split, bool allow_tall, int wg, Tile2D& out,
                                            const RowMap* probe = nullptr)
{
    const TileSchedule sc = scan_experts(offsets, E_local, mt, n_tiles, max_rows, nk, may_split, allow_tall, probe);
    out.kt_begin = 0;
    out.kt_end = nk;
    out.slot = -1;
    const int tail_units = sc.total_tail * sc.split;
    const bool tails_first = tail_units <= kSplitUnits;
    const int total = sc.total_tall + sc.total_full + tail_units;
    const int xcd = static_cast<int>(static_cast<unsigned>(wg) % kXcdCount);
    const int kinds = (sc.total_tall > 0 ? 1 : 0) + (sc.total_full > 0 ? 1 : 0) + (tail_units > 0 ? 1 : 0);
    const bool balanced = total <= kBalancedMaxRounds * kSplitUnits || kinds <= 1;
    int pos = balanced ? static_cast<int>(static_cast<unsigned>(wg) / kXcdCount) : chunked_item_of_workgroup(wg);  // in the XCD's queue / in the list
    if (!balanced && pos >= total) return false;
    int rot = 0, begin = 0;
#pragma unroll
    for (int c = 0; c < 3; ++c) {
        const int kind = c == 0 ? kTileTall : ((tails_first ? c == 1 : c == 2) ? kTileTail : kTileFull);
        const int n = kind == kTileTall ? sc.total_tall : (kind == kTileTail ? tail_units : sc.total_full);
        const int share = balanced ? xcd_share(n, xcd, rot, begin) : n;
        if (pos < share) {
            const int u = begin + pos;
            // (K slices exist only while tail_units <= kSplitUnits, the range udiv_small is exact in)
            const int tail_tile = sc.split > 1 ? static_cast<int>(udiv_small(static_cast<unsigned>(u), static_cast<unsigned>(sc.split))) : u;
            if (!decode_tile(sc, E_local, mt, n_tiles, kind, kind == kTileTail ? tail_tile : u, out)) return false;
            if (kind == kTileTail && sc.split > 1) {
                const int slice = u - tail_tile * sc.split;
                out.kt_begin = __builtin_amdgcn_readfirstlane(slice * nk / sc.split);
                out.kt_end = __builtin_amdgcn_readfirstlane((slice + 1) * nk / sc.split);
                out.slot = __builtin_amdgcn_readfirstlane(u);
            }
            return true;
        }
        pos -= share;
    }
    return false;
}

// ---------------------------------------------------------------------------- bf16 MFMA kernel
// XOR swizzle of the 16-byte chunk index inside a tile row, chosen so that the lanes of one
// ds_read_b128 (consecutive rows, same logical chunk) fall on distinct banks.
//   SWZ 0: 128-byte rows -> row & 7;        64-byte rows -> (row >> 1) & 3
//   SWZ 1: 128-byte rows -> (row >> 1) & 7  (16 consecutive rows distinct over 64 banks)
template <int KT, int SWZ>
__device__ __forceinline__ int chunk_swizzle(int row)
{
    if constexpr (KT == 64) return SWZ == 1 ? ((row >> 1) & 7) : (row & 7);
    return (row >> 1) & 3;
}

// A pointer that is the same in every lane, moved to scalar registers.
__device__ __forceinline__ const unsigned char* uniform_ptr(const unsigned char* p)
{
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v));
    const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v >> 32));
    return reinterpret_cast<const unsigned char*>((static_cast<uint64_t>(hi) << 32) | lo);
}

// One wavefront-wide direct-to-LDS load: lane i fetches 16 bytes at base + voff and they land at
// LDS byte address lds_addr + 16*i (M0 carries the wavefront-uniform LDS address).  Issued as
// inline assembly on purpose: the compiler then keeps exact lgkmcnt waits for the ds_read
// operand fetches, and the landing of these loads is awaited explicitly with wait_vmcnt.
__device__ __forceinline__ void lds_dma_16B(const unsigned char* base, uint32_t voff, uint32_t lds_addr)
{
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1\n" : : "v"(voff), "s"(base), "s"(lds_addr) : "memory");
#else
    (void)base; (void)voff; (void)lds_addr;
#endif
}

// One wavefront-wide direct-to-LDS load of 4 bytes per lane: lane i fetches base + voff and the word
// lands at LDS byte address lds_addr + 4*i.
__device__ __forceinline__ void lds_dma_4B(const unsigned char* base, uint32_t voff, uint32_t lds_addr)
{
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1\n" : : "v"(voff), "s"(base), "s"(lds_addr) : "memory");
#else
    (void)base; (void)voff; (void)lds_addr;
#endif
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
#endif
}

// One output tile: rows [row_begin,row_end) (at most MT) x columns [n0, n0+NT) of expert weights wexp,
// summed over K tiles [kt_begin, kt_end).  With `partial` set (SPLIT instantiations only) the fp32
// sums are written there, in the order partial_index() gives, and no epilogue runs.
template <int TN, int TM>
__device__ __forceinline__ int partial_index(int wave, int a, int b, int g, int lane)
{
    return ((((wave * TN + a) * TM + b) * 4 + g) * kWave) + lane;  // in units of float4: a store covers 1 KiB
}

template <int MT, int NT, int KT, int STAGES, int WM, int WN, int SWZ, int EPI, bool BIAS, bool SPLIT>
__device__ __forceinline__ void gemm_tile(const bf16_t* __restrict__ act, const bf16_t* __restrict__ wexp,
                                          const bf16_t* __restrict__ bias_e, int row_begin, int row_end, int n0, int K, int N,
                                          bf16_t* __restrict__ out, unsigned char* smem, const RowMap& map, int kt_begin,
                                          int kt_end, float4* __restrict__ partial, int ids_off = -1, int hid_shift = 0)
{
    constexpr int NWAVES = WM * WN;
    constexpr int RB = KT * 2;              // bytes per tile row
    constexpr int CPR = RB / 16;            // 16-byte chunks per tile row
    constexpr int RPI = 1024 / RB;          // tile rows covered by one wavefront-wide direct-to-LDS load
    constexpr int LPW = (MT + NT) / RPI / NWAVES;  // direct-to-LDS load instructions per K tile and wavefront
    constexpr int STAGE_BYTES = (MT + NT) * RB;
    constexpr int WTM = MT / WM, WTN = NT / WN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int KSTEPS = KT / 16;
    static_assert(KT == 32 || KT == 64, "row swizzle is written for 64- and 128-byte tile rows");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wavefront tile is made of 32x32 MFMA tiles");
    static_assert((STAGES - 1) * LPW < 64, "outstanding loads must fit the vmcnt counter");

    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int wm = wave / WN, wn = wave % WN;

    // ---- per-lane sources of this wavefront's direct-to-LDS loads ---------------------------
    // A stage holds MT activation rows followed by NT weight rows.  One wavefront-wide load
    // covers RPI consecutive rows (1 KiB of LDS): lane -> row lane/CPR of the group and the
    // 16-byte chunk (lane%CPR) ^ swizzle(row); it lands at LDS byte group*1024 + lane*16.
    // Every wavefront owns LA activation groups and LW weight groups; sources are kept as 32-bit
    // byte offsets from the two (uniform) base pointers.
    constexpr int LA = MT / RPI / NWAVES, LW = NT / RPI / NWAVES;
    static_assert(LA * RPI * NWAVES == MT && LW * RPI * NWAVES == NT, "tile rows must split evenly over the wavefronts");
    // Gathered activation rows need their row ids first - a dependent load in front of the tile's
    // first loads.  With a two-stage ring and a scratch area behind it (ids_off >= 0) the ids are
    // fetched straight into LDS, the weight loads of both stages are issued behind them, and the ids
    // are read back once only the weight loads are outstanding: ids and weights travel together.
    // (Through a register the id load would be awaited with vmcnt(0), i.e. together with the weights.)
    const bool ids_via_lds = STAGES == 2 && map.a_row != nullptr && ids_off >= 0;
    uint32_t off_a[LA], off_w[LW];
    auto set_off_a = [&](bool from_lds) {
#pragma unroll
        for (int i = 0; i < LA; ++i) {
            const int row = (wave * LA + i) * RPI + lane / CPR;
            const int chunk = (lane % CPR) ^ chunk_swizzle<KT, SWZ>(row);
            int r = min(row_begin + row, row_end - 1);  // rows past the tile end re-read the last valid row
            if (from_lds) r = *reinterpret_cast<const int*>(smem + ids_off + (wave * LA + i) * 256 + lane * 4) / map.a_div;
            else if (map.a_row != nullptr) r = map.a_row[r] / map.a_div;
            if (map.hidden_act != 0) {
                // (never gathered)  Consecutive lanes take consecutive ROWS of one piece - consecutive 16-byte
                // words of the hidden layout, which the memory pipeline merges into whole lines; the 1 KiB LDS
                // group of this load then holds [piece][row] instead of [row][piece] (see frag_off_a).
                const int row_t = (wave * LA + i) * RPI + lane % RPI;
                const uint32_t h = static_cast<uint32_t>(min(row_begin + row_t, row_end - 1) + hid_shift);
                // (odd groups hold their pieces pairwise exchanged: two groups that are read together then sit in different banks)
                off_a[i] = static_cast<uint32_t>(hidden_offset(h, static_cast<uint32_t>((lane / RPI) ^ ((wave * LA + i) & 1)), static_cast<uint32_t>(K) / 8u));
            } else {
                off_a[i] = (static_cast<uint32_t>(r) * static_cast<uint32_t>(K) + chunk * 8) * 2u;
            }
        }
    };
    if (!ids_via_lds) set_off_a(false);
#pragma unroll
    for (int i = 0; i < LW; ++i) {
        const int row = (wave * LW + i) * RPI + lane / CPR;
        const int chunk = (lane % CPR) ^ chunk_swizzle<KT, SWZ>(MT + row);
        const int r = min(n0 + row, N - 1);
        off_w[i] = (static_cast<uint32_t>(r) * static_cast<uint32_t>(K) + chunk * 8) * 2u;
    }
    const size_t k_skip = static_cast<size_t>(kt_begin) * (KT * 2);  // bytes of a row in front of this K range
    // bytes from one K tile of the activation operand to the next: KT columns of a row, or KT/8 pieces of a 32-row block
    const size_t a_kstride = map.hidden_act != 0 ? static_cast<size_t>(KT / 8) * kHiddenPieceStride : static_cast<size_t>(KT * 2);
    const unsigned char* act_b = uniform_ptr(reinterpret_cast<const unsigned char*>(act) + static_cast<size_t>(kt_begin) * a_kstride);
    const unsigned char* wgt_b = uniform_ptr(reinterpret_cast<const unsigned char*>(wexp) + k_skip);

    // ---- per-lane LDS byte offsets of the MFMA operand reads -------------------------------
    // operand row = base + lane%32; K step ks uses logical chunk 2*ks + lane/32
    int frag_off[KSTEPS];
    {
        const int row = lane & 31;
        const int swz = chunk_swizzle<KT, SWZ>(row);
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) frag_off[ks] = row * RB + (((2 * ks + (lane >> 5)) ^ swz) * 16);
    }
    // activation operand from the hidden layout: LDS groups hold [piece][row] (no swizzle needed: the 8 lanes
    // served together read 8 consecutive rows of one piece = 128 contiguous bytes)
    int frag_off_a[KSTEPS];
    {
        const int row = lane & 31;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks)
            frag_off_a[ks] = map.hidden_act != 0
                                 ? (row / RPI) * 1024 + ((2 * ks + (lane >> 5)) ^ ((row / RPI) & 1)) * (RPI * 16) + (row % RPI) * 16
                                 : frag_off[ks];
    }
    const int act_base = (wm * WTM) * RB;            // activation rows of this wavefront inside a stage
    const int wgt_base = (MT + wn * WTN) * RB;       // weight rows of this wavefront inside a stage

    f32x16_t acc[TN][TM];
#pragma unroll
    for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    const int nk = kt_end - kt_begin;
    const uint32_t smem_addr = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
        (__attribute__((address_space(3))) unsigned char*)smem));  // LDS byte address of the ring
    auto issue = [&](int kt) {
        const uint32_t stage = smem_addr + (kt % STAGES) * STAGE_BYTES;
        const size_t kbyte = static_cast<size_t>(kt) * (KT * 2);
#pragma unroll
        for (int i = 0; i < LA; ++i) lds_dma_16B(act_b + static_cast<size_t>(kt) * a_kstride, off_a[i], stage + (wave * LA + i) * 1024);
#pragma unroll
        for (int i = 0; i < LW; ++i) lds_dma_16B(wgt_b + kbyte, off_w[i], stage + MT * RB + (wave * LW + i) * 1024);
    };

    // one of the LPW loads of K tile kt (i < LA: activation group, else weight group)
    auto issue_one = [&](int kt, int i) {
        const uint32_t stage = smem_addr + (kt % STAGES) * STAGE_BYTES;
        const size_t kbyte = static_cast<size_t>(kt) * (KT * 2);
        if (i < LA) lds_dma_16B(act_b + static_cast<size_t>(kt) * a_kstride, off_a[i < LA ? i : 0], stage + (wave * LA + i) * 1024);
        else lds_dma_16B(wgt_b + kbyte, off_w[i >= LA ? i - LA : 0], stage + MT * RB + (wave * LW + (i - LA)) * 1024);
    };

    // ---- main loop ---------------------------------------------------------------------------------
    // One software pipeline over all K steps of the tile.  MFMA operands are double-buffered in
    // registers and fetched one K step ahead, also across K tiles.  The barrier that hands over K
    // tile kt+1 (everyone's share of it has landed; everyone is done reading tile kt) sits in the
    // MIDDLE of the last K step of tile kt: the MFMAs issued just before it keep the matrix cores
    // busy while the wavefronts meet, the MFMAs after it cover the latency of the first operand
    // fetches from the new K tile.  At the barrier the stage of tile kt is free, so tile kt+STAGES
    // is requested at once: all STAGES stages are in flight.  The issue order is hand-placed (the
    // scheduling barriers pin it): slot m of a K step is MFMA m, operand fetches sit in front of
    // slots, and the (slow to issue) direct-to-LDS loads go one at a time behind the slots that
    // follow a hand-over.
    static_assert(KSTEPS % 2 == 0, "register double-buffering assumes an even number of K steps per K tile");
    if (ids_via_lds) {
        if constexpr (STAGES == 2) {
            const int n_first = min(nk, 2);
            const unsigned char* ids_b = uniform_ptr(reinterpret_cast<const unsigned char*>(map.a_row));
#pragma unroll
            for (int i = 0; i < LA; ++i) {
                const int row = (wave * LA + i) * RPI + lane / CPR;
                lds_dma_4B(ids_b, static_cast<uint32_t>(min(row_begin + row, row_end - 1)) * 4u,
                           smem_addr + static_cast<uint32_t>(ids_off) + (wave * LA + i) * 256);
            }
            for (int s = 0; s < n_first; ++s) {
                const uint32_t stage = smem_addr + s * STAGE_BYTES;
#pragma unroll
                for (int i = 0; i < LW; ++i)
                    lds_dma_16B(wgt_b + static_cast<size_t>(s) * (KT * 2), off_w[i], stage + MT * RB + (wave * LW + i) * 1024);
            }
            if (n_first == 2) wait_vmcnt<2 * LW>();  // loads land in order: the ids are in LDS
            else wait_vmcnt<LW>();
            set_off_a(true);
            for (int s = 0; s < n_first; ++s) {
                const uint32_t stage = smem_addr + s * STAGE_BYTES;
#pragma unroll
                for (int i = 0; i < LA; ++i)
                    lds_dma_16B(act_b + static_cast<size_t>(s) * a_kstride, off_a[i], stage + (wave * LA + i) * 1024);
            }
            if (n_first == 2) wait_vmcnt<LA>();  // K tile 0 complete; the activation rows of K tile 1 may be in flight
            else wait_vmcnt<0>();
        }
    } else {
#pragma unroll
    for (int s = 0; s < STAGES; ++s)
        if (s < nk) issue(s);
    }
    if (!ids_via_lds) {
        const int younger = min(nk, STAGES) - 1;
        static_assert(STAGES >= 2 && STAGES <= 8 && (STAGES - 1) * LPW < 64, "pipeline depth against the 6-bit vmcnt");
        if (STAGES >= 8 && younger >= 7) wait_vmcnt<(STAGES >= 8 ? 7 : 0) * LPW>();
        else if (STAGES >= 7 && younger >= 6) wait_vmcnt<(STAGES >= 7 ? 6 : 0) * LPW>();
        else if (STAGES >= 6 && younger >= 5) wait_vmcnt<(STAGES >= 6 ? 5 : 0) * LPW>();
        else if (STAGES >= 5 && younger >= 4) wait_vmcnt<(STAGES >= 5 ? 4 : 0) * LPW>();
        else if (STAGES >= 4 && younger >= 3) wait_vmcnt<(STAGES >= 4 ? 3 : 0) * LPW>();
        else if (STAGES >= 3 && younger >= 2) wait_vmcnt<(STAGES >= 3 ? 2 : 0) * LPW>();
        else if (younger >= 1) wait_vmcnt<LPW>();
        else wait_vmcnt<0>();
    }
    __syncthreads();
    timeline_stamp(map, 2);
    // Operand register ring: FD K steps deep (fetches run FD-1 K steps ahead of the MFMAs).  Two is
    // enough when a K step holds many MFMAs; a wavefront tile of one or two MFMAs per K step (the
    // remainder tiles) takes four, or every K step would expose a full LDS round trip.
    constexpr int kFragDepthSmall = 4;  // (2 measured slower on remainder tiles)
    constexpr int SLOTS = TN * TM;
    constexpr int FD = (SLOTS <= 2 && KSTEPS % kFragDepthSmall == 0) ? kFragDepthSmall : 2;
    static_assert(KSTEPS % FD == 0, "the ring index of a K step must not depend on the K tile");
    bf16x8_t fa[FD][TN], fb[FD][TM];
    auto fetch = [&](const unsigned char* stage, int ks, int r) {  // operand r of K step ks from a stage
        if (r < TN) fa[ks % FD][r] = *reinterpret_cast<const bf16x8_t*>(stage + wgt_base + r * 32 * RB + frag_off[ks]);
        else fb[ks % FD][r - TN] = *reinterpret_cast<const bf16x8_t*>(stage + act_base + (r - TN) * 32 * RB + frag_off_a[ks]);
    };
    constexpr int NFRAG = TN + TM;
#pragma unroll
    for (int ks = 0; ks < FD - 1; ++ks)
#pragma unroll
        for (int r = 0; r < NFRAG; ++r) fetch(smem, ks, r);
    constexpr int HALF = SLOTS / 2;                                     // MFMAs of the last K step in front of the hand-over
    constexpr int READ_GAP = SLOTS / NFRAG > 0 ? SLOTS / NFRAG : 1;     // inside a K tile: one fetch every READ_GAP slots
    constexpr int READS_PER_SLOT = (NFRAG + SLOTS - 1) / SLOTS;
    constexpr int NFRAG_HAND = (FD - 1) * NFRAG;                        // fetches behind a hand-over: K steps 0..FD-2 of the new tile
    constexpr int READS_PER_SLOT_LAST = (NFRAG_HAND + (SLOTS - HALF) - 1) / (SLOTS - HALF);
    constexpr int LOAD_SLOTS = (KSTEPS >= 4 ? 2 : 1) * SLOTS;            // slots over which a K tile's loads are spread
    static_assert(LOAD_SLOTS <= KSTEPS * SLOTS, "a K tile's loads must all be issued before the next hand-over");
    for (int kt = 0; kt < nk; ++kt) {
        const unsigned char* stage_cur = smem + (kt % STAGES) * STAGE_BYTES;
        const unsigned char* stage_nxt = smem + ((kt + 1) % STAGES) * STAGE_BYTES;
        const bool more = kt + 1 < nk;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            const int cur = ks % FD;
            const bool last = ks == KSTEPS - 1;
#pragma unroll
            for (int m = 0; m < SLOTS; ++m) {
                if (last && m == HALF) {
                    if (more) {  // my share of K tile kt+1 has landed; younger tiles may still be in flight
                        const int younger = min(nk - 1, kt + STAGES - 1) - (kt + 1);
                        if (STAGES >= 8 && younger >= 6) wait_vmcnt<(STAGES >= 8 ? 6 : 0) * LPW>();
                        else if (STAGES >= 7 && younger >= 5) wait_vmcnt<(STAGES >= 7 ? 5 : 0) * LPW>();
                        else if (STAGES >= 6 && younger >= 4) wait_vmcnt<(STAGES >= 6 ? 4 : 0) * LPW>();
                        else if (STAGES >= 5 && younger >= 3) wait_vmcnt<(STAGES >= 5 ? 3 : 0) * LPW>();
                        else if (STAGES >= 4 && younger >= 2) wait_vmcnt<(STAGES >= 4 ? 2 : 0) * LPW>();
                        else if (STAGES >= 3 && younger >= 1) wait_vmcnt<(STAGES >= 3 ? 1 : 0) * LPW>();
                        else wait_vmcnt<0>();
                    }
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // my operand fetches from tile kt are complete
                    __syncthreads();
                }
                // operand fetches: K step ks+FD-1 of this tile, or (behind the hand-over) the first
                // FD-1 K steps of the next tile
                if (ks + FD - 1 < KSTEPS) {
                    if (m % READ_GAP == 0) {
#pragma unroll
                        for (int q = 0; q < READS_PER_SLOT; ++q) {
                            const int r = (m / READ_GAP) * READS_PER_SLOT + q;
                            if (r < NFRAG) fetch(stage_cur, ks + FD - 1 < KSTEPS ? ks + FD - 1 : 0, r);
                        }
                    }
                }
                if (last && m >= HALF && more) {
#pragma unroll
                    for (int q = 0; q < READS_PER_SLOT_LAST; ++q) {
                        const int i = (m - HALF) * READS_PER_SLOT_LAST + q;
                        if (i < NFRAG_HAND) fetch(stage_nxt, i / NFRAG, i % NFRAG);
                    }
                }
                acc[m / TM][m % TM] =
                    __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][m / TM], fb[cur][m % TM], acc[m / TM][m % TM], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                {
                    // slot position since the latest hand-over, and the K tile refilled there
                    const bool after = last && m >= HALF;
                    const int p = after ? m - HALF : (SLOTS - HALF) + ks * SLOTS + m;
                    const int load_tile = after ? kt + STAGES : kt - 1 + STAGES;
                    if (p < LOAD_SLOTS) {
                        const bool do_load = load_tile < nk && (after || kt >= 1);
#pragma unroll
                        for (int i = 0; i < LPW; ++i)
                            if (i * LOAD_SLOTS / LPW == p && do_load) issue_one(load_tile, i);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
        }
    }
    timeline_stamp(map, 3);
    if constexpr (SPLIT) {
        if (partial != nullptr) {  // a K slice: hand the raw sums to the kernel that adds the slices
#pragma unroll
            for (int a = 0; a < TN; ++a)
#pragma unroll
                for (int b = 0; b < TM; ++b)
#pragma unroll
                    for (int g = 0; g < 4; ++g)
                        partial[partial_index<TN, TM>(wave, a, b, g, lane)] =
                            make_float4(acc[a][b][g * 4 + 0], acc[a][b][g * 4 + 1], acc[a][b][g * 4 + 2], acc[a][b][g * 4 + 3]);
            return;
        }
    }
    // ---- epilogue -----------------------------------------------------------------------------
    // A lane holds, for output row m = .. + lane%32, the columns n = .. + 8*g + 4*(lane/32) + r.
    // Writing that straight to memory would touch 32 rows per store instruction, so every
    // wavefront transposes its tile through its own slice of the (now idle) LDS ring, 64 rows at a
    // time, and stores whole 16-byte chunks of contiguous row segments.
    constexpr int BP = (TM >= 2 && TM % 2 == 0) ? 2 : 1;  // 32-row MFMA tiles per pass
    constexpr int ROW_BYTES = WTN * 2;
    constexpr int S = ROW_BYTES + 8;               // padded LDS row stride: conflict-free 8-byte writes
    constexpr int REGION = BP * 32 * S;
    constexpr int CW = ROW_BYTES / 16;             // 16-byte chunks per row segment
    constexpr int RPI_OUT = 64 / CW;               // rows covered by one wavefront-wide 16-byte access
    static_assert(NWAVES * REGION <= STAGES * STAGE_BYTES, "epilogue staging must fit in the LDS ring");
    static_assert(64 % CW == 0 && (BP * 32) % RPI_OUT == 0, "row segments must tile the wavefront");
    // (no barrier here: behind the last hand-over nobody reads the LDS ring any more)
    unsigned char* region = smem + wave * REGION;
    const int n_wave = n0 + wn * WTN;
    // bias of the 4 columns a lane owns in every (a, g) group; the same for all of its rows
    float bias_v[TN][4][4];
    if constexpr (BIAS) {
        const bf16_t* bexp = bias_e;
#pragma unroll
        for (int a = 0; a < TN; ++a)
#pragma unroll
            for (int g = 0; g < 4; ++g)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    bias_v[a][g][r] = bf16_to_f32(bexp[min(n_wave + a * 32 + g * 8 + (lane >> 5) * 4 + r, N - 1)]);
    }
    if (map.hidden_out != 0) {
        // hidden layout: no transposition.  For a pair of column groups (g, g+1) the lower half of the
        // wavefront gives its 4 columns of group g+1 to the upper half and receives the upper half's 4
        // columns of group g: every lane then holds 8 consecutive columns of its row = one 16-byte piece,
        // the lower half of group g, the upper half of group g+1 - 1 KiB contiguous per store.
        const uint32_t pieces = static_cast<uint32_t>(N) / 8u;
#pragma unroll
        for (int b = 0; b < TM; ++b) {
            const int m = row_begin + wm * WTM + b * 32 + (lane & 31);
            const uint32_t h = static_cast<uint32_t>(m + hid_shift);
            unsigned char* row_base = reinterpret_cast<unsigned char*>(out) + hidden_offset(h, 0u, pieces);
#pragma unroll
            for (int a = 0; a < TN; ++a) {
#pragma unroll
                for (int gp = 0; gp < 2; ++gp) {
                    uint32_t w[2][2];
#pragma unroll
                    for (int q = 0; q < 2; ++q) {
                        const int g = 2 * gp + q;
                        float v[4];
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            float z = acc[a][b][g * 4 + r];
                            if constexpr (BIAS) z += bias_v[a][g][r];
                            if constexpr (EPI == kEpiGeluErf) z = gelu_erf_fast(z);
                            if constexpr (EPI == kEpiGeluTanh) z = gelu_tanh_fast(z);
                            v[r] = z;
                        }
                        w[q][0] = pack_bf16x2(v[0], v[1]);
                        w[q][1] = pack_bf16x2(v[2], v[3]);
                    }
                    // w[0] lanes 32..63 <-> w[1] lanes 0..31
                    const auto s0 = __builtin_amdgcn_permlane32_swap(w[0][0], w[1][0], false, false);
                    const auto s1 = __builtin_amdgcn_permlane32_swap(w[0][1], w[1][1], false, false);
                    const uint4 val = make_uint4(s0[0], s1[0], s0[1], s1[1]);
                    const int n = n_wave + a * 32 + gp * 16 + (lane >> 5) * 8;
                    if (m < row_end && n < N)
                        store_stream16(reinterpret_cast<uint4*>(row_base + static_cast<size_t>(n / 8) * kHiddenPieceStride), val);
                }
            }
        }
        return;
    }
    constexpr int NIT = BP * 32 / RPI_OUT;          // store instructions per pass
    const bool scatter = EPI == kEpiNone && map.out_row != nullptr;
#pragma unroll
    for (int pass = 0; pass < TM / BP; ++pass) {
        const int m_pass = row_begin + wm * WTM + pass * BP * 32;
        // scattered output: target rows of this lane's stores and gate weights of this lane's values
        int dst[NIT];
        float scale[BP];
#pragma unroll
        for (int it = 0; it < NIT; ++it) dst[it] = m_pass + it * RPI_OUT + lane / CW;
#pragma unroll
        for (int bl = 0; bl < BP; ++bl) scale[bl] = 1.0f;
        if constexpr (EPI == kEpiNone) {
            if (scatter) {
#pragma unroll
                for (int it = 0; it < NIT; ++it) dst[it] = map.out_row[min(dst[it], row_end - 1)];
#pragma unroll
                for (int bl = 0; bl < BP; ++bl)
                    scale[bl] = map.out_scale[map.out_row[min(m_pass + bl * 32 + (lane & 31), row_end - 1)]];
            }
        }
#pragma unroll
        for (int bl = 0; bl < BP; ++bl) {
            const int b = pass * BP + bl;
#pragma unroll
            for (int a = 0; a < TN; ++a) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int col = a * 32 + g * 8 + (lane >> 5) * 4;
                    float v[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        float z = acc[a][b][g * 4 + r];
                        if constexpr (BIAS) z += bias_v[a][g][r];
                        if constexpr (EPI == kEpiGeluErf) z = gelu_erf_fast(z);
                        if constexpr (EPI == kEpiGeluTanh) z = gelu_tanh_fast(z);
                        if constexpr (EPI == kEpiNone) z *= scale[bl];
                        v[r] = z;
                    }
                    uint2 packed;
                    packed.x = pack_bf16x2(v[0], v[1]);
                    packed.y = pack_bf16x2(v[2], v[3]);
                    *reinterpret_cast<uint2*>(region + (bl * 32 + (lane & 31)) * S + col * 2) = packed;
                }
            }
        }
        // same wavefront reads back what it just wrote (LDS operations of a wavefront execute in order)
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int r = it * RPI_OUT + lane / CW;
            const int c = lane % CW;
            const uint4 val = *reinterpret_cast<const uint4*>(region + r * S + c * 16);
            const int m = m_pass + r;
            const int n = n_wave + c * 8;
            // streaming stores: the tile is not read again in this launch, and keeping it out of the
            // write-back cache leaves that cache to the weight panels the neighbouring tiles share
            if (m < row_end && n < N)  // N % 8 == 0: a chunk is entirely inside or outside
                store_stream16(reinterpret_cast<uint4*>(out + static_cast<size_t>(dst[it]) * N + n), val);
        }
    }
}

template <int MT, int NT, int KT, int STAGES, int WM, int WN, int SWZ, int OCC, int EPI, bool BIAS>
__global__ __launch_bounds__(WM* WN * 64, OCC) void grouped_gemm_bf16_kernel(const bf16_t* __restrict__ act,     // [A,K]
                                                                         const int32_t* __restrict__ offsets,
                                                                         const bf16_t* __restrict__ weight,  // [E_local,N,K]
                                                                         const bf16_t* __restrict__ bias,    // [E_local,N] or null
                                                                         int max_rows, int K, int N, int E_local,
                                                                         bf16_t* __restrict__ out,           // [A,N]
                                                                         const RowMap map,
                                                                         float4* __restrict__ partial)       // K-slice sums or null
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    timeline_stamp(map, 0);
    if (map.timeline != nullptr && threadIdx.x == 0 && static_cast<int>(blockIdx.x) < map.timeline_cap)
        map.timeline[static_cast<size_t>(blockIdx.x) * 8 + 4] = 0ull;  // stays zero if this workgroup has no tile
    if (map.unrouted != nullptr) {
        // output rows no sorted row writes (dropped or remote assignments): one wavefront looks at 64
        // rows at a time and clears those it finds, all lanes together
        const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
        const int lane = lane_id();
        const int64_t stride = static_cast<int64_t>(gridDim.x) * (WM * WN) * kWave;
        for (int64_t first = (static_cast<int64_t>(blockIdx.x) * (WM * WN) + wave) * kWave; first < map.n_unrouted; first += stride) {
            const int64_t t = first + lane;
            const int pos = t < map.n_unrouted ? map.unrouted[t] : 0;
            unsigned long long todo = __ballot(pos < 0);
            while (todo != 0) {
                const int b = __builtin_ctzll(todo);
                todo &= todo - 1;
                uint4* row = reinterpret_cast<uint4*>(out + static_cast<size_t>(first + b) * N);
                for (int c = lane; c < N / 8; c += kWave) row[c] = make_uint4(0u, 0u, 0u, 0u);
            }
        }
    }
    Tile2D tile;
    const int n_tiles = (N + NT - 1) / NT;
    constexpr bool TALL = tall_tiles_supported(MT, NT, KT, STAGES, WM);
    constexpr int kIdsOff = row_id_scratch_bytes(MT, NT, KT, STAGES, WM, WM * WN) > 0 ? ring_bytes(MT, NT, KT, STAGES, WM) : -1;
    if (!locate_tile(offsets, E_local, MT, n_tiles, max_rows, K / KT, partial != nullptr && MT > kTailRows, TALL,
                     static_cast<int>(blockIdx.x), tile, &map))
        return;
    timeline_stamp(map, 1);
    if (map.timeline != nullptr && threadIdx.x == 0 && static_cast<int>(blockIdx.x) < map.timeline_cap) {
        unsigned hw = 0, xcc = 0;
#if defined(__HIP_DEVICE_COMPILE__)
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw));
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
#endif
        unsigned long long* rec = map.timeline + static_cast<size_t>(blockIdx.x) * 8;
        rec[5] = static_cast<unsigned long long>(hw) | (static_cast<unsigned long long>(xcc & 0xfu) << 32);
        rec[6] = static_cast<unsigned long long>(tile.tail ? 1 : (tile.tall ? 2 : 0)) | (static_cast<unsigned long long>(tile.expert) << 8) |
                 (static_cast<unsigned long long>(tile.n_tile) << 16) | (static_cast<unsigned long long>(tile.row_end - tile.row_begin) << 32) |
                 (static_cast<unsigned long long>(tile.kt_end - tile.kt_begin) << 48);
    }
    const bf16_t* wexp = weight + static_cast<size_t>(tile.expert) * N * K;
    const bf16_t* bias_e = BIAS ? bias + static_cast<size_t>(tile.expert) * N : nullptr;
    if (tile.tall) {
        if constexpr (TALL)
            gemm_tile<MT + kTailRows, NT, KT, STAGES, WM, WN, SWZ, EPI, BIAS, false>(act, wexp, bias_e, tile.row_begin, tile.row_end,
                                                                                     tile.n_tile * NT, K, N, out, smem, map, 0, K / KT,
                                                                                     nullptr, kIdsOff, tile.hid_shift);
    } else if (!tile.tail || MT <= kTailRows) {
        gemm_tile<MT, NT, KT, STAGES, WM, WN, SWZ, EPI, BIAS, false>(act, wexp, bias_e, tile.row_begin, tile.row_end,
                                                                     tile.n_tile * NT, K, N, out, smem, map, 0, K / KT, nullptr, kIdsOff,
                                                                     tile.hid_shift);
    } else if constexpr (MT > kTailRows) {
        // remainder rows: the wavefronts side by side over the columns, kTailRows rows each (two rows
        // of wavefronts when a column strip would become narrower than one MFMA tile).  A
        // tail stage is smaller than a full one, so the same LDS ring holds a deeper pipeline -
        // which the tail needs, because it has little MFMA work per K tile to hide the loads.
        constexpr int kRing = STAGES * (MT + NT) * KT * 2;
        constexpr int kFit = kRing / ((kTailRows + NT) * KT * 2);
        constexpr int kTailStagesMax = 4;  // (5 and 6, also with the whole 160 KB of LDS, measured slower)
        constexpr int STAGES_T = kFit >= kTailStagesMax ? kTailStagesMax : (kFit >= 2 ? kFit : 2);
        constexpr int WM_T = NT / (WM * WN) >= 32 ? 1 : 2;
        float4* slot = tile.slot >= 0 ? partial + static_cast<size_t>(tile.slot) * (kTailRows * NT / 4) : nullptr;
        gemm_tile<kTailRows, NT, KT, STAGES_T, WM_T, WM * WN / WM_T, SWZ, EPI, BIAS, true>(
            act, wexp, bias_e, tile.row_begin, tile.row_end, tile.n_tile * NT, K, N, out, smem, map, tile.kt_begin, tile.kt_end, slot,
            -1, tile.hid_shift);
    }
    timeline_stamp(map, 4);
}

// Adds the K slices of every tail tile and applies the epilogue the slices skipped.  A workgroup owns
// one group of four columns per lane (a, b, g of the accumulator layout) of one tail tile; its threads
// take the elements the same (wavefront, lane) held in the GEMM, so the slices are read back as they
// were written (1 KiB per wavefront and load), all slices requested at once, and summed in slice
// order.  Does nothing when the launch before it did not split (the same schedule is derived from
// expert_offsets).
template <int MT, int NT, int KT, int WM, int WN, bool TALL, int EPI, bool BIAS>
__global__ __launch_bounds__(WM* WN * 64) void tail_reduce_bf16_kernel(const int32_t* __restrict__ offsets,
                                                                        const bf16_t* __restrict__ bias,  // [E_local,N] or null
                                                                        int max_rows, int K, int N, int E_local,
                                                                        const float4* __restrict__ partial,
                                                                        bf16_t* __restrict__ out, const RowMap map)
{
    constexpr int WM_T = NT / (WM * WN) >= 32 ? 1 : 2, WN_T = WM * WN / WM_T;
    constexpr int WTM = kTailRows / WM_T, WTN = NT / WN_T;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int GROUPS = TN * TM * 4;
    constexpr int SLOT = kTailRows * NT / 4;  // float4 per slice
    const int n_tiles = (N + NT - 1) / NT;
    const TileSchedule sc = scan_experts(offsets, E_local, MT, n_tiles, max_rows, K / KT, true, TALL);
    const int j = blockIdx.x / GROUPS, q = blockIdx.x % GROUPS;
    if (sc.split <= 1 || j >= sc.total_tail) return;
    Tile2D tile;
    if (!decode_tile(sc, E_local, MT, n_tiles, kTileTail, j, tile)) return;
    const int a = q / (TM * 4), b = (q / 4) % TM, g = q % 4;
    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int wm = wave / WN_T, wn = wave % WN_T;
    const float4* mine = partial + static_cast<size_t>(j) * sc.split * SLOT + partial_index<TN, TM>(wave, a, b, g, lane);
    float4 v[kSplitMax];
#pragma unroll
    for (int sl = 0; sl < kSplitMax; ++sl) v[sl] = mine[static_cast<size_t>(min(sl, sc.split - 1)) * SLOT];
    float z[4] = {v[0].x, v[0].y, v[0].z, v[0].w};
#pragma unroll
    for (int sl = 1; sl < kSplitMax; ++sl) {
        if (sl < sc.split) {
            z[0] += v[sl].x;
            z[1] += v[sl].y;
            z[2] += v[sl].z;
            z[3] += v[sl].w;
        }
    }
    const int m = tile.row_begin + wm * WTM + b * 32 + (lane & 31);
    const int n = tile.n_tile * NT + wn * WTN + a * 32 + g * 8 + (lane >> 5) * 4;
    int dst = m;
    float scale = 1.0f;
    if (EPI == kEpiNone && map.out_row != nullptr) {
        dst = map.out_row[min(m, tile.row_end - 1)];
        scale = map.out_scale[dst];
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        if constexpr (BIAS) z[r] += bf16_to_f32(bias[static_cast<size_t>(tile.expert) * N + min(n + r, N - 1)]);
        if constexpr (EPI == kEpiGeluErf) z[r] = gelu_erf_fast(z[r]);
        if constexpr (EPI == kEpiGeluTanh) z[r] = gelu_tanh_fast(z[r]);
        if constexpr (EPI == kEpiNone) z[r] *= scale;
    }
    uint2 packed;
    packed.x = pack_bf16x2(z[0], z[1]);
    packed.y = pack_bf16x2(z[2], z[3]);
    if (m < tile.row_end && n < N)  // N % 8 == 0: the four columns are inside or outside together
        *reinterpret_cast<uint2*>(out + static_cast<size_t>(dst) * N + n) = packed;
}

// ---------------------------------------------------------------------------- fp32 kernel
template <int EPI>
__global__ __launch_bounds__(256) void grouped_gemm_f32_kernel(const float* __restrict__ act, const int32_t* __restrict__ offsets,
                                                                const float* __restrict__ weight, const float* __restrict__ bias,
                                                                int max_rows, int K, int N, int E_local, float* __restrict__ out,
                                                                const RowMap map)
{
    constexpr int MT = 64, NT = 64, KT = 16;
    __shared__ float As[KT][MT + 4];
    __shared__ float Bs[KT][NT + 4];
    if (map.unrouted != nullptr) {  // output rows no sorted row writes: one thread per row clears it
        const int64_t stride = static_cast<int64_t>(gridDim.x) * gridDim.y * 256;
        for (int64_t t = (static_cast<int64_t>(blockIdx.y) * gridDim.x + blockIdx.x) * 256 + threadIdx.x; t < map.n_unrouted; t += stride)
            if (map.unrouted[t] < 0) {
                float4* row = reinterpret_cast<float4*>(out + static_cast<size_t>(t) * N);
                for (int c = 0; c < N / 4; ++c) row[c] = make_float4(0.f, 0.f, 0.f, 0.f);
            }
    }
    const TileRef tile = locate_row_tile(offsets, E_local, MT, blockIdx.x, max_rows);
    if (tile.expert < 0) return;
    const int n0 = blockIdx.y * NT;
    const float* wexp = weight + static_cast<size_t>(tile.expert) * N * K;
    const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
    const int lrow = threadIdx.x / 4, lk = (threadIdx.x % 4) * 4;
    int a_row = min(tile.row_begin + lrow, tile.row_end - 1);
    if (map.a_row != nullptr) a_row = map.a_row[a_row] / map.a_div;
    const float* arow = act + static_cast<size_t>(a_row) * K;
    const float* brow = wexp + static_cast<size_t>(min(n0 + lrow, N - 1)) * K;
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.0f;
    for (int k0 = 0; k0 < K; k0 += KT) {
        float4 a = make_float4(0.f, 0.f, 0.f, 0.f), b = a;
        if (k0 + lk < K) {  // K % 4 == 0
            a = *reinterpret_cast<const float4*>(arow + k0 + lk);
            b = *reinterpret_cast<const float4*>(brow + k0 + lk);
        }
        __syncthreads();
        As[lk + 0][lrow] = a.x; As[lk + 1][lrow] = a.y; As[lk + 2][lrow] = a.z; As[lk + 3][lrow] = a.w;
        Bs[lk + 0][lrow] = b.x; Bs[lk + 1][lrow] = b.y; Bs[lk + 2][lrow] = b.z; Bs[lk + 3][lrow] = b.w;
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < KT; ++kk) {
            float av[4], bv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) av[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) bv[j] = Bs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
        }
    }
    const float* bexp = bias != nullptr ? bias + static_cast<size_t>(tile.expert) * N : nullptr;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = tile.row_begin + ty * 4 + i;
        if (m >= tile.row_end) continue;
        const int n = n0 + tx * 4;
        if (n >= N) continue;  // N % 4 == 0
        int dst = m;
        float scale = 1.0f;
        if (EPI == kEpiNone && map.out_row != nullptr) {
            dst = map.out_row[m];
            scale = map.out_scale[dst];
        }
        float v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float z = acc[i][j];
            if (bexp != nullptr) z += bexp[n + j];
            if constexpr (EPI == kEpiGeluErf) z = gelu_erf_exact(z);
            if constexpr (EPI == kEpiGeluTanh) z = gelu_tanh_exact(z);
            if constexpr (EPI == kEpiNone) z *= scale;
            v[j] = z;
        }
        *reinterpret_cast<float4*>(out + static_cast<size_t>(dst) * N + n) = make_float4(v[0], v[1], v[2], v[3]);
    }
}

// ---------------------------------------------------------------------------- host launchers
template <int MT, int NT, int KT, int STAGES, int WM, int WN, int SWZ, int OCC>
static int launch_bf16(const void* act, const int32_t* offsets, const void* weight, const void* bias, int64_t A, int K, int N,
                       int E_local, int epi, void* out, hipStream_t stream, const RowMap& map = RowMap{}, void* partial = nullptr)
{
    constexpr size_t lds = static_cast<size_t>(ring_bytes(MT, NT, KT, STAGES, WM)) + row_id_scratch_bytes(MT, NT, KT, STAGES, WM, WM * WN);
    static_assert(NT <= kSplitMaxCols, "a partial-sum slot holds kTailRows x kSplitMaxCols values");
    // worst case: A/MT unmasked row tiles plus, for every expert, its tail tiles or one masked tile;
    // cutting tail tiles into K slices adds fewer than kSplitUnits work items
    const int64_t n_tiles = (N + NT - 1) / NT;
    const int64_t row_tiles = A / MT + static_cast<int64_t>(E_local) * max_tail_tiles(MT);
    const int64_t ub = row_tiles * n_tiles + (partial != nullptr ? kSplitUnits : 0);
    const int64_t round = static_cast<int64_t>(kXcdCount) * kXcdChunk;
    const int64_t grid = (ub + round - 1) / round * round;
    if (grid >= (1ll << 31)) return fail(EXF_ERR_BAD_SHAPE, "moe_expert_ffn: too many tiles");
#define EXF_LAUNCH_BF16(EPI, BIAS)                                                                                              \
    do {                                                                                                                        \
        auto kern = grouped_gemm_bf16_kernel<MT, NT, KT, STAGES, WM, WN, SWZ, OCC, EPI, BIAS>;                                  \
        if (lds > 64 * 1024) {                                                                                                  \
            hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, \
                                                 static_cast<int>(lds));                                                       \
            if (err != hipSuccess) return fail(EXF_ERR_HIP, "moe_expert_ffn: LDS attribute: %s", hipGetErrorString(err));       \
        }                                                                                                                       \
        hipLaunchKernelGGL(kern, dim3(static_cast<unsigned>(grid)), dim3(WM* WN * 64), lds, stream,                              \
                           static_cast<const bf16_t*>(act), offsets, static_cast<const bf16_t*>(weight),                        \
                           static_cast<const bf16_t*>(bias), static_cast<int>(A), K, N, E_local, static_cast<bf16_t*>(out),     \
                           map, static_cast<float4*>(partial));                                                                 \
        if (partial != nullptr && MT > kTailRows && K / KT >= 2 * kSplitMinKTiles)                                              \
            hipLaunchKernelGGL((tail_reduce_bf16_kernel<MT, NT, KT, WM, WN, tall_tiles_supported(MT, NT, KT, STAGES, WM), EPI, BIAS>),                                        \
                               dim3(kSplitUnits / 2 * (kTailRows * NT / (WM * WN * 64 * 4))),                                   \
                               dim3(WM* WN * 64), 0, stream, offsets, static_cast<const bf16_t*>(bias), static_cast<int>(A), K, \
                               N, E_local, static_cast<const float4*>(partial), static_cast<bf16_t*>(out), map);                \
    } while (0)
    if (bias == nullptr) {
        if (epi == kEpiNone) EXF_LAUNCH_BF16(kEpiNone, false);
        else if (epi == kEpiGeluErf) EXF_LAUNCH_BF16(kEpiGeluErf, false);
        else EXF_LAUNCH_BF16(kEpiGeluTanh, false);
    } else {
        if (epi == kEpiNone) EXF_LAUNCH_BF16(kEpiNone, true);
        else if (epi == kEpiGeluErf) EXF_LAUNCH_BF16(kEpiGeluErf, true);
        else EXF_LAUNCH_BF16(kEpiGeluTanh, true);
    }
#undef EXF_LAUNCH_BF16
    return EXF_OK;
}

static int launch_f32(const void* act, const int32_t* offsets, const void* weight, const void* bias, int64_t A, int K, int N,
                      int E_local, int epi, void* out, hipStream_t stream, const RowMap& map = RowMap{})
{
    const int64_t row_tiles = (A + 63) / 64 + E_local;
    const int64_t n_tiles = (N + 63) / 64;
    if (row_tiles >= (1ll << 31) || n_tiles > 65535) return fail(EXF_ERR_BAD_SHAPE, "moe_expert_ffn: too many tiles");
    const dim3 grid(static_cast<unsigned>(row_tiles), static_cast<unsigned>(n_tiles));
    const float* a = static_cast<const float*>(act);
    const float* w = static_cast<const float*>(weight);
    const float* b = static_cast<const float*>(bias);
    float* o = static_cast<float*>(out);
    if (epi == kEpiNone)
        hipLaunchKernelGGL(grouped_gemm_f32_kernel<kEpiNone>, grid, dim3(256), 0, stream, a, offsets, w, b, static_cast<int>(A), K, N, E_local, o, map);
    else if (epi == kEpiGeluErf)
        hipLaunchKernelGGL(grouped_gemm_f32_kernel<kEpiGeluErf>, grid, dim3(256), 0, stream, a, offsets, w, b, static_cast<int>(A), K, N, E_local, o, map);
    else
        hipLaunchKernelGGL(grouped_gemm_f32_kernel<kEpiGeluTanh>, grid, dim3(256), 0, stream, a, offsets, w, b, static_cast<int>(A), K, N, E_local, o, map);
    return EXF_OK;
}

// Tile configurations of the two contractions: <MT, NT, KT, STAGES, WM, WN, SWZ, OCC> (OCC = wavefronts
// per SIMD the register allocation must leave room for).  kWideTile: 256x256x64, two stages, 2x4
// wavefronts of 128x64; kNarrowTile: 256x128x64, three stages, 4x2 wavefronts of 64x64.
template <typename... Args>
static int launch_wide_tile(Args&&... args)
{
    return launch_bf16<256, 256, 64, 2, 2, 4, 1, 1>(static_cast<Args&&>(args)...);
}
template <typename... Args>
static int launch_narrow_tile(Args&&... args)
{
    return launch_bf16<256, 128, 64, 3, 4, 2, 1, 1>(static_cast<Args&&>(args)...);
}

// The second contraction has few output columns (N = d).  With 256x128 tiles it offers twice as many
// tiles, which a short batch needs to fill the chip; the 256x256 tile of the first contraction moves
// a third less operand data per flop through the L2s and is taken once it, too, gives every compute
// unit at least kWideRounds tiles.
constexpr int kWideRounds = 2;  // (1 measured the same on 16384 and 32768 tokens)
static int launch_second_contraction(const void* act, const int32_t* offsets, const void* weight, const void* bias, int64_t A,
                                     int K, int N, int E_local, void* out, hipStream_t stream, const RowMap& map, void* partial)
{
    const int64_t wide_tiles = (A / 256) * ((N + 255) / 256);
    if (wide_tiles >= static_cast<int64_t>(kWideRounds) * kSplitUnits)
        return launch_wide_tile(act, offsets, weight, bias, A, K, N, E_local, static_cast<int>(kEpiNone), out, stream, map, partial);
    return launch_narrow_tile(act, offsets, weight, bias, A, K, N, E_local, static_cast<int>(kEpiNone), out, stream, map, partial);
}

}  // namespace exf


namespace exf {
// Bytes of the hidden activations of A sorted rows.  bf16: every expert starts on a 32-row boundary
// (see RowMap), so up to 32 rows per expert are padding.
static size_t hidden_bytes(int64_t A, int f, int E_local, int dt)
{
    size_t rows = static_cast<size_t>(A > 0 ? A : 1);
    if (dt == EXF_BF16) rows = (rows + static_cast<size_t>(kHiddenRowBlock) * (E_local > 0 ? E_local : 1) + kHiddenRowBlock - 1) / kHiddenRowBlock * kHiddenRowBlock;
    return align_up(rows * static_cast<size_t>(f) * (dt == EXF_BF16 ? 2 : 4), 256);
}
}  // namespace exf

extern "C" size_t moe_expert_ffn_workspace_bytes(int64_t A, int d, int f, int E_local, int dt)
{
    (void)d;
    if (A < 0 || f < 1 || (dt != EXF_F32 && dt != EXF_BF16)) return 0;
    return exf::hidden_bytes(A, f, E_local, dt) + (dt == EXF_BF16 ? exf::kSplitBytes : 0);  // bf16: + the partial sums of K-sliced tail tiles
}

extern "C" int moe_expert_ffn(const void* x_sorted, const int32_t* expert_offsets, const void* w1, const void* b1, const void* w2,
                              const void* b2, int64_t A, int d, int f, int E_local, int act, int dt, void* y_sorted,
                              void* workspace, size_t workspace_bytes, void* stream)
{
    using namespace exf;
    if (dt != EXF_F32 && dt != EXF_BF16) return fail(EXF_ERR_BAD_DTYPE, "moe_expert_ffn: dt = %d", dt);
    if (act != EXF_ACT_GELU_ERF && act != EXF_ACT_GELU_TANH) return fail(EXF_ERR_BAD_SHAPE, "moe_expert_ffn: act = %d", act);
    if (A < 0 || A >= (1ll << 31)) return fail(EXF_ERR_BAD_SHAPE, "moe_expert_ffn: A = %lld outside [0,2^31)", static_cast<long long>(A));
    if (E_local < 1 || E_local > EXF_MAX_EXPERTS)
        return fail(EXF_ERR_BAD_SHAPE, "moe_expert_ffn: E_local = %d outside [1,%d]", E_local, EXF_MAX_EXPERTS);
    const int gran = dt == EXF_BF16 ? 64 : 4;
    if (d < gran || d % gran != 0 || f < gran || f % gran != 0)
        return fail(EXF_ERR_BAD_SHAPE, "moe_expert_ffn: d = %d and f = %d must be positive multiples of %d", d, f, gran);
    if (dt == EXF_BF16) {  // the bf16 kernel addresses rows with 32-bit byte offsets
        const unsigned long long widest = static_cast<unsigned long long>(d > f ? d : f);
        const unsigned long long rows = static_cast<unsigned long long>(A) + static_cast<unsigned long long>(kHiddenRowBlock) * (E_local + 1);
        if (rows * widest * 2ull >= (1ull << 32) ||
            static_cast<unsigned long long>(d) * static_cast<unsigned long long>(f) * 2ull >= (1ull << 32))
            return fail(EXF_ERR_BAD_SHAPE, "moe_expert_ffn: (A + 32 (E_local + 1))*max(d,f) and d*f must stay below 2^31 elements (bf16)");
    }
    if (A == 0) return EXF_OK;
    EXF_REQUIRE_PTR(x_sorted);
    EXF_REQUIRE_PTR(expert_offsets);
    EXF_REQUIRE_PTR(w1);
    EXF_REQUIRE_PTR(w2);
    EXF_REQUIRE_PTR(y_sorted);
    EXF_REQUIRE_PTR(workspace);
    EXF_REQUIRE_ALIGNED(x_sorted);
    EXF_REQUIRE_ALIGNED(w1);
    EXF_REQUIRE_ALIGNED(w2);
    EXF_REQUIRE_ALIGNED(y_sorted);
    EXF_REQUIRE_ALIGNED(workspace);
    if (workspace_bytes < moe_expert_ffn_workspace_bytes(A, d, f, E_local, dt))
        return fail(EXF_ERR_WORKSPACE_TOO_SMALL, "moe_expert_ffn: workspace %zu < %zu bytes", workspace_bytes,
                    moe_expert_ffn_workspace_bytes(A, d, f, E_local, dt));
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int epi = act == EXF_ACT_GELU_ERF ? kEpiGeluErf : kEpiGeluTanh;
    int rc;
    if (dt == EXF_F32) {
        rc = launch_f32(x_sorted, expert_offsets, w1, b1, A, d, f, E_local, epi, workspace, s);
        if (rc == EXF_OK) rc = launch_f32(workspace, expert_offsets, w2, b2, A, f, d, E_local, kEpiNone, y_sorted, s);
    } else {
        void* partial = static_cast<unsigned char*>(workspace) + hidden_bytes(A, f, E_local, dt);
        RowMap first{}, second{};
        first.hidden_out = 1;
        second.hidden_act = 1;
        rc = launch_wide_tile(x_sorted, expert_offsets, w1, b1, A, d, f, E_local, epi, workspace, s, first,
                              kSplitFirstContraction ? partial : nullptr);
        if (rc == EXF_OK)
            rc = launch_second_contraction(workspace, expert_offsets, w2, b2, A, f, d, E_local, y_sorted, s, second, partial);
    }
    if (rc != EXF_OK) return rc;
    return check_launch("moe_expert_ffn");
}

extern "C" int moe_combine(const void* y_sorted, const int32_t* sorted_of_src, const float* topk_w, int64_t T, int d, int k,
                           int dt, void* out, void* stream);

extern "C" size_t moe_expert_ffn_fused_workspace_bytes(int64_t T, int k, int d, int f, int E_local, int dt)
{
    if (T < 0 || k < 1 || k > EXF_MAX_TOPK || d < 1 || f < 1 || (dt != EXF_BF16 && dt != EXF_F32)) return 0;
    const size_t elem = dt == EXF_BF16 ? 2 : 4;
    const size_t A = static_cast<size_t>(T > 0 ? T : 1) * static_cast<size_t>(k);
    size_t bytes = exf::hidden_bytes(static_cast<int64_t>(A), f, E_local, dt);  // hidden activations of A rows
    if (k > 1) bytes += exf::align_up(A * static_cast<size_t>(d) * elem, 256);   // sorted expert outputs [A,d]
    return bytes + (dt == EXF_BF16 ? exf::kSplitBytes : 0);                      // bf16: partial sums of K-sliced tail tiles
}

static int ffn_fused_run(const char* fn, const void* x, const int32_t* src_of_sorted, const int32_t* sorted_of_src, const float* topk_w,
                         const int32_t* expert_offsets, const void* w1, const void* b1, const void* w2, const void* b2, int64_t T, int k,
                         int d, int f, int E_local, int act, int dt, void* out, void* workspace, size_t workspace_bytes, void* stream,
                         unsigned long long* timeline, int timeline_cap)
{
    using namespace exf;
    (void)fn;
    if (dt != EXF_F32 && dt != EXF_BF16) return fail(EXF_ERR_BAD_DTYPE, "moe_expert_ffn_fused: dt = %d", dt);
    if (act != EXF_ACT_GELU_ERF && act != EXF_ACT_GELU_TANH) return fail(EXF_ERR_BAD_SHAPE, "moe_expert_ffn_fused: act = %d", act);
    if (k < 1 || k > EXF_MAX_TOPK) return fail(EXF_ERR_BAD_SHAPE, "moe_expert_ffn_fused: k = %d outside [1,%d]", k, EXF_MAX_TOPK);
    if (T < 0 || T * k >= (1ll << 31))
        return fail(EXF_ERR_BAD_SHAPE, "moe_expert_ffn_fused: T = %lld, T*k outside [0,2^31)", static_cast<long long>(T));
    if (E_local < 1 || E_local > EXF_MAX_EXPERTS)
        return fail(EXF_ERR_BAD_SHAPE, "moe_expert_ffn_fused: E_local = %d outside [1,%d]", E_local, EXF_MAX_EXPERTS);
    const int gran = dt == EXF_BF16 ? 64 : 4;
    if (d < gran || d % gran != 0 || f < gran || f % gran != 0)
        return fail(EXF_ERR_BAD_SHAPE, "moe_expert_ffn_fused: d = %d and f = %d must be positive multiples of %d", d, f, gran);
    const int64_t A = T * k;
    if (dt == EXF_BF16) {  // the bf16 kernel addresses rows with 32-bit byte offsets
        const unsigned long long widest = static_cast<unsigned long long>(d > f ? d : f);
        const unsigned long long rows = static_cast<unsigned long long>(A) + static_cast<unsigned long long>(kHiddenRowBlock) * (E_local + 1);
        if (rows * widest * 2ull >= (1ull << 32) ||
            static_cast<unsigned long long>(d) * static_cast<unsigned long long>(f) * 2ull >= (1ull << 32))
            return fail(EXF_ERR_BAD_SHAPE, "moe_expert_ffn_fused: (T*k + 32 (E_local + 1))*max(d,f) and d*f must stay below 2^31 elements");
    }
    if (T == 0) return EXF_OK;
    EXF_REQUIRE_PTR(x);
    EXF_REQUIRE_PTR(src_of_sorted);
    EXF_REQUIRE_PTR(sorted_of_src);
    EXF_REQUIRE_PTR(topk_w);
    EXF_REQUIRE_PTR(expert_offsets);
    EXF_REQUIRE_PTR(w1);
    EXF_REQUIRE_PTR(w2);
    EXF_REQUIRE_PTR(out);
    EXF_REQUIRE_PTR(workspace);
    EXF_REQUIRE_ALIGNED(x);
    EXF_REQUIRE_ALIGNED(w1);
    EXF_REQUIRE_ALIGNED(w2);
    EXF_REQUIRE_ALIGNED(out);
    EXF_REQUIRE_ALIGNED(workspace);
    if (x == out) return fail(EXF_ERR_BAD_SHAPE, "moe_expert_ffn_fused: out must not alias x");
    const size_t need = moe_expert_ffn_fused_workspace_bytes(T, k, d, f, E_local, dt);
    if (workspace_bytes < need) return fail(EXF_ERR_WORKSPACE_TOO_SMALL, "moe_expert_ffn_fused: workspace %zu < %zu bytes", workspace_bytes, need);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int epi = act == EXF_ACT_GELU_ERF ? kEpiGeluErf : kEpiGeluTanh;
    const size_t elem = dt == EXF_BF16 ? 2 : 4;
    unsigned char* hidden = static_cast<unsigned char*>(workspace);
    RowMap gather{};
    gather.a_row = src_of_sorted;
    gather.a_div = k;
    gather.timeline = timeline;  // first contraction: records [0, cap), second: [cap, 2 cap)
    gather.timeline_cap = timeline_cap;
    RowMap scatter{};
    scatter.timeline = timeline != nullptr ? timeline + static_cast<size_t>(timeline_cap) * 8 : nullptr;
    scatter.timeline_cap = timeline_cap;
    if (k == 1) {
        scatter.out_row = src_of_sorted;  // k = 1: the flat assignment index is the token
        scatter.out_scale = topk_w;
        scatter.unrouted = sorted_of_src;
        scatter.n_unrouted = static_cast<int>(T);
    }
    unsigned char* y_sorted = hidden + hidden_bytes(A, f, E_local, dt);
    if (dt == EXF_BF16) {
        gather.hidden_out = 1;
        scatter.hidden_act = 1;
    }
    void* second_out = k == 1 ? out : static_cast<void*>(y_sorted);
    int rc;
    if (dt == EXF_F32) {
        rc = launch_f32(x, expert_offsets, w1, b1, A, d, f, E_local, epi, hidden, s, gather);
        if (rc == EXF_OK) rc = launch_f32(hidden, expert_offsets, w2, b2, A, f, d, E_local, kEpiNone, second_out, s, scatter);
    } else {
        void* partial = y_sorted + (k > 1 ? align_up(static_cast<size_t>(A) * static_cast<size_t>(d) * 2, 256) : 0);
        rc = launch_wide_tile(x, expert_offsets, w1, b1, A, d, f, E_local, epi, hidden, s, gather,
                              kSplitFirstContraction ? partial : nullptr);
        if (rc == EXF_OK) rc = launch_second_contraction(hidden, expert_offsets, w2, b2, A, f, d, E_local, second_out, s, scatter, partial);
    }
    if (rc != EXF_OK) return rc;
    if (k == 1) return check_launch("moe_expert_ffn_fused");
    rc = check_launch("moe_expert_ffn_fused");
    if (rc != EXF_OK) return rc;
    return moe_combine(y_sorted, sorted_of_src, topk_w, T, d, k, dt, out, stream);
}

extern "C" int moe_expert_ffn_fused(const void* x, const int32_t* src_of_sorted, const int32_t* sorted_of_src, const float* topk_w,
                                    const int32_t* expert_offsets, const void* w1, const void* b1, const void* w2, const void* b2,
                                    int64_t T, int k, int d, int f, int E_local, int act, int dt, void* out, void* workspace,
                                    size_t workspace_bytes, void* stream)
{
    return ffn_fused_run("moe_expert_ffn_fused", x, src_of_sorted, sorted_of_src, topk_w, expert_offsets, w1, b1, w2, b2, T, k, d, f,
                         E_local, act, dt, out, workspace, workspace_bytes, stream, nullptr, 0);
}

// moe_expert_ffn_fused (bf16) with a per-workgroup timeline of both contractions (see RowMap::timeline).
extern "C" int exf_probe_ffn_timeline(const void* x, const int32_t* src_of_sorted, const int32_t* sorted_of_src, const float* topk_w,
                                      const int32_t* expert_offsets, const void* w1, const void* w2, int64_t T, int k, int d, int f,
                                      int E_local, void* out, void* workspace, size_t workspace_bytes, uint64_t* timeline,
                                      int capacity, void* stream)
{
    EXF_REQUIRE_PTR(timeline);
    if (capacity < 1) return exf::fail(EXF_ERR_BAD_SHAPE, "exf_probe_ffn_timeline: capacity = %d < 1", capacity);
    return ffn_fused_run("exf_probe_ffn_timeline", x, src_of_sorted, sorted_of_src, topk_w, expert_offsets, w1, nullptr, w2, nullptr, T, k,
                         d, f, E_local, EXF_ACT_GELU_ERF, EXF_BF16, out, workspace, workspace_bytes, stream,
                         reinterpret_cast<unsigned long long*>(timeline), capacity);
}
