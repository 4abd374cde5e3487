// moe_dispatch: stable counting sort of the token-to-expert assignments + row gather.
//
//   1. count   : every workgroup histograms its chunk of CH consecutive assignments into LDS
//                and stores one row of per-expert counts.
//   2. scan    : the [blocks x E_local] count matrix becomes per-chunk start positions (exclusive
//                scan down each expert column) plus expert_counts / expert_offsets.  Up to 256
//                chunks every scatter workgroup does this for itself from the small matrix; a
//                separate one-workgroup scan kernel serves longer inputs.
//   3. place   : every workgroup takes a slice of 32 or 64 assignments of one chunk, ranks it —
//                assignments of the chunk in front of the slice recounted from the ids, rank
//                inside the slice = number of lower lanes that hold the same expert (those lanes
//                are found with one ballot per bit of the id) — which keeps equal experts in
//                ascending assignment order (stable, hence
//                a unique permutation), writes both index maps and copies the slice's rows
//                x_sorted[position] = x[assignment / k] as 16-byte vector copies.
//                (Without rows to move, dispatch_scatter_kernel ranks whole chunks instead.)
//   Index maps only and at most 16384 assignments: ONE workgroup of 1024 threads does all three steps
//   in a single launch (dispatch_small_kernel) - at that size the launches, not the work, are the cost.
// No step needs the host to know a data-dependent size.
#include <mutex>

#include "common.hpp"

namespace exf {

constexpr int kDispThreads = 256;
constexpr int kDispWaves = kDispThreads / kWave;
constexpr int kDispChunk = 1024;  // assignments per workgroup in count / scatter
constexpr int kDispFusedScanBlocks = 256;  // up to this many chunks every scatter workgroup scans the count matrix itself

constexpr int kDispRounds = kDispChunk / kDispThreads;  // assignments per thread

// Local expert ids of this thread's kDispRounds assignments (a = base + r*kDispThreads + tid), -1
// for assignments past the end, outside [0,E) or mapped to no local expert.  All global ids are
// loaded first and all map entries next, each through a clamped (never branched-around) address:
// two memory round trips for the whole chunk instead of two per assignment.
__device__ __forceinline__ void load_local_experts(const int32_t* __restrict__ topk_idx, const int32_t* __restrict__ expert_map,
                                                   int64_t base, int64_t A, int E, int E_local, int (&e)[kDispRounds])
{
    int g[kDispRounds];
#pragma unroll
    for (int r = 0; r < kDispRounds; ++r) {
        const int64_t a = base + r * kDispThreads + threadIdx.x;
        g[r] = topk_idx[min(a, A - 1)];
        if (a >= A) g[r] = -1;
    }
    if (expert_map != nullptr) {
#pragma unroll
        for (int r = 0; r < kDispRounds; ++r) {
            const bool ok = g[r] >= 0 && g[r] < E;
            const int m = expert_map[ok ? g[r] : 0];
            e[r] = (ok && m >= 0 && m < E_local) ? m : -1;
        }
    } else {
#pragma unroll
        for (int r = 0; r < kDispRounds; ++r) e[r] = (g[r] >= 0 && g[r] < E && g[r] < E_local) ? g[r] : -1;
    }
}

// Lanes of the wavefront that hold the same local expert as this lane (meaningful where e >= 0): the
// ids are compared bit by bit, log2(E_local) ballots instead of one ballot per expert.
__device__ __forceinline__ unsigned long long same_expert_lanes(int e, int E_local)
{
    unsigned long long m = __ballot(e >= 0);
    for (int bit = 1; bit < E_local; bit <<= 1) {
        const unsigned long long b = __ballot((e & bit) != 0);
        m &= (e & bit) != 0 ? b : ~b;
    }
    return m;
}

__global__ __launch_bounds__(kDispThreads) void dispatch_count_kernel(const int32_t* __restrict__ topk_idx,
                                                                       const int32_t* __restrict__ expert_map, int64_t A,
                                                                       int E, int E_local,
                                                                       int32_t* __restrict__ block_counts)
{
    __shared__ int cnt[EXF_MAX_EXPERTS];
    if (threadIdx.x < EXF_MAX_EXPERTS) cnt[threadIdx.x] = 0;
    __syncthreads();
    const int64_t base = static_cast<int64_t>(blockIdx.x) * kDispChunk;
    int e[kDispRounds];
    load_local_experts(topk_idx, expert_map, base, A, E, E_local, e);
#pragma unroll
    for (int r = 0; r < kDispRounds; ++r)
        if (e[r] >= 0) atomicAdd(&cnt[e[r]], 1);
    __syncthreads();
    if (threadIdx.x < E_local) block_counts[static_cast<int64_t>(blockIdx.x) * E_local + threadIdx.x] = cnt[threadIdx.x];
}

// One workgroup of 64 threads: thread e walks down column e of block_counts.
__global__ __launch_bounds__(kWave) void dispatch_scan_kernel(int32_t* __restrict__ block_counts, int n_blocks, int E_local,
                                                               int32_t* __restrict__ expert_counts,
                                                               int32_t* __restrict__ expert_offsets)
{
    const int e = threadIdx.x;
    int total = 0;
    if (e < E_local) {
        for (int b = 0; b < n_blocks; ++b) {
            const int64_t i = static_cast<int64_t>(b) * E_local + e;
            const int c = block_counts[i];
            block_counts[i] = total;  // start of this chunk inside expert e's bucket
            total += c;
        }
        expert_counts[e] = total;
    }
    const int incl = wave_inclusive_scan(e < E_local ? total : 0);
    if (e < E_local) expert_offsets[e] = incl - total;
    if (e == E_local - 1) expert_offsets[E_local] = incl;
}

// FUSED_SCAN: block_base holds the RAW per-chunk counts of dispatch_count_kernel and every
// workgroup derives its own start positions (column sums over the chunks before it) and the
// expert offsets (column totals) from that small matrix - no separate scan launch.  Otherwise
// block_base already holds the scanned start positions.
template <bool FUSED_SCAN>
__global__ __launch_bounds__(kDispThreads) void dispatch_scatter_kernel(
    const int32_t* __restrict__ topk_idx, const int32_t* __restrict__ expert_map, int64_t A, int E, int E_local,
    const int32_t* __restrict__ block_base, int32_t* __restrict__ expert_counts, int32_t* __restrict__ expert_offsets,
    int32_t* __restrict__ src_of_sorted, int32_t* __restrict__ sorted_of_src)
{
    __shared__ int cursor[EXF_MAX_EXPERTS];               // next free sorted position per expert
    __shared__ int wave_cnt[kDispRounds][kDispWaves][EXF_MAX_EXPERTS];  // per-round, per-wavefront counts
    const int lane = lane_id();
    const int wave = threadIdx.x / kWave;
    int e_mine[kDispRounds];
    const int64_t base = static_cast<int64_t>(blockIdx.x) * kDispChunk;
    load_local_experts(topk_idx, expert_map, base, A, E, E_local, e_mine);  // in flight during the scan
    for (int i = threadIdx.x; i < kDispRounds * kDispWaves * EXF_MAX_EXPERTS; i += kDispThreads) (&wave_cnt[0][0][0])[i] = 0;
    if constexpr (FUSED_SCAN) {
        // column sums of the count matrix [chunks][E_local]: over all chunks (expert totals) and over
        // the chunks before this one; all threads load side by side, four entries each per pass
        __shared__ int col_total[EXF_MAX_EXPERTS], col_before[EXF_MAX_EXPERTS];
        if (threadIdx.x < EXF_MAX_EXPERTS) {
            col_total[threadIdx.x] = 0;
            col_before[threadIdx.x] = 0;
        }
        __syncthreads();
        const int n = static_cast<int>(gridDim.x) * E_local;
        const int mine = static_cast<int>(blockIdx.x) * E_local;  // entries below belong to earlier chunks
        constexpr int UL = 4;
        for (int i0 = threadIdx.x; i0 < n; i0 += kDispThreads * UL) {
            int c[UL];
#pragma unroll
            for (int u = 0; u < UL; ++u) c[u] = block_base[min(i0 + u * kDispThreads, n - 1)];
#pragma unroll
            for (int u = 0; u < UL; ++u) {
                const int i = i0 + u * kDispThreads;
                if (i < n && c[u] != 0) {
                    const int q = i % E_local;
                    atomicAdd(&col_total[q], c[u]);
                    if (i < mine) atomicAdd(&col_before[q], c[u]);
                }
            }
        }
        __syncthreads();
        if (wave == 0) {
            const int total = lane < E_local ? col_total[lane] : 0;
            const int incl = wave_inclusive_scan(total);
            if (lane < E_local) cursor[lane] = incl - total + col_before[lane];
            if (blockIdx.x == 0) {
                if (lane < E_local) {
                    expert_counts[lane] = total;
                    expert_offsets[lane] = incl - total;
                }
                if (lane == E_local - 1) expert_offsets[E_local] = incl;
            }
        }
    } else {
        if (threadIdx.x < E_local)
            cursor[threadIdx.x] = expert_offsets[threadIdx.x] + block_base[static_cast<int64_t>(blockIdx.x) * E_local + threadIdx.x];
    }
    __syncthreads();

    // Rank of an assignment among the chunk's assignments to the same expert = those in earlier
    // rounds and wavefronts (per-round, per-wavefront counts, exchanged through LDS once) plus the
    // lanes below it in its own wavefront (ballot).  Assignments are numbered round-major, so this
    // is ascending assignment order: the sort is stable and the permutation unique.
    const unsigned long long below = (1ull << lane) - 1ull;
    int rank[kDispRounds];
#pragma unroll
    for (int round = 0; round < kDispRounds; ++round) {
        const int e = e_mine[round];
        const unsigned long long m = same_expert_lanes(e, E_local);
        rank[round] = __popcll(m & below);
        if (e >= 0 && (m & below) == 0ull) wave_cnt[round][wave][e] = __popcll(m);  // the lowest lane of every expert present
    }
    __syncthreads();  // counts of all rounds and wavefronts, and the cursors, are in LDS
#pragma unroll
    for (int round = 0; round < kDispRounds; ++round) {
        const int64_t a = base + round * kDispThreads + threadIdx.x;
        const int e = e_mine[round];
        if (e >= 0) {
            int pos = cursor[e] + rank[round];
            const int* earlier = &wave_cnt[0][0][e];
            const int n_earlier = round * kDispWaves + wave;
            for (int i = 0; i < n_earlier; ++i) pos += earlier[i * EXF_MAX_EXPERTS];
            src_of_sorted[pos] = static_cast<int32_t>(a);
            sorted_of_src[a] = pos;
        } else if (a < A) {
            sorted_of_src[a] = -1;
        }
    }
}

// Count, scan and scatter of a short assignment list in one workgroup of 16 wavefronts (index maps
// only).  Thread t takes the assignments a = r*1024 + t, r < R.  A "segment" is what one wavefront
// holds in one round; segments in (round, wavefront) order are ascending assignment order.  Every
// segment counts its experts with the ballots of same_expert_lanes, a wavefront per expert scans the
// R*16 segment counts into segment starts and the expert's total, one wavefront scans the totals into
// the bucket starts: position = bucket start + segment start + lower lanes with the same expert - the
// same stable permutation as the chunked kernels.
constexpr int kSmallThreads = 1024;
constexpr int kSmallWaves = kSmallThreads / kWave;
constexpr int kSmallMaxRounds = 16;
template <int R>
__global__ __launch_bounds__(kSmallThreads) void dispatch_small_kernel(const int32_t* __restrict__ topk_idx,
                                                                        const int32_t* __restrict__ expert_map, int64_t A, int E,
                                                                        int E_local, int32_t* __restrict__ expert_counts,
                                                                        int32_t* __restrict__ expert_offsets,
                                                                        int32_t* __restrict__ src_of_sorted,
                                                                        int32_t* __restrict__ sorted_of_src)
{
    constexpr int SEG = R * kSmallWaves;       // segments
    constexpr int PER = SEG / kWave;           // consecutive segments a lane scans
    static_assert(SEG % kWave == 0 && R <= kSmallMaxRounds, "segment scan layout");
    __shared__ unsigned short seg[EXF_MAX_EXPERTS][SEG];  // count, then start, of a segment inside its expert's bucket (<= 16384)
    __shared__ int total[EXF_MAX_EXPERTS];
    const int lane = lane_id();
    const int wave = threadIdx.x / kWave;

    int g[R], e[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {  // all ids first, all map entries next: two memory round trips in total
        const int64_t a = static_cast<int64_t>(r) * kSmallThreads + threadIdx.x;
        g[r] = topk_idx[min(a, A - 1)];
    }
    {   // (cleared while the ids are on their way)
        uint32_t* words = reinterpret_cast<uint32_t*>(&seg[0][0]);
        for (int i = threadIdx.x; i < EXF_MAX_EXPERTS * SEG / 2; i += kSmallThreads) words[i] = 0u;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int64_t a = static_cast<int64_t>(r) * kSmallThreads + threadIdx.x;
        const bool ok = a < A && g[r] >= 0 && g[r] < E;
        if (expert_map != nullptr) {
            const int m = expert_map[ok ? g[r] : 0];
            e[r] = (ok && m >= 0 && m < E_local) ? m : -1;
        } else {
            e[r] = (ok && g[r] < E_local) ? g[r] : -1;
        }
    }

    const unsigned long long below = (1ull << lane) - 1ull;
    int rank[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const unsigned long long m = same_expert_lanes(e[r], E_local);
        rank[r] = __popcll(m & below);
        if (e[r] >= 0 && (m & below) == 0ull) seg[e[r]][r * kSmallWaves + wave] = static_cast<unsigned short>(__popcll(m));
    }
    __syncthreads();

    for (int q = wave; q < E_local; q += kSmallWaves) {
        int c[PER], sum = 0;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            c[j] = seg[q][lane * PER + j];
            sum += c[j];
        }
        const int incl = wave_inclusive_scan(sum);
        int run = incl - sum;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            seg[q][lane * PER + j] = static_cast<unsigned short>(run);
            run += c[j];
        }
        if (lane == kWave - 1) total[q] = incl;
    }
    __syncthreads();
    // every wavefront scans the totals for itself: lane q then holds the start of expert q's bucket
    const int t = lane < E_local ? total[lane] : 0;
    const int incl = wave_inclusive_scan(t);
    const int bucket = incl - t;
    if (wave == 0) {
        if (lane < E_local) {
            expert_counts[lane] = t;
            expert_offsets[lane] = bucket;
        }
        if (lane == E_local - 1) expert_offsets[E_local] = incl;
    }

#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int64_t a = static_cast<int64_t>(r) * kSmallThreads + threadIdx.x;
        const int start = __shfl(bucket, max(e[r], 0));  // (all lanes take part: a shuffle reads active lanes only)
        if (e[r] >= 0) {
            const int pos = start + seg[e[r]][r * kSmallWaves + wave] + rank[r];
            src_of_sorted[pos] = static_cast<int32_t>(a);
            sorted_of_src[a] = pos;
        } else if (a < A) {
            sorted_of_src[a] = -1;
        }
    }
}

// Scatter and row move in one launch (used whenever rows are moved).  A workgroup owns MOVE
// consecutive assignments - a slice of one 1024-assignment chunk of the count matrix.  It
//   - derives the chunk's start positions like dispatch_scatter_kernel (column sums, or the scanned
//     matrix), adds the assignments of its chunk that precede its slice (recounted from the ids,
//     LDS atomics), and ranks its own slice by the lanes below that hold the same expert: stable, same permutation;
//   - writes both index maps for its slice;
//   - copies its rows x[a / k] -> x_sorted[position]: every wavefront takes MOVE/4 rows and streams
//     them as a flat sequence of 16-byte chunks (`vec_per_row` = row bytes / 16) with non-temporal
//     loads and stores, four chunks per lane in flight and the next four requested before these
//     are stored (branch-free when every row of the wavefront is kept and the chunks divide evenly).
template <bool FUSED_SCAN, int MOVE>
__global__ __launch_bounds__(kDispThreads) void dispatch_place_kernel(
    const int32_t* __restrict__ topk_idx, const int32_t* __restrict__ expert_map, int64_t A, int E, int E_local, int n_coarse,
    const int32_t* __restrict__ block_base, int32_t* __restrict__ expert_counts, int32_t* __restrict__ expert_offsets,
    int32_t* __restrict__ src_of_sorted, int32_t* __restrict__ sorted_of_src, const uint4* __restrict__ x, int k, int vec_per_row,
    uint4* __restrict__ x_sorted)
{
    static_assert(MOVE == 32 || MOVE == 64, "a slice is ranked by one wavefront and split over four");
    constexpr int SUBS = kDispChunk / MOVE;  // slices per chunk
    constexpr int ROWS = MOVE / kDispWaves;  // rows a wavefront moves
    __shared__ int cursor[EXF_MAX_EXPERTS];  // start of the chunk inside every expert's bucket
    __shared__ int pre[EXF_MAX_EXPERTS];     // assignments of the chunk in front of the slice, per expert
    __shared__ int pos_s[MOVE];              // sorted position of every assignment of the slice (-1: not kept)
    const int lane = lane_id();
    const int wave = threadIdx.x / kWave;
    const int cc = blockIdx.x / SUBS, sub = blockIdx.x % SUBS;
    const int64_t base = static_cast<int64_t>(cc) * kDispChunk;
    const int first = sub * MOVE;  // the slice: assignments base + first .. base + first + MOVE - 1
    int e_mine[kDispRounds];
    load_local_experts(topk_idx, expert_map, base, A, E, E_local, e_mine);  // whole chunk: thread t holds base + r*256 + t
    if (threadIdx.x < EXF_MAX_EXPERTS) pre[threadIdx.x] = 0;
    if constexpr (FUSED_SCAN) {
        __shared__ int col_total[EXF_MAX_EXPERTS], col_before[EXF_MAX_EXPERTS];
        if (threadIdx.x < EXF_MAX_EXPERTS) {
            col_total[threadIdx.x] = 0;
            col_before[threadIdx.x] = 0;
        }
        __syncthreads();
        const int n = n_coarse * E_local;
        const int mine = cc * E_local;  // entries below belong to earlier chunks
        constexpr int UL = 4;
        for (int i0 = threadIdx.x; i0 < n; i0 += kDispThreads * UL) {
            int c[UL];
#pragma unroll
            for (int u = 0; u < UL; ++u) c[u] = block_base[min(i0 + u * kDispThreads, n - 1)];
#pragma unroll
            for (int u = 0; u < UL; ++u) {
                const int i = i0 + u * kDispThreads;
                if (i < n && c[u] != 0) {
                    const int q = i % E_local;
                    atomicAdd(&col_total[q], c[u]);
                    if (i < mine) atomicAdd(&col_before[q], c[u]);
                }
            }
        }
        __syncthreads();
        if (wave == 0) {
            const int total = lane < E_local ? col_total[lane] : 0;
            const int incl = wave_inclusive_scan(total);
            if (lane < E_local) cursor[lane] = incl - total + col_before[lane];
            if (blockIdx.x == 0) {
                if (lane < E_local) {
                    expert_counts[lane] = total;
                    expert_offsets[lane] = incl - total;
                }
                if (lane == E_local - 1) expert_offsets[E_local] = incl;
            }
        }
    } else {
        if (threadIdx.x < E_local)
            cursor[threadIdx.x] = expert_offsets[threadIdx.x] + block_base[static_cast<int64_t>(cc) * E_local + threadIdx.x];
        __syncthreads();
    }
    // assignments of the chunk in front of the slice
#pragma unroll
    for (int r = 0; r < kDispRounds; ++r) {
        const int i = r * kDispThreads + static_cast<int>(threadIdx.x);
        if (i < first && e_mine[r] >= 0) atomicAdd(&pre[e_mine[r]], 1);
    }
    __syncthreads();

    // the slice sits in one round of one wavefront
    const int round_s = first / kDispThreads, wave_s = (first % kDispThreads) / kWave, lane_s = first % kWave;
    if (wave == wave_s) {
        int e = -1;
#pragma unroll
        for (int r = 0; r < kDispRounds; ++r)
            if (r == round_s) e = e_mine[r];
        const bool in_slice = lane >= lane_s && lane < lane_s + MOVE;
        if (!in_slice) e = -1;
        const unsigned long long below = (1ull << lane) - 1ull;
        const int rank = __popcll(same_expert_lanes(e, E_local) & below);
        if (in_slice) {
            const int64_t a = base + first + (lane - lane_s);
            int pos = -1;
            if (e >= 0) {
                pos = cursor[e] + pre[e] + rank;
                src_of_sorted[pos] = static_cast<int32_t>(a);
            }
            if (a < A) sorted_of_src[a] = pos;
            pos_s[lane - lane_s] = pos;
        }
    }
    __syncthreads();

    // ---- rows: wavefront w moves rows w*ROWS .. w*ROWS+ROWS-1 of the slice -----------------------
    constexpr int U = 4;
    int tok = 0, dst = -1;
    if (lane < ROWS) {
        const int j = wave * ROWS + lane;
        tok = static_cast<int>(min(base + first + j, A - 1) / k);
        dst = pos_s[j];
    }
    const float rcp = 1.0f / static_cast<float>(vec_per_row);
    const int total = ROWS * vec_per_row;
    constexpr int kPass = kWave * U;  // chunks the wavefront moves per pass
    const bool all_kept = __ballot(lane < ROWS && dst < 0) == 0ull;
    if (all_kept && total % kPass == 0) {
        const int n_pass = total / kPass;
        auto load_pass = [&](int pass, uint4(&v)[U]) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = pass * kPass + u * kWave + lane;
                const int r = row_of_chunk(c, vec_per_row, rcp);
                const int col = c - r * vec_per_row;
                const int t = __shfl(tok, r, kWave);
                v[u] = load_stream16(x + static_cast<int64_t>(t) * vec_per_row + col);
            }
        };
        auto store_pass = [&](int pass, const uint4(&v)[U]) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = pass * kPass + u * kWave + lane;
                const int r = row_of_chunk(c, vec_per_row, rcp);
                const int col = c - r * vec_per_row;
                const int p = __shfl(dst, r, kWave);
                store_stream16(x_sorted + static_cast<int64_t>(p) * vec_per_row + col, v[u]);
            }
        };
        uint4 cur[U], nxt[U];
        load_pass(0, cur);
        for (int pass = 0; pass + 1 < n_pass; ++pass) {
            load_pass(pass + 1, nxt);
            store_pass(pass, cur);
#pragma unroll
            for (int u = 0; u < U; ++u) cur[u] = nxt[u];
        }
        store_pass(n_pass - 1, cur);
        return;
    }
    for (int c0 = lane; c0 < total; c0 += kWave * U) {  // some row not kept, or a ragged chunk count: every chunk checked
        uint4 v[U];
        int p[U], col[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = c0 + u * kWave;
            const bool live = c < total;
            const int r = live ? row_of_chunk(c, vec_per_row, rcp) : 0;
            col[u] = c - r * vec_per_row;
            const int t = __shfl(tok, r, kWave);
            p[u] = live ? __shfl(dst, r, kWave) : -1;
            v[u] = p[u] >= 0 ? load_stream16(x + static_cast<int64_t>(t) * vec_per_row + col[u]) : uint4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (p[u] >= 0) store_stream16(x_sorted + static_cast<int64_t>(p[u]) * vec_per_row + col[u], v[u]);
    }
}

static int64_t dispatch_blocks(int64_t A) { return (A + kDispChunk - 1) / kDispChunk; }

}  // namespace exf

extern "C" size_t moe_dispatch_workspace_bytes(int64_t T, int k, int E_local)
{
    if (T < 0 || k < 1 || E_local < 1) return 0;
    const int64_t blocks = exf::dispatch_blocks(T * k);
    return exf::align_up(static_cast<size_t>(blocks > 0 ? blocks : 1) * static_cast<size_t>(E_local) * sizeof(int32_t), 256);
}

namespace exf {

// Validation and launches shared by moe_dispatch (chunk counts in the caller's workspace) and
// moe_dispatch_static (chunk counts in this library's own device array).
static int dispatch_run(const void* x, const int32_t* topk_idx, const int32_t* expert_map, int64_t T, int d, int k, int E, int E_local,
                        int dt, void* x_sorted, int32_t* src_of_sorted, int32_t* sorted_of_src, int32_t* expert_counts,
                        int32_t* expert_offsets, void* workspace, size_t workspace_bytes, void* stream)
{
    if (dt != EXF_F32 && dt != EXF_BF16) return fail(EXF_ERR_BAD_DTYPE, "moe_dispatch: dt = %d", dt);
    if (T < 0) return fail(EXF_ERR_BAD_SHAPE, "moe_dispatch: T = %lld < 0", static_cast<long long>(T));
    if (k < 1 || k > EXF_MAX_TOPK) return fail(EXF_ERR_BAD_SHAPE, "moe_dispatch: k = %d outside [1,%d]", k, EXF_MAX_TOPK);
    if (E < 1) return fail(EXF_ERR_BAD_SHAPE, "moe_dispatch: E = %d < 1", E);
    if (E_local < 1 || E_local > EXF_MAX_EXPERTS)
        return fail(EXF_ERR_BAD_SHAPE, "moe_dispatch: E_local = %d outside [1,%d]", E_local, EXF_MAX_EXPERTS);
    const int64_t A = T * k;
    if (A >= (1ll << 31)) return fail(EXF_ERR_BAD_SHAPE, "moe_dispatch: T*k must be below 2^31");
    const int gran = dt == EXF_BF16 ? 8 : 4;
    if (x_sorted != nullptr && (d < gran || d % gran != 0))
        return fail(EXF_ERR_BAD_SHAPE, "moe_dispatch: d = %d must be a positive multiple of %d", d, gran);
    EXF_REQUIRE_PTR(expert_counts);
    EXF_REQUIRE_PTR(expert_offsets);
    EXF_REQUIRE_PTR(workspace);
    if (workspace_bytes < moe_dispatch_workspace_bytes(T, k, E_local))
        return fail(EXF_ERR_WORKSPACE_TOO_SMALL, "moe_dispatch: workspace %zu < %zu bytes", workspace_bytes,
                    moe_dispatch_workspace_bytes(T, k, E_local));
    if (A > 0) {
        EXF_REQUIRE_PTR(topk_idx);
        EXF_REQUIRE_PTR(src_of_sorted);
        EXF_REQUIRE_PTR(sorted_of_src);
        if (x_sorted != nullptr) {
            EXF_REQUIRE_PTR(x);
            EXF_REQUIRE_ALIGNED(x);
            EXF_REQUIRE_ALIGNED(x_sorted);
        }
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    int32_t* block_counts = static_cast<int32_t*>(workspace);
    const int n_blocks = static_cast<int>(dispatch_blocks(A));
    if (A > 0 && x_sorted == nullptr && A <= static_cast<int64_t>(kSmallMaxRounds) * kSmallThreads) {
        // index maps of a short list: one launch, the workspace stays untouched
#define EXF_LAUNCH_SMALL(R)                                                                                                  \
    hipLaunchKernelGGL(dispatch_small_kernel<R>, dim3(1), dim3(kSmallThreads), 0, s, topk_idx, expert_map, A, E, E_local, \
                       expert_counts, expert_offsets, src_of_sorted, sorted_of_src)
        if (A <= 4 * kSmallThreads) EXF_LAUNCH_SMALL(4);
        else if (A <= 8 * kSmallThreads) EXF_LAUNCH_SMALL(8);
        else EXF_LAUNCH_SMALL(16);
#undef EXF_LAUNCH_SMALL
        return check_launch("moe_dispatch");
    }
    if (n_blocks > 0)
        hipLaunchKernelGGL(dispatch_count_kernel, dim3(n_blocks), dim3(kDispThreads), 0, s, topk_idx, expert_map, A, E, E_local,
                           block_counts);
    const bool fused = n_blocks > 0 && n_blocks <= kDispFusedScanBlocks;
    if (!fused)
        hipLaunchKernelGGL(dispatch_scan_kernel, dim3(1), dim3(kWave), 0, s, block_counts, n_blocks, E_local, expert_counts,
                           expert_offsets);
    if (n_blocks > 0) {
        if (x_sorted == nullptr) {  // index maps only
            if (fused)
                hipLaunchKernelGGL(dispatch_scatter_kernel<true>, dim3(n_blocks), dim3(kDispThreads), 0, s, topk_idx, expert_map, A, E,
                                   E_local, block_counts, expert_counts, expert_offsets, src_of_sorted, sorted_of_src);
            else
                hipLaunchKernelGGL(dispatch_scatter_kernel<false>, dim3(n_blocks), dim3(kDispThreads), 0, s, topk_idx, expert_map, A,
                                   E, E_local, block_counts, expert_counts, expert_offsets, src_of_sorted, sorted_of_src);
        } else {
            // index maps and rows in one launch; slices of 32 assignments while that still leaves few workgroups
            const int vec_per_row = d * (dt == EXF_BF16 ? 2 : 4) / 16;
            const bool small = (A + 63) / 64 < 512;
            const int move = small ? 32 : 64;
            const unsigned grid = static_cast<unsigned>((A + move - 1) / move);
            const uint4* xs = static_cast<const uint4*>(x);
            uint4* xd = static_cast<uint4*>(x_sorted);
#define EXF_LAUNCH_PLACE(FUSED, MOVE)                                                                                             \
    hipLaunchKernelGGL((dispatch_place_kernel<FUSED, MOVE>), dim3(grid), dim3(kDispThreads), 0, s, topk_idx, expert_map, A, E,     \
                       E_local, n_blocks, block_counts, expert_counts, expert_offsets, src_of_sorted, sorted_of_src, xs, k,       \
                       vec_per_row, xd)
            if (fused && small) EXF_LAUNCH_PLACE(true, 32);
            else if (fused) EXF_LAUNCH_PLACE(true, 64);
            else if (small) EXF_LAUNCH_PLACE(false, 32);
            else EXF_LAUNCH_PLACE(false, 64);
#undef EXF_LAUNCH_PLACE
        }
    }
    return check_launch("moe_dispatch");
}

// ---- the entry point that allocates nothing --------------------------------------------------
// Chunk counts of moe_dispatch_static: EXF_DISPATCH_STATIC_MAX_ASSIGNMENTS / 1024 chunks x 64 experts
// of int32 = 256 KiB, held by every GPU the library runs on until the process ends.  Host code must
// never pass the array's name to a kernel or a copy: the name is a host-side stand-in, the device
// address comes from hipGetSymbolAddress, once per device.
constexpr int64_t kStaticChunks = EXF_DISPATCH_STATIC_MAX_ASSIGNMENTS / kDispChunk;
static __device__ __align__(256) int32_t scratch[kStaticChunks * EXF_MAX_EXPERTS];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static int32_t* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up on the first call per device).
static int scratch_of_current_device(int32_t** out)
{
    int dev = -1;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return fail(EXF_ERR_HIP, "moe_dispatch_static: hipGetDevice: %s", hipGetErrorString(err));
    if (dev < 0 || dev >= kMaxDevices) return fail(EXF_ERR_HIP, "moe_dispatch_static: device %d outside [0,%d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (err != hipSuccess || p == nullptr)
            return fail(EXF_ERR_HIP, "moe_dispatch_static: hipGetSymbolAddress: %s", hipGetErrorString(err));
        g_scratch_ptr[dev] = static_cast<int32_t*>(p);
    }
    *out = g_scratch_ptr[dev];
    return EXF_OK;
}

}  // namespace exf

extern "C" int moe_dispatch(const void* x, const int32_t* topk_idx, const int32_t* expert_map, int64_t T, int d, int k, int E,
                            int E_local, int dt, void* x_sorted, int32_t* src_of_sorted, int32_t* sorted_of_src,
                            int32_t* expert_counts, int32_t* expert_offsets, void* workspace, size_t workspace_bytes,
                            void* stream)
{
    return exf::dispatch_run(x, topk_idx, expert_map, T, d, k, E, E_local, dt, x_sorted, src_of_sorted, sorted_of_src, expert_counts,
                             expert_offsets, workspace, workspace_bytes, stream);
}

extern "C" int moe_dispatch_static(const void* x, const int32_t* topk_idx, const int32_t* expert_map, int64_t T, int d, int k, int E,
                                   int E_local, int dt, void* x_sorted, int32_t* src_of_sorted, int32_t* sorted_of_src,
                                   int32_t* expert_counts, int32_t* expert_offsets, void* stream)
{
    using namespace exf;
    if (T < 0 || k < 1 || k > EXF_MAX_TOPK || T > EXF_DISPATCH_STATIC_MAX_ASSIGNMENTS || T * k > EXF_DISPATCH_STATIC_MAX_ASSIGNMENTS)
        return fail(EXF_ERR_BAD_SHAPE, "moe_dispatch_static: T*k = %lld*%d exceeds the %lld assignments the built-in scratch holds",
                    static_cast<long long>(T), k, static_cast<long long>(EXF_DISPATCH_STATIC_MAX_ASSIGNMENTS));
    if (E_local < 1 || E_local > EXF_MAX_EXPERTS)
        return fail(EXF_ERR_BAD_SHAPE, "moe_dispatch_static: E_local = %d outside [1,%d]", E_local, EXF_MAX_EXPERTS);
    int32_t* ptr = nullptr;
    const int rc = scratch_of_current_device(&ptr);
    if (rc != EXF_OK) return rc;
    // every entry of the count matrix that a launch reads is written by the count launch in front of
    // it, so nothing has to be cleared between calls
    return dispatch_run(x, topk_idx, expert_map, T, d, k, E, E_local, dt, x_sorted, src_of_sorted, sorted_of_src, expert_counts,
                        expert_offsets, ptr, sizeof(int32_t) * kStaticChunks * EXF_MAX_EXPERTS, stream);
}
