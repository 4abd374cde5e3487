// moe_dispatch: stable counting sort of the token-to-expert assignments + row gather.
//
//   1. count   : every workgroup histograms its chunk of CH consecutive assignments into LDS
//                and stores one row of per-expert counts.
//   2. scan    : the [blocks x E_local] count matrix becomes per-chunk start positions (exclusive
//                scan down each expert column) plus expert_counts / expert_offsets.  Up to 256
//                chunks every scatter workgroup does this for itself from the small matrix; a
//                separate one-workgroup scan kernel serves longer inputs.
//   3. scatter : every workgroup ranks its chunk again — rank inside a wavefront from a ballot
//                per expert (lanes with a lower id and the same expert), wavefronts ordered
//                through LDS — which keeps equal experts in ascending assignment order
//                (stable, hence a unique permutation), and writes both index maps.
//   4. gather  : x_sorted[s] = x[src_of_sorted[s] / k] as 16-byte vector copies.
// No step needs the host to know a data-dependent size.
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
        rank[round] = 0;
        for (int q = 0; q < E_local; ++q) {
            const unsigned long long m = __ballot(e == q);
            if (e == q) rank[round] = __popcll(m & below);
            if (lane == q) wave_cnt[round][wave][q] = __popcll(m);
        }
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

// x_sorted[s] = x[src_of_sorted[s] / k] for the kept rows, in batches of `row_batch` (at most 16) sorted rows per
// wavefront: the lanes fetch the batch's source rows first, then the wavefront streams the batch
// as a flat sequence of 16-byte chunks (`vec_per_row` = row bytes / 16), four per lane in flight.
__global__ __launch_bounds__(256) void dispatch_gather_kernel(const uint4* __restrict__ x, const int32_t* __restrict__ src_of_sorted,
                                                               const int32_t* __restrict__ expert_offsets, int E_local, int k,
                                                               int vec_per_row, int64_t A, int row_batch, uint4* __restrict__ x_sorted)
{
    constexpr int U = 4;
    const int lane = lane_id();
    const int64_t kept = min(static_cast<int64_t>(max(expert_offsets[E_local], 0)), A);
    const int64_t n_batches = (kept + row_batch - 1) / row_batch;
    const int64_t n_waves = static_cast<int64_t>(gridDim.x) * (blockDim.x / kWave);
    const float rcp = 1.0f / static_cast<float>(vec_per_row);
    for (int64_t b = static_cast<int64_t>(blockIdx.x) * (blockDim.x / kWave) + threadIdx.x / kWave; b < n_batches; b += n_waves) {
        const int64_t s0 = b * row_batch;
        const int rows = static_cast<int>(min(static_cast<int64_t>(row_batch), kept - s0));
        const int src_row = lane < rows ? src_of_sorted[s0 + lane] / k : 0;
        const int total = rows * vec_per_row;
        constexpr int kPass = kWave * U;  // chunks the wavefront moves per pass
        if (total % kPass == 0) {
            // Every lane has a chunk in every pass: no condition anywhere near the loads, and the loads
            // of the next pass are issued before the stores of this one (with a branch around a load the
            // compiler waits for all outstanding memory operations at every pass).
            const int n_pass = total / kPass;
            auto load_pass = [&](int pass, uint4(&v)[U]) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int c = pass * kPass + u * kWave + lane;
                    const int r = row_of_chunk(c, vec_per_row, rcp);
                    const int col = c - r * vec_per_row;
                    const int t = __shfl(src_row, r, kWave);
                    v[u] = load_stream16(x + static_cast<int64_t>(t) * vec_per_row + col);
                }
            };
            auto store_pass = [&](int pass, const uint4(&v)[U]) {
#pragma unroll
                for (int u = 0; u < U; ++u) store_stream16(x_sorted + s0 * vec_per_row + pass * kPass + u * kWave + lane, v[u]);
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
            continue;
        }
        for (int c0 = lane; c0 < total; c0 += kWave * U) {  // ragged batch: every chunk checked
            uint4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = c0 + u * kWave;
                const bool live = c < total;
                const int r = live ? row_of_chunk(c, vec_per_row, rcp) : 0;
                const int col = c - r * vec_per_row;
                const int t = __shfl(src_row, r, kWave);
                v[u] = live ? load_stream16(x + static_cast<int64_t>(t) * vec_per_row + col) : uint4{0u, 0u, 0u, 0u};
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = c0 + u * kWave;
                if (c < total) store_stream16(x_sorted + s0 * vec_per_row + c, v[u]);
            }
        }
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

extern "C" int moe_dispatch(const void* x, const int32_t* topk_idx, const int32_t* expert_map, int64_t T, int d, int k, int E,
                            int E_local, int dt, void* x_sorted, int32_t* src_of_sorted, int32_t* sorted_of_src,
                            int32_t* expert_counts, int32_t* expert_offsets, void* workspace, size_t workspace_bytes,
                            void* stream)
{
    using namespace exf;
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
    if (n_blocks > 0)
        hipLaunchKernelGGL(dispatch_count_kernel, dim3(n_blocks), dim3(kDispThreads), 0, s, topk_idx, expert_map, A, E, E_local,
                           block_counts);
    const bool fused = n_blocks > 0 && n_blocks <= kDispFusedScanBlocks;
    if (!fused)
        hipLaunchKernelGGL(dispatch_scan_kernel, dim3(1), dim3(kWave), 0, s, block_counts, n_blocks, E_local, expert_counts,
                           expert_offsets);
    if (n_blocks > 0) {
        if (fused)
            hipLaunchKernelGGL(dispatch_scatter_kernel<true>, dim3(n_blocks), dim3(kDispThreads), 0, s, topk_idx, expert_map, A, E,
                               E_local, block_counts, expert_counts, expert_offsets, src_of_sorted, sorted_of_src);
        else
            hipLaunchKernelGGL(dispatch_scatter_kernel<false>, dim3(n_blocks), dim3(kDispThreads), 0, s, topk_idx, expert_map, A, E,
                               E_local, block_counts, expert_counts, expert_offsets, src_of_sorted, sorted_of_src);
        if (x_sorted != nullptr) {
            const int vec_per_row = d * (dt == EXF_BF16 ? 2 : 4) / 16;
            const int row_batch = row_batch_for(A);
            int64_t blocks = ((A + row_batch - 1) / row_batch + 3) / 4;  // four wavefronts (row batches) per workgroup
            if (blocks > kStreamWorkgroups) blocks = kStreamWorkgroups;
            if (blocks < 1) blocks = 1;
            hipLaunchKernelGGL(dispatch_gather_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, s,
                               static_cast<const uint4*>(x), src_of_sorted, expert_offsets, E_local, k, vec_per_row, A, row_batch,
                               static_cast<uint4*>(x_sorted));
        }
    }
    return check_launch("moe_dispatch");
}
