// affinity_histogram and placement_locality: reductions over a routing trace [L,N] (int32,
// layer-major).  Both are bound by the HBM read of the trace (4 bytes per token and layer).
//
// affinity_histogram
//   partial : a workgroup owns a chunk of tokens and a group of `g` consecutive layer pairs.
//             It keeps the g E x E histograms in LDS (replicated when E*E is small so that hot
//             bins do not serialise), walks the g+1 trace columns with the previous layer's ids
//             held in registers, bins every transition with an LDS atomic, and stores its
//             histograms as 32-bit partials.  Workgroups of one token chunk are mapped to one
//             XCD so that the column shared by neighbouring pair groups is served by that
//             XCD's L2.
//   finalize: one wavefront per (pair, source expert) row sums the partials over the chunks
//             into int64 counts, forms the row sum, the layer loads and the conditional
//             probabilities; a last small kernel derives the loads of the final layer.
//   Entries outside [0,E) are tallied; a transition touching one is not binned, but the valid
//   end still counts towards its layer's load through small "orphan" histograms.
//
// placement_locality
//   a workgroup owns a chunk of tokens for ALL layers (each trace entry is read exactly once),
//   maps expert -> device through an LDS copy of the placement, and counts per pair the tokens
//   whose device does not change; per-chunk partial counts are summed by a second kernel.
#include "common.hpp"

namespace exf {

constexpr int kXcds = 8;
constexpr int kAffThreads = 256;
constexpr int kAffSlots = 4;                                  // register-held token groups per thread
constexpr size_t kAffHistBudget = 48 * 1024;                  // LDS bytes for the pair histograms

struct AffinityPlan {
    int g;           // layer pairs per workgroup
    int Q;           // pair groups
    int copies;      // histogram replicas (power of two)
    int64_t chunk;   // tokens per workgroup
    int C;           // token chunks
    int vec;         // 4 if 16-byte trace loads are possible, else 1
    // workspace layout (32-bit words unless noted)
    size_t off_counts, off_orphan_next, off_orphan_last, off_invalid, total_bytes;
};

static AffinityPlan make_affinity_plan(int L, int64_t N, int E, bool aligned)
{
    AffinityPlan p;
    const int pairs = L > 1 ? L - 1 : 0;
    const size_t bins = static_cast<size_t>(E) * E;
    p.copies = 1;
    while (p.copies < 16 && bins * (p.copies * 2) <= 1024) p.copies *= 2;
    int g = static_cast<int>(kAffHistBudget / (bins * p.copies * sizeof(uint32_t)));
    if (g < 1) g = 1;
    if (g > 4) g = 4;
    if (pairs > 0 && g > pairs) g = pairs;
    p.g = g;
    p.Q = pairs > 0 ? (pairs + g - 1) / g : 1;
    p.vec = (aligned && N % 4 == 0) ? 4 : 1;
    // tokens per workgroup: at least one full sweep of the registers, at most what keeps the
    // partial-histogram traffic an order of magnitude below the trace itself.
    const int64_t sweep = static_cast<int64_t>(kAffThreads) * kAffSlots * p.vec;
    int64_t chunk = static_cast<int64_t>(bins) * 8;  // one partial bin is stored per 8 tokens binned
    if (chunk < sweep) chunk = sweep;
    chunk = (chunk + sweep - 1) / sweep * sweep;
    p.chunk = chunk;
    p.C = static_cast<int>(N > 0 ? (N + chunk - 1) / chunk : 0);
    size_t off = 0;
    p.off_counts = off;
    off += align_up(static_cast<size_t>(p.C) * pairs * bins * sizeof(uint32_t), 256);
    p.off_orphan_next = off;
    off += align_up(static_cast<size_t>(p.C) * (pairs > 0 ? pairs : 1) * E * sizeof(uint32_t), 256);
    p.off_orphan_last = off;
    off += align_up(static_cast<size_t>(p.C) * E * sizeof(uint32_t), 256);
    p.off_invalid = off;
    off += align_up(static_cast<size_t>(p.C) * p.Q * sizeof(uint32_t), 256);
    p.total_bytes = off > 0 ? off : 256;
    return p;
}

template <int VEC>
struct TokVec {
    int v[VEC];
};

template <int VEC>
__device__ __forceinline__ TokVec<VEC> load_tokens(const int32_t* __restrict__ col, int64_t n, int64_t end)
{
    TokVec<VEC> r;
    if constexpr (VEC == 4) {
        if (n + 3 < end) {
            const int4 q = *reinterpret_cast<const int4*>(col + n);
            r.v[0] = q.x;
            r.v[1] = q.y;
            r.v[2] = q.z;
            r.v[3] = q.w;
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u) r.v[u] = (n + u < end) ? col[n + u] : 0;
        }
    } else {
        r.v[0] = n < end ? col[n] : 0;
    }
    return r;
}

template <int VEC>
__global__ __launch_bounds__(kAffThreads) void affinity_partial_kernel(const int32_t* __restrict__ trace, int L, int64_t N, int E,
                                                                        int g, int Q, int copies, int64_t chunk, int C,
                                                                        uint32_t* __restrict__ part_counts,
                                                                        uint32_t* __restrict__ part_orphan_next,
                                                                        uint32_t* __restrict__ part_orphan_last,
                                                                        uint32_t* __restrict__ part_invalid)
{
    extern __shared__ uint32_t lds[];
    const int bins = E * E;
    uint32_t* hist = lds;                                 // [copies][g][bins]
    uint32_t* orphan_next = hist + copies * g * bins;     // [g][E]   valid id whose successor is invalid
    uint32_t* orphan_last = orphan_next + g * E;          // [E]      valid id of the final layer whose predecessor is invalid
    uint32_t* invalid_cnt = orphan_last + E;              // [1]

    // XCD-aware decomposition: consecutive workgroup ids are dealt round-robin to the XCDs, so
    // the XCD is blockIdx % 8; all pair groups of one token chunk are given to the same XCD.
    const int xcd = blockIdx.x % kXcds;
    const int j = blockIdx.x / kXcds;
    const int c = (j / Q) * kXcds + xcd;
    const int q = j % Q;
    if (c >= C) return;

    const int lds_words = copies * g * bins + g * E + E + 1;
    for (int i = threadIdx.x; i < lds_words; i += kAffThreads) lds[i] = 0u;
    __syncthreads();

    const int pairs = L - 1;
    const int l0 = q * g;                                  // first column of this group
    const int l1 = pairs > 0 ? min(l0 + g, pairs) : 0;     // last column (pairs l0 .. l1-1)
    const bool owns_last = (l1 == L - 1);
    const int64_t n_begin = static_cast<int64_t>(c) * chunk;
    const int64_t n_end = min(N, n_begin + chunk);
    uint32_t* my_hist = hist + (threadIdx.x & (copies - 1)) * g * bins;
    uint32_t invalid_local = 0;

    for (int64_t base = n_begin; base < n_end; base += static_cast<int64_t>(kAffThreads) * kAffSlots * VEC) {
        TokVec<VEC> prev[kAffSlots];
        int64_t n0[kAffSlots];
#pragma unroll
        for (int s = 0; s < kAffSlots; ++s) {
            n0[s] = base + (static_cast<int64_t>(s) * kAffThreads + threadIdx.x) * VEC;
            prev[s] = load_tokens<VEC>(trace + static_cast<int64_t>(l0) * N, n0[s], n_end);
        }
        for (int l = l0 + 1; l <= l1; ++l) {
            TokVec<VEC> cur[kAffSlots];
#pragma unroll
            for (int s = 0; s < kAffSlots; ++s) cur[s] = load_tokens<VEC>(trace + static_cast<int64_t>(l) * N, n0[s], n_end);
            uint32_t* h = my_hist + (l - 1 - l0) * bins;
            const bool last = (l == L - 1);
#pragma unroll
            for (int s = 0; s < kAffSlots; ++s) {
#pragma unroll
                for (int u = 0; u < VEC; ++u) {
                    if (n0[s] + u < n_end) {
                        const int a = prev[s].v[u];
                        const int b = cur[s].v[u];
                        const bool va = static_cast<unsigned>(a) < static_cast<unsigned>(E);
                        const bool vb = static_cast<unsigned>(b) < static_cast<unsigned>(E);
                        if (va && vb) {
                            atomicAdd(&h[a * E + b], 1u);
                        } else if (va) {
                            atomicAdd(&orphan_next[(l - 1 - l0) * E + a], 1u);
                        }
                        if (!va) invalid_local += 1;             // layer l-1 belongs to this group
                        if (last) {
                            if (!vb) invalid_local += 1;
                            else if (!va) atomicAdd(&orphan_last[b], 1u);
                        }
                    }
                    prev[s].v[u] = cur[s].v[u];
                }
            }
        }
        if (L == 1) {  // no pair at all: the single column only feeds loads and the invalid tally
#pragma unroll
            for (int s = 0; s < kAffSlots; ++s)
#pragma unroll
                for (int u = 0; u < VEC; ++u)
                    if (n0[s] + u < n_end) {
                        const int a = prev[s].v[u];
                        if (static_cast<unsigned>(a) < static_cast<unsigned>(E)) atomicAdd(&orphan_last[a], 1u);
                        else invalid_local += 1;
                    }
        }
    }
    if (invalid_local) atomicAdd(invalid_cnt, invalid_local);
    __syncthreads();

    // flush: sum the replicas, store 32-bit partials
    const int my_pairs = l1 - l0;
    for (int i = threadIdx.x; i < my_pairs * bins; i += kAffThreads) {
        uint32_t s = 0;
        for (int r = 0; r < copies; ++r) s += hist[r * g * bins + i];
        part_counts[(static_cast<size_t>(c) * pairs + l0) * bins + i] = s;
    }
    for (int i = threadIdx.x; i < my_pairs * E; i += kAffThreads)
        part_orphan_next[(static_cast<size_t>(c) * pairs + l0) * E + i] = orphan_next[i];
    if (owns_last || L == 1)
        for (int i = threadIdx.x; i < E; i += kAffThreads) part_orphan_last[static_cast<size_t>(c) * E + i] = orphan_last[i];
    if (threadIdx.x == 0) part_invalid[static_cast<size_t>(c) * Q + q] = *invalid_cnt;
}

// One wavefront per (pair l, source expert i): lane p sums bin (i,p) over the chunks.
__global__ __launch_bounds__(kWave) void affinity_finalize_kernel(const uint32_t* __restrict__ part_counts,
                                                                   const uint32_t* __restrict__ part_orphan_next, int C, int L,
                                                                   int E, int64_t* __restrict__ counts, int64_t* __restrict__ loads,
                                                                   float* __restrict__ cond_prob)
{
    const int pairs = L - 1;
    const int l = blockIdx.x / E;
    const int i = blockIdx.x % E;
    const int p = threadIdx.x;
    const size_t bins = static_cast<size_t>(E) * E;
    long long cnt = 0;
    if (p < E)
        for (int c = 0; c < C; ++c) cnt += part_counts[(static_cast<size_t>(c) * pairs + l) * bins + static_cast<size_t>(i) * E + p];
    const long long row = wave_sum(cnt);
    if (p < E) {
        const size_t o = (static_cast<size_t>(l) * E + i) * E + p;
        counts[o] = cnt;
        if (cond_prob != nullptr) cond_prob[o] = row > 0 ? static_cast<float>(static_cast<double>(cnt) / static_cast<double>(row)) : 0.0f;
    }
    if (loads != nullptr && p == 0) {
        long long orphan = 0;
        for (int c = 0; c < C; ++c) orphan += part_orphan_next[(static_cast<size_t>(c) * pairs + l) * E + i];
        loads[static_cast<size_t>(l) * E + i] = row + orphan;
    }
}

// loads of the final layer (column sums of the last pair + orphans) and the invalid tally.
__global__ __launch_bounds__(kWave) void affinity_tail_kernel(const uint32_t* __restrict__ part_orphan_last,
                                                               const uint32_t* __restrict__ part_invalid, int C, int Q, int L, int E,
                                                               const int64_t* __restrict__ counts, int64_t* __restrict__ loads,
                                                               int64_t* __restrict__ n_invalid)
{
    const int p = threadIdx.x;
    if (loads != nullptr && p < E) {
        long long s = 0;
        if (L > 1)
            for (int i = 0; i < E; ++i) s += counts[(static_cast<size_t>(L - 2) * E + i) * E + p];
        for (int c = 0; c < C; ++c) s += part_orphan_last[static_cast<size_t>(c) * E + p];
        loads[static_cast<size_t>(L - 1) * E + p] = s;
    }
    if (n_invalid != nullptr) {
        long long s = 0;
        for (int i = p; i < C * Q; i += kWave) s += part_invalid[i];
        s = wave_sum(s);
        if (p == 0) *n_invalid = s;
    }
}

// ------------------------------------------------------------------------------------------
constexpr int kLocThreads = 256;
constexpr int kLocSlots = 4;

template <int VEC>
__global__ __launch_bounds__(kLocThreads) void locality_partial_kernel(const int32_t* __restrict__ trace,
                                                                        const int32_t* __restrict__ placement, int L, int64_t N,
                                                                        int E, int64_t chunk, uint32_t* __restrict__ part)
{
    extern __shared__ int32_t lds_i[];
    int32_t* pl = lds_i;                                          // [L][E]
    uint32_t* pair_cnt = reinterpret_cast<uint32_t*>(lds_i + L * E);  // [L-1]
    for (int i = threadIdx.x; i < L * E; i += kLocThreads) pl[i] = placement[i];
    for (int i = threadIdx.x; i < L - 1; i += kLocThreads) pair_cnt[i] = 0u;
    __syncthreads();

    const int lane = lane_id();
    const int64_t n_begin = static_cast<int64_t>(blockIdx.x) * chunk;
    const int64_t n_end = min(N, n_begin + chunk);
    for (int64_t base = n_begin; base < n_end; base += static_cast<int64_t>(kLocThreads) * kLocSlots * VEC) {
        int dev_prev[kLocSlots][VEC];
        bool ok_prev[kLocSlots][VEC];
        int64_t n0[kLocSlots];
#pragma unroll
        for (int s = 0; s < kLocSlots; ++s) {
            n0[s] = base + (static_cast<int64_t>(s) * kLocThreads + threadIdx.x) * VEC;
            const TokVec<VEC> t = load_tokens<VEC>(trace, n0[s], n_end);
#pragma unroll
            for (int u = 0; u < VEC; ++u) {
                ok_prev[s][u] = (n0[s] + u < n_end) && static_cast<unsigned>(t.v[u]) < static_cast<unsigned>(E);
                dev_prev[s][u] = ok_prev[s][u] ? pl[t.v[u]] : 0;
            }
        }
        for (int l = 1; l < L; ++l) {
            TokVec<VEC> cur[kLocSlots];
#pragma unroll
            for (int s = 0; s < kLocSlots; ++s) cur[s] = load_tokens<VEC>(trace + static_cast<int64_t>(l) * N, n0[s], n_end);
            int same = 0;
#pragma unroll
            for (int s = 0; s < kLocSlots; ++s) {
#pragma unroll
                for (int u = 0; u < VEC; ++u) {
                    const bool ok = (n0[s] + u < n_end) && static_cast<unsigned>(cur[s].v[u]) < static_cast<unsigned>(E);
                    const int dev = ok ? pl[l * E + cur[s].v[u]] : 0;
                    same += (ok && ok_prev[s][u] && dev == dev_prev[s][u]) ? 1 : 0;
                    ok_prev[s][u] = ok;
                    dev_prev[s][u] = dev;
                }
            }
            same = wave_sum(same);
            if (lane == 0 && same != 0) atomicAdd(&pair_cnt[l - 1], static_cast<uint32_t>(same));
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < L - 1; i += kLocThreads) part[static_cast<size_t>(blockIdx.x) * (L - 1) + i] = pair_cnt[i];
}

__global__ __launch_bounds__(kWave) void locality_finalize_kernel(const uint32_t* __restrict__ part, int C, int pairs,
                                                                   int64_t* __restrict__ local_per_pair)
{
    const int l = blockIdx.x;
    long long s = 0;
    for (int c = threadIdx.x; c < C; c += kWave) s += part[static_cast<size_t>(c) * pairs + l];
    s = wave_sum(s);
    if (threadIdx.x == 0) local_per_pair[l] = s;
}

static int64_t locality_chunk(int64_t N, int vec)
{
    const int64_t sweep = static_cast<int64_t>(kLocThreads) * kLocSlots * vec;
    // aim at ~4 workgroups per CU, at least one register sweep each
    int64_t chunk = (N + 1023) / 1024;
    chunk = (chunk + sweep - 1) / sweep * sweep;
    return chunk < sweep ? sweep : chunk;
}

static int validate_trace_args(const char* fn, int L, int64_t N, int E)
{
    if (L < 1 || L > EXF_MAX_TRACE_LAYERS) return fail(EXF_ERR_BAD_SHAPE, "%s: L = %d outside [1,%d]", fn, L, EXF_MAX_TRACE_LAYERS);
    if (N < 0) return fail(EXF_ERR_BAD_SHAPE, "%s: N = %lld < 0", fn, static_cast<long long>(N));
    if (E < 1 || E > EXF_MAX_EXPERTS) return fail(EXF_ERR_BAD_SHAPE, "%s: E = %d outside [1,%d]", fn, E, EXF_MAX_EXPERTS);
    if (N >= (1ll << 40)) return fail(EXF_ERR_BAD_SHAPE, "%s: N must be below 2^40", fn);
    return EXF_OK;
}

}  // namespace exf

extern "C" size_t affinity_histogram_workspace_bytes(int L, int64_t N, int E)
{
    if (L < 1 || N < 0 || E < 1 || E > EXF_MAX_EXPERTS) return 0;
    // the aligned and unaligned plans differ only in chunk granularity; size for the larger one
    const size_t a = exf::make_affinity_plan(L, N, E, true).total_bytes;
    const size_t b = exf::make_affinity_plan(L, N, E, false).total_bytes;
    return a > b ? a : b;
}

extern "C" int affinity_histogram(const int32_t* trace, int L, int64_t N, int E, int64_t* counts, int64_t* loads,
                                  float* cond_prob, int64_t* n_invalid, void* workspace, size_t workspace_bytes, void* stream)
{
    using namespace exf;
    if (int rc = validate_trace_args("affinity_histogram", L, N, E)) return rc;
    if (N > 0) EXF_REQUIRE_PTR(trace);
    if (L > 1) EXF_REQUIRE_PTR(counts);
    EXF_REQUIRE_PTR(workspace);
    const AffinityPlan p = make_affinity_plan(L, N, E, aligned16(trace));
    if (workspace_bytes < p.total_bytes)
        return fail(EXF_ERR_WORKSPACE_TOO_SMALL, "affinity_histogram: workspace %zu < %zu bytes", workspace_bytes, p.total_bytes);
    hipStream_t s = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    uint32_t* part_counts = reinterpret_cast<uint32_t*>(ws + p.off_counts);
    uint32_t* part_orphan_next = reinterpret_cast<uint32_t*>(ws + p.off_orphan_next);
    uint32_t* part_orphan_last = reinterpret_cast<uint32_t*>(ws + p.off_orphan_last);
    uint32_t* part_invalid = reinterpret_cast<uint32_t*>(ws + p.off_invalid);
    if (p.C > 0) {
        const int c_pad = (p.C + kXcds - 1) / kXcds * kXcds;
        const unsigned grid = static_cast<unsigned>(c_pad) * p.Q;
        const size_t lds = (static_cast<size_t>(p.copies) * p.g * E * E + static_cast<size_t>(p.g) * E + E + 1) * sizeof(uint32_t);
        if (p.vec == 4)
            hipLaunchKernelGGL(affinity_partial_kernel<4>, dim3(grid), dim3(kAffThreads), lds, s, trace, L, N, E, p.g, p.Q, p.copies,
                               p.chunk, p.C, part_counts, part_orphan_next, part_orphan_last, part_invalid);
        else
            hipLaunchKernelGGL(affinity_partial_kernel<1>, dim3(grid), dim3(kAffThreads), lds, s, trace, L, N, E, p.g, p.Q, p.copies,
                               p.chunk, p.C, part_counts, part_orphan_next, part_orphan_last, part_invalid);
    }
    if (L > 1)
        hipLaunchKernelGGL(affinity_finalize_kernel, dim3(static_cast<unsigned>((L - 1) * E)), dim3(kWave), 0, s, part_counts,
                           part_orphan_next, p.C, L, E, counts, loads, cond_prob);
    if (loads != nullptr || n_invalid != nullptr)
        hipLaunchKernelGGL(affinity_tail_kernel, dim3(1), dim3(kWave), 0, s, part_orphan_last, part_invalid, p.C, p.Q, L, E, counts,
                           loads, n_invalid);
    return check_launch("affinity_histogram");
}

extern "C" size_t placement_locality_workspace_bytes(int L, int64_t N)
{
    if (L < 1 || N < 0) return 0;
    const int64_t chunk = exf::locality_chunk(N, 1);  // the scalar plan has the most chunks
    const int64_t C = N > 0 ? (N + chunk - 1) / chunk : 0;
    return exf::align_up(static_cast<size_t>(C > 0 ? C : 1) * static_cast<size_t>(L > 1 ? L - 1 : 1) * sizeof(uint32_t), 256);
}

extern "C" int placement_locality(const int32_t* trace, const int32_t* placement, int L, int64_t N, int E, int G,
                                  int64_t* local_per_pair, void* workspace, size_t workspace_bytes, void* stream)
{
    using namespace exf;
    if (int rc = validate_trace_args("placement_locality", L, N, E)) return rc;
    if (G < 1) return fail(EXF_ERR_BAD_SHAPE, "placement_locality: G = %d < 1", G);
    if (L == 1) return EXF_OK;  // no transition, no output element
    EXF_REQUIRE_PTR(placement);
    EXF_REQUIRE_PTR(local_per_pair);
    EXF_REQUIRE_PTR(workspace);
    if (N > 0) EXF_REQUIRE_PTR(trace);
    if (workspace_bytes < placement_locality_workspace_bytes(L, N))
        return fail(EXF_ERR_WORKSPACE_TOO_SMALL, "placement_locality: workspace %zu < %zu bytes", workspace_bytes,
                    placement_locality_workspace_bytes(L, N));
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int vec = (aligned16(trace) && N % 4 == 0) ? 4 : 1;
    const int64_t chunk = locality_chunk(N, vec);
    const int C = static_cast<int>(N > 0 ? (N + chunk - 1) / chunk : 0);
    uint32_t* part = static_cast<uint32_t*>(workspace);
    if (C > 0) {
        const size_t lds = (static_cast<size_t>(L) * E + (L - 1)) * sizeof(int32_t);
        if (vec == 4)
            hipLaunchKernelGGL(locality_partial_kernel<4>, dim3(C), dim3(kLocThreads), lds, s, trace, placement, L, N, E, chunk, part);
        else
            hipLaunchKernelGGL(locality_partial_kernel<1>, dim3(C), dim3(kLocThreads), lds, s, trace, placement, L, N, E, chunk, part);
    }
    hipLaunchKernelGGL(locality_finalize_kernel, dim3(L - 1), dim3(kWave), 0, s, part, C, L - 1, local_per_pair);
    return check_launch("placement_locality");
}
