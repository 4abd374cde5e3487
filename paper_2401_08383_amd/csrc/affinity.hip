// affinity_histogram and placement_locality: reductions over a routing trace [L,N] (int32,
// layer-major).  Both are bound by the HBM read of the trace (4 bytes per token and layer), so
// both are shaped like a streaming read: about one 1024-thread workgroup per CU, every thread
// keeping several 16-byte loads in flight.
//
// affinity_histogram
//   partial : a workgroup owns a chunk of tokens (< 65536) and a group of g <= 3 consecutive
//             layer pairs.  A thread loads the g+1 trace columns of its tokens at once, then walks
//             the pairs and bins every transition with one LDS atomic.  The g E x E histograms
//             live in LDS as 16-bit counters packed two to a word (a workgroup can never count
//             more than its chunk, so they cannot overflow), replicated when E*E is small so that
//             hot bins do not serialise.  The packed words are stored as per-chunk partials.
//             Workgroups of one token chunk are mapped to one XCD, so the column shared by two
//             neighbouring pair groups is served by that XCD's L2.
//   finalize: one wavefront per (pair, source expert) row sums the partials over the chunks
//             into int64 counts, forms the row sum (a wavefront reduction: no LDS, no barrier), the
//             layer loads and the conditional probabilities; extra workgroups of the same launch
//             derive the loads of the final layer and the invalid tally.
//   Entries outside [0,E) are tallied; a transition touching one is not binned, but the valid
//   end still counts towards its layer's load through small "orphan" histograms.
//
// placement_locality
//   a workgroup owns a chunk of tokens for ALL layers (each trace entry is read exactly once),
//   maps expert -> device through an LDS copy of the placement, keeps the loads of four layers in
//   flight, and counts per pair the tokens whose device does not change; per-chunk partial counts
//   are summed by a second kernel.
#include "common.hpp"

namespace exf {

constexpr int kXcds = 8;
constexpr int kTraceThreads = 1024;
constexpr int kAffMaxGroup = 3;                 // layer pairs per workgroup (4 columns in registers; 3 measured best,
                                                // 29 against 34 us with 6 on a 24 x 1M trace)
constexpr size_t kAffHistBudget = 48 * 1024;    // LDS bytes for the packed pair histograms
constexpr int64_t kAffMaxChunk = 61440;         // tokens per workgroup: 16-bit counters cannot overflow
constexpr int kTargetWorkgroups = 256;          // about one per CU

struct AffinityPlan {
    int g;           // layer pairs per workgroup
    int Q;           // pair groups
    int copies;      // histogram replicas (power of two)
    int words;       // 32-bit words of one packed E x E histogram
    int64_t chunk;   // tokens per workgroup
    int C;           // token chunks
    int vec;         // 4 if 16-byte trace loads are possible, else 1
    size_t off_counts, off_orphan_next, off_orphan_last, off_invalid, off_local, total_bytes;
};

static AffinityPlan make_affinity_plan(int L, int64_t N, int E, bool aligned)
{
    AffinityPlan p;
    const int pairs = L > 1 ? L - 1 : 0;
    p.words = (E * E + 1) / 2;
    const size_t hist_bytes = static_cast<size_t>(p.words) * sizeof(uint32_t);
    int g = static_cast<int>(kAffHistBudget / hist_bytes);
    if (g > kAffMaxGroup) g = kAffMaxGroup;
    if (g < 1) g = 1;
    if (pairs > 0 && g > pairs) g = pairs;
    p.g = g;
    p.copies = 1;
    while (p.copies < 16 && hist_bytes * g * (p.copies * 2) <= kAffHistBudget) p.copies *= 2;
    p.Q = pairs > 0 ? (pairs + g - 1) / g : 1;
    p.vec = (aligned && N % 4 == 0) ? 4 : 1;
    const int64_t sweep = static_cast<int64_t>(kTraceThreads) * p.vec;  // tokens one pass of the workgroup covers
    int c_target = kTargetWorkgroups / p.Q;
    if (c_target < 1) c_target = 1;
    int64_t chunk = (N + c_target - 1) / c_target;
    chunk = (chunk + sweep - 1) / sweep * sweep;
    if (chunk < sweep) chunk = sweep;
    if (chunk > kAffMaxChunk) chunk = kAffMaxChunk / sweep * sweep;
    p.chunk = chunk;
    p.C = static_cast<int>(N > 0 ? (N + chunk - 1) / chunk : 0);
    size_t off = 0;
    p.off_counts = off;
    off += align_up(static_cast<size_t>(p.C) * pairs * p.words * sizeof(uint32_t), 256);
    p.off_orphan_next = off;
    off += align_up(static_cast<size_t>(p.C) * (pairs > 0 ? pairs : 1) * E * sizeof(uint32_t), 256);
    p.off_orphan_last = off;
    off += align_up(static_cast<size_t>(p.C) * E * sizeof(uint32_t), 256);
    p.off_invalid = off;
    off += align_up(static_cast<size_t>(p.C) * p.Q * sizeof(uint32_t), 256);
    p.off_local = off;  // per chunk and pair: transitions that stay on their device (affinity_statistics)
    off += align_up(static_cast<size_t>(p.C) * (pairs > 0 ? pairs : 1) * sizeof(uint32_t), 256);
    p.total_bytes = off > 0 ? off : 256;
    return p;
}

template <int VEC>
struct TokVec {
    int v[VEC];
};

// Loads the ids of tokens n .. n+VEC-1 of one trace column.  The load is UNCONDITIONAL: a lane past
// the end of its chunk re-reads the chunk's last vector (the caller masks such lanes through its own
// range test).  Keeping branches away from the loads matters: with a branch around each of them the
// compiler can no longer count the loads in flight and waits for all earlier ones before every new
// one, which leaves a single load in flight per wavefront.  With VEC = 4 the column base, n and end
// are multiples of four, so a vector is never cut by the end of the chunk.
template <int VEC>
__device__ __forceinline__ TokVec<VEC> load_tokens(const int32_t* __restrict__ col, int64_t n, int64_t end)
{
    TokVec<VEC> r;
    const int64_t n_safe = min(n, end - VEC);  // callers guarantee end - begin >= VEC
    if constexpr (VEC == 4) {
        typedef __attribute__((__vector_size__(4 * sizeof(int)))) int i32x4_v;
        const i32x4_v q = __builtin_nontemporal_load(reinterpret_cast<const i32x4_v*>(col + n_safe));  // streamed once
        r.v[0] = q[0];
        r.v[1] = q[1];
        r.v[2] = q[2];
        r.v[3] = q[3];
    } else {
        r.v[0] = __builtin_nontemporal_load(col + n_safe);
    }
    return r;
}

template <int VEC>
__global__ __launch_bounds__(kTraceThreads) void affinity_partial_kernel(const int32_t* __restrict__ trace, int L, int64_t N, int E,
                                                                          int g, int Q, int copies, int words, int64_t chunk, int C,
                                                                          uint32_t* __restrict__ part_counts,
                                                                          uint32_t* __restrict__ part_orphan_next,
                                                                          uint32_t* __restrict__ part_orphan_last,
                                                                          uint32_t* __restrict__ part_invalid,
                                                                          const int32_t* __restrict__ placement,  // [L,E] or null
                                                                          uint32_t* __restrict__ part_local)      // with placement
{
    extern __shared__ uint32_t lds[];
    uint32_t* hist = lds;                                 // [copies][g][words], two 16-bit counters per word
    uint32_t* orphan_next = hist + copies * g * words;    // [g][E]   valid id whose successor is invalid
    uint32_t* orphan_last = orphan_next + g * E;          // [E]      valid id of the final layer whose predecessor is invalid
    uint32_t* invalid_cnt = orphan_last + E;              // [1]
    uint32_t* stay_cnt = invalid_cnt + 1;                 // [g]      transitions whose two experts share a device
    int32_t* device = reinterpret_cast<int32_t*>(stay_cnt + g);  // [g+1][E] placement rows of this group's layers

    // XCD-aware decomposition: consecutive workgroup ids are dealt round-robin to the XCDs, so
    // the XCD is blockIdx % 8; all pair groups of one token chunk are given to the same XCD.
    const int xcd = blockIdx.x % kXcds;
    const int j = blockIdx.x / kXcds;
    const int c = (j / Q) * kXcds + xcd;
    const int q = j % Q;
    if (c >= C) return;

    const int lds_words = copies * g * words + g * E + E + 1 + g;
    for (int i = threadIdx.x; i < lds_words; i += kTraceThreads) lds[i] = 0u;
    const int pairs = L - 1;
    const int l0 = q * g;                                  // first column of this group
    const int l1 = pairs > 0 ? min(l0 + g, pairs) : 0;     // last column (pairs l0 .. l1-1)
    if (placement != nullptr)
        for (int i = threadIdx.x; i < (l1 - l0 + 1) * E; i += kTraceThreads) device[i] = placement[l0 * E + i];
    __syncthreads();

    const bool owns_last = (l1 == L - 1);
    const int64_t n_begin = static_cast<int64_t>(c) * chunk;
    const int64_t n_end = min(N, n_begin + chunk);
    uint32_t* my_hist = hist + (threadIdx.x & (copies - 1)) * g * words;
    uint32_t invalid_local = 0;

    // Software pipeline over the sweeps of the chunk: the (up to four) 16-byte column loads of the
    // NEXT sweep are issued before the current sweep is binned, so that the memory system is never
    // idle while the LDS atomics run.
    const int64_t sweep = static_cast<int64_t>(kTraceThreads) * VEC;
    // (columns past the group's last one and sweeps past the chunk's end are clamped, not skipped:
    // the loads stay free of branches, the duplicates are cache hits)
    auto load_cols = [&](int64_t n0, TokVec<VEC>(&col)[kAffMaxGroup + 1]) {
#pragma unroll
        for (int s = 0; s <= kAffMaxGroup; ++s)
            col[s] = load_tokens<VEC>(trace + static_cast<int64_t>(min(l0 + s, l1)) * N, n0, n_end);
    };
    TokVec<VEC> col[kAffMaxGroup + 1], nxt[kAffMaxGroup + 1];
    load_cols(n_begin + static_cast<int64_t>(threadIdx.x) * VEC, col);
    for (int64_t base = n_begin; base < n_end; base += sweep) {
        const int64_t n0 = base + static_cast<int64_t>(threadIdx.x) * VEC;
        load_cols(n0 + sweep, nxt);
        // Fast path (the normal case): every id this wavefront holds in the sweep is inside [0,E) and
        // no lane is past the end of the chunk - one multiply-add, a shift and one LDS atomic per
        // transition.  Anything else goes through the fully checked path below.
        bool clean = n0 + VEC <= n_end;
#pragma unroll
        for (int s = 0; s <= kAffMaxGroup; ++s) {
            if (l0 + s > l1 && s != 0) break;
            unsigned m = 0;
#pragma unroll
            for (int u = 0; u < VEC; ++u) m = max(m, static_cast<unsigned>(col[s].v[u]));
            clean = clean && m < static_cast<unsigned>(E);
        }
        if (__ballot(!clean) == 0ull && L > 1) {
#pragma unroll
            for (int s = 1; s <= kAffMaxGroup; ++s) {
                if (l0 + s > l1) break;
                uint32_t* h = my_hist + (s - 1) * words;
#pragma unroll
                for (int u = 0; u < VEC; ++u) {
                    const int bin = col[s - 1].v[u] * E + col[s].v[u];
                    atomicAdd(&h[bin >> 1], 1u << ((bin & 1) * 16));
                }
            }
        } else {
#pragma unroll
        for (int s = 1; s <= kAffMaxGroup; ++s) {
            const int l = l0 + s;
            if (l > l1) break;
            uint32_t* h = my_hist + (s - 1) * words;
            const bool last = (l == L - 1);
#pragma unroll
            for (int u = 0; u < VEC; ++u) {
                if (n0 + u < n_end) {
                    const int a = col[s - 1].v[u];
                    const int b = col[s].v[u];
                    const bool va = static_cast<unsigned>(a) < static_cast<unsigned>(E);
                    const bool vb = static_cast<unsigned>(b) < static_cast<unsigned>(E);
                    if (va && vb) {
                        const int bin = a * E + b;
                        atomicAdd(&h[bin >> 1], (bin & 1) ? 0x10000u : 1u);
                    } else if (va) {
                        atomicAdd(&orphan_next[(s - 1) * E + a], 1u);
                    }
                    if (!va) invalid_local += 1;  // layer l-1 belongs to this group
                    if (last) {
                        if (!vb) invalid_local += 1;
                        else if (!va) atomicAdd(&orphan_last[b], 1u);
                    }
                }
            }
        }
        }
        if (L == 1) {  // no pair at all: the single column only feeds loads and the invalid tally
#pragma unroll
            for (int u = 0; u < VEC; ++u)
                if (n0 + u < n_end) {
                    const int a = col[0].v[u];
                    if (static_cast<unsigned>(a) < static_cast<unsigned>(E)) atomicAdd(&orphan_last[a], 1u);
                    else invalid_local += 1;
                }
        }
#pragma unroll
        for (int s = 0; s <= kAffMaxGroup; ++s) col[s] = nxt[s];
    }
    if (invalid_local) atomicAdd(invalid_cnt, invalid_local);
    __syncthreads();

    // flush: sum the replicas (packed halves cannot carry: a bin holds at most `chunk` < 65536); with a
    // placement, also count per pair the transitions of the bins whose two experts share a device
    const int my_pairs = l1 - l0;
    for (int i = threadIdx.x; i < my_pairs * words; i += kTraceThreads) {
        uint32_t s = 0;
        for (int r = 0; r < copies; ++r) s += hist[r * g * words + i];
        part_counts[(static_cast<size_t>(c) * pairs + l0) * words + i] = s;
        if (placement != nullptr) {
            const int pr = i / words, wd = i - pr * words;
            const int32_t* here = device + pr * E;
            const int32_t* there = here + E;
            uint32_t stay = 0;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int bin = 2 * wd + h;
                if (bin < E * E && here[bin / E] == there[bin % E]) stay += (s >> (16 * h)) & 0xffffu;
            }
            if (stay != 0) atomicAdd(&stay_cnt[pr], stay);
        }
    }
    if (placement != nullptr) {
        __syncthreads();
        if (static_cast<int>(threadIdx.x) < my_pairs) part_local[static_cast<size_t>(c) * pairs + l0 + threadIdx.x] = stay_cnt[threadIdx.x];
    }
    for (int i = threadIdx.x; i < my_pairs * E; i += kTraceThreads)
        part_orphan_next[(static_cast<size_t>(c) * pairs + l0) * E + i] = orphan_next[i];
    if (owns_last || L == 1)
        for (int i = threadIdx.x; i < E; i += kTraceThreads) part_orphan_last[static_cast<size_t>(c) * E + i] = orphan_last[i];
    if (threadIdx.x == 0) part_invalid[static_cast<size_t>(c) * Q + q] = *invalid_cnt;
}

// Counts for EVERY ordered layer pair l < m (the appendix statistic), pairs numbered source layer
// first.  A workgroup owns a chunk of tokens and a group (l; m0 .. m0+g-1): it loads column l and
// the g target columns and bins (col l, col m) - the same four-columns-for-three-pairs economy as
// the one-hop kernel.  Groups are numbered q = 0 .. Q-1 in pair order; transitions with an invalid
// end are skipped; the packed per-chunk partials go to part_counts[chunk][pair][words].
template <int VEC>
__global__ __launch_bounds__(kTraceThreads) void multihop_partial_kernel(const int32_t* __restrict__ trace, int L, int64_t N, int E,
                                                                          int g, int Q, int copies, int words, int64_t chunk, int C,
                                                                          uint32_t* __restrict__ part_counts)
{
    extern __shared__ uint32_t lds[];
    uint32_t* hist = lds;  // [copies][g][words], two 16-bit counters per word
    const int xcd = blockIdx.x % kXcds;
    const int j = blockIdx.x / kXcds;
    const int c = (j / Q) * kXcds + xcd;
    const int q = j % Q;
    if (c >= C) return;
    for (int i = threadIdx.x; i < copies * g * words; i += kTraceThreads) lds[i] = 0u;
    __syncthreads();

    // group q -> source layer l, first target m0, number of pairs
    int l = 0, before = 0, pair_base = 0;
    for (;; ++l) {
        const int targets = L - 1 - l;
        const int groups = (targets + g - 1) / g;
        if (q < before + groups) break;
        before += groups;
        pair_base += targets;
    }
    const int m0 = l + 1 + (q - before) * g;
    const int my_pairs = min(g, L - m0);
    pair_base += m0 - (l + 1);
    const int total_pairs = L * (L - 1) / 2;

    const int64_t n_begin = static_cast<int64_t>(c) * chunk;
    const int64_t n_end = min(N, n_begin + chunk);
    uint32_t* my_hist = hist + (threadIdx.x & (copies - 1)) * g * words;
    const int64_t sweep = static_cast<int64_t>(kTraceThreads) * VEC;
    auto load_cols = [&](int64_t n0, TokVec<VEC>(&col)[kAffMaxGroup + 1]) {  // clamped, never skipped
        col[0] = load_tokens<VEC>(trace + static_cast<int64_t>(l) * N, n0, n_end);
#pragma unroll
        for (int s = 1; s <= kAffMaxGroup; ++s)
            col[s] = load_tokens<VEC>(trace + static_cast<int64_t>(min(m0 + s - 1, L - 1)) * N, n0, n_end);
    };
    TokVec<VEC> col[kAffMaxGroup + 1], nxt[kAffMaxGroup + 1];
    load_cols(n_begin + static_cast<int64_t>(threadIdx.x) * VEC, col);
    for (int64_t base = n_begin; base < n_end; base += sweep) {
        const int64_t n0 = base + static_cast<int64_t>(threadIdx.x) * VEC;
        load_cols(n0 + sweep, nxt);
        bool clean = n0 + VEC <= n_end;
#pragma unroll
        for (int s = 0; s <= kAffMaxGroup; ++s) {
            unsigned m = 0;
#pragma unroll
            for (int u = 0; u < VEC; ++u) m = max(m, static_cast<unsigned>(col[s].v[u]));
            clean = clean && m < static_cast<unsigned>(E);  // (clamped duplicate columns repeat a checked one)
        }
        if (__ballot(!clean) == 0ull) {
#pragma unroll
            for (int s = 1; s <= kAffMaxGroup; ++s) {
                if (s > my_pairs) break;
                uint32_t* h = my_hist + (s - 1) * words;
#pragma unroll
                for (int u = 0; u < VEC; ++u) {
                    const int bin = col[0].v[u] * E + col[s].v[u];
                    atomicAdd(&h[bin >> 1], 1u << ((bin & 1) * 16));
                }
            }
        } else {
#pragma unroll
            for (int s = 1; s <= kAffMaxGroup; ++s) {
                if (s > my_pairs) break;
                uint32_t* h = my_hist + (s - 1) * words;
#pragma unroll
                for (int u = 0; u < VEC; ++u) {
                    const int a = col[0].v[u], b = col[s].v[u];
                    if (n0 + u < n_end && static_cast<unsigned>(a) < static_cast<unsigned>(E) &&
                        static_cast<unsigned>(b) < static_cast<unsigned>(E)) {
                        const int bin = a * E + b;
                        atomicAdd(&h[bin >> 1], (bin & 1) ? 0x10000u : 1u);
                    }
                }
            }
        }
#pragma unroll
        for (int s = 0; s <= kAffMaxGroup; ++s) col[s] = nxt[s];
    }
    __syncthreads();
    for (int i = threadIdx.x; i < my_pairs * words; i += kTraceThreads) {
        uint32_t sum = 0;
        for (int r = 0; r < copies; ++r) sum += hist[r * g * words + i];
        part_counts[(static_cast<size_t>(c) * total_pairs + pair_base) * words + i] = sum;
    }
}

// Workgroups of 256 threads.  The first ceil((L-1)*E / 4) give every wavefront one (pair l, source
// expert i) row: lane p sums bin (i, p) over all chunks (16 independent loads in flight), the row sum
// is a wavefront reduction -> counts, load of (l, i), conditional probabilities; nothing goes through
// LDS and no workgroup barrier is needed.  The next E workgroups take one
// expert p of the FINAL layer each: its load is the column sum of the last pair (taken from the
// partials, so that no result of another workgroup is needed) plus the orphans.  One workgroup
// adds up the invalid tally.  With a placement, L-1 more workgroups form the locality numerators.
constexpr int kFinRowsPerWorkgroup = 4;
__global__ __launch_bounds__(256) void affinity_finalize_kernel(const uint32_t* __restrict__ part_counts,
                                                                const uint32_t* __restrict__ part_orphan_next,
                                                                const uint32_t* __restrict__ part_orphan_last,
                                                                const uint32_t* __restrict__ part_invalid, int C, int Q, int L, int E,
                                                                int words, int64_t* __restrict__ counts, int64_t* __restrict__ loads,
                                                                float* __restrict__ cond_prob, int64_t* __restrict__ n_invalid,
                                                                const uint32_t* __restrict__ part_local,  // [C][L-1] or null
                                                                int64_t* __restrict__ local)              // [L-1] (with part_local)
{
    __shared__ long long orphan_red[4];
    const int pairs = L - 1;
    const int p = lane_id();
    const int w = threadIdx.x / kWave;
    const int rows = pairs * E;
    const int row_blocks = (rows + kFinRowsPerWorkgroup - 1) / kFinRowsPerWorkgroup;
    if (static_cast<int>(blockIdx.x) < row_blocks) {
        const int row = static_cast<int>(blockIdx.x) * kFinRowsPerWorkgroup + w;
        if (row >= rows) return;  // (whole wavefronts; no barrier follows)
        const int l = row / E;
        const int i = row % E;
        long long cnt = 0;
        if (p < E) {
            const int bin = i * E + p;
            const int shift = (bin & 1) * 16;
            const uint32_t* src = part_counts + static_cast<size_t>(l) * words + (bin >> 1);
            const size_t step = static_cast<size_t>(pairs) * words;
            // 16 independent loads in flight (clamped, never branched around)
            for (int c0 = 0; c0 < C; c0 += 16) {
                uint32_t v[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) v[u] = src[min(c0 + u, C - 1) * step];
#pragma unroll
                for (int u = 0; u < 16; ++u)
                    if (c0 + u < C) cnt += (v[u] >> shift) & 0xffffu;
            }
        }
        long long orphan = 0;
        if (loads != nullptr)  // (the multi-hop statistic has no orphan tallies)
            for (int c = p; c < C; c += kWave) orphan += part_orphan_next[(static_cast<size_t>(c) * pairs + l) * E + i];
        orphan = wave_sum(orphan);
        const long long row_sum = wave_sum(cnt);
        if (p < E) {
            const size_t o = (static_cast<size_t>(l) * E + i) * E + p;
            counts[o] = cnt;
            if (cond_prob != nullptr)
                cond_prob[o] = row_sum > 0 ? static_cast<float>(static_cast<double>(cnt) / static_cast<double>(row_sum)) : 0.0f;
        }
        if (loads != nullptr && p == 0) loads[static_cast<size_t>(l) * E + i] = row_sum + orphan;
    } else if (static_cast<int>(blockIdx.x) < row_blocks + E) {
        if (loads == nullptr) return;
        const int pe = blockIdx.x - row_blocks;  // expert of the final layer
        long long s = 0;
        if (pairs > 0) {  // column pe of the last pair: sum over chunks c and source experts i
            const int total = C * E;
            for (int j0 = threadIdx.x; j0 < total; j0 += 256 * 8) {
                uint32_t v[8];
                int sh[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int j = min(j0 + 256 * u, total - 1);
                    const int c = j / E, i = j - c * E;
                    const int bin = i * E + pe;
                    sh[u] = (bin & 1) * 16;
                    v[u] = part_counts[(static_cast<size_t>(c) * pairs + (pairs - 1)) * words + (bin >> 1)];
                }
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (j0 + 256 * u < total) s += (v[u] >> sh[u]) & 0xffffu;
            }
        }
        for (int c = threadIdx.x; c < C; c += 256) s += part_orphan_last[static_cast<size_t>(c) * E + pe];
        s = wave_sum(s);
        if (p == 0) orphan_red[w] = s;
        __syncthreads();
        if (threadIdx.x == 0) loads[static_cast<size_t>(L - 1) * E + pe] = orphan_red[0] + orphan_red[1] + orphan_red[2] + orphan_red[3];
    } else if (static_cast<int>(blockIdx.x) == row_blocks + E) {
        if (n_invalid == nullptr) return;
        long long inv = 0;
        for (int i = threadIdx.x; i < C * Q; i += 256) inv += part_invalid[i];
        inv = wave_sum(inv);
        if (p == 0) orphan_red[w] = inv;
        __syncthreads();
        if (threadIdx.x == 0) *n_invalid = orphan_red[0] + orphan_red[1] + orphan_red[2] + orphan_red[3];
    } else {
        // locality numerator of pair l: the per-chunk counts of the first launch added up
        if (part_local == nullptr) return;
        const int l = blockIdx.x - (row_blocks + E + 1);
        long long stay = 0;
        for (int c = threadIdx.x; c < C; c += 256) stay += part_local[static_cast<size_t>(c) * pairs + l];
        stay = wave_sum(stay);
        if (p == 0) orphan_red[w] = stay;
        __syncthreads();
        if (threadIdx.x == 0) local[l] = orphan_red[0] + orphan_red[1] + orphan_red[2] + orphan_red[3];
    }
}

// ------------------------------------------------------------------------------------------
constexpr int kLocAhead = 2;  // trace layers whose loads are in flight together

// HOME: additionally counts, per layer, the tokens whose expert sits on another device than
// home[n] (the device that owns the token's request); the per-chunk partials then hold the L-1 pair
// counts followed by the L away counts.
template <int VEC, bool HOME>
__global__ __launch_bounds__(kTraceThreads) void locality_partial_kernel(const int32_t* __restrict__ trace,
                                                                          const int32_t* __restrict__ placement,
                                                                          const int32_t* __restrict__ home, int L, int64_t N, int E,
                                                                          int64_t chunk, uint32_t* __restrict__ part)
{
    extern __shared__ int32_t lds_i[];
    int32_t* pl = lds_i;                                              // [L][E]
    uint32_t* pair_cnt = reinterpret_cast<uint32_t*>(lds_i + L * E);  // [L-1] pairs, then (HOME) [L] away counts
    uint32_t* away_cnt = pair_cnt + (L - 1);
    const int n_out = (L - 1) + (HOME ? L : 0);
    for (int i = threadIdx.x; i < L * E; i += kTraceThreads) pl[i] = placement[i];
    for (int i = threadIdx.x; i < n_out; i += kTraceThreads) pair_cnt[i] = 0u;
    __syncthreads();

    const int lane = lane_id();
    const int64_t n_begin = static_cast<int64_t>(blockIdx.x) * chunk;
    const int64_t n_end = min(N, n_begin + chunk);
    for (int64_t base = n_begin; base < n_end; base += static_cast<int64_t>(kTraceThreads) * VEC) {
        const int64_t n0 = base + static_cast<int64_t>(threadIdx.x) * VEC;
        int dev_prev[VEC];
        bool ok_prev[VEC];
        const bool in_range = n0 + VEC <= n_end;  // all tokens of this lane exist
        bool prev_clean;                           // all ids of the previous layer valid (and in range)
        TokVec<VEC> hm;
        if constexpr (HOME) hm = load_tokens<VEC>(home, n0, n_end);
        {
            const TokVec<VEC> t = load_tokens<VEC>(trace, n0, n_end);
            prev_clean = in_range;
            int away = 0;
#pragma unroll
            for (int u = 0; u < VEC; ++u) {
                ok_prev[u] = (n0 + u < n_end) && static_cast<unsigned>(t.v[u]) < static_cast<unsigned>(E);
                dev_prev[u] = ok_prev[u] ? pl[t.v[u]] : 0;
                prev_clean = prev_clean && ok_prev[u];
                if constexpr (HOME) away += __popcll(__ballot(ok_prev[u] && dev_prev[u] != hm.v[u]));
            }
            if constexpr (HOME)
                if (lane == 0 && away != 0) atomicAdd(&away_cnt[0], static_cast<uint32_t>(away));
        }
        auto load_layers = [&](int lb, TokVec<VEC>(&dst)[kLocAhead]) {
#pragma unroll
            for (int a = 0; a < kLocAhead; ++a)  // layers past the last one are clamped, not skipped: no branch at the loads
                dst[a] = load_tokens<VEC>(trace + static_cast<int64_t>(min(lb + a, L - 1)) * N, n0, n_end);
        };
        // software pipeline over batches of kLocAhead layers: the next batch is requested before the
        // current one is counted
        TokVec<VEC> cur[kLocAhead], nxt[kLocAhead];
        load_layers(1, cur);
        for (int lb = 1; lb < L; lb += kLocAhead) {
            load_layers(lb + kLocAhead, nxt);
#pragma unroll
            for (int a = 0; a < kLocAhead; ++a) {
                const int l = lb + a;
                if (l >= L) break;
                unsigned m = 0;
#pragma unroll
                for (int u = 0; u < VEC; ++u) m = max(m, static_cast<unsigned>(cur[a].v[u]));
                const bool clean = in_range && m < static_cast<unsigned>(E);
                // wavefront total of "device unchanged" flags by ballot + popcount (scalar unit)
                int same = 0, away = 0;
                if (__ballot(!(clean && prev_clean)) == 0ull) {
                    // fast path: every id of this wavefront is valid in both layers - one table
                    // look-up and one compare per transition
#pragma unroll
                    for (int u = 0; u < VEC; ++u) {
                        const int dev = pl[l * E + cur[a].v[u]];
                        same += __popcll(__ballot(dev == dev_prev[u]));
                        if constexpr (HOME) away += __popcll(__ballot(dev != hm.v[u]));
                        dev_prev[u] = dev;
                    }
                } else {
#pragma unroll
                    for (int u = 0; u < VEC; ++u) {
                        const bool ok = (n0 + u < n_end) && static_cast<unsigned>(cur[a].v[u]) < static_cast<unsigned>(E);
                        const int dev = ok ? pl[l * E + cur[a].v[u]] : 0;
                        same += __popcll(__ballot(ok && ok_prev[u] && dev == dev_prev[u]));
                        if constexpr (HOME) away += __popcll(__ballot(ok && dev != hm.v[u]));
                        ok_prev[u] = ok;
                        dev_prev[u] = dev;
                    }
                }
                if constexpr (HOME)
                    if (lane == 0 && away != 0) atomicAdd(&away_cnt[l], static_cast<uint32_t>(away));
                if (clean) {  // the flags the checked path would have produced
#pragma unroll
                    for (int u = 0; u < VEC; ++u) ok_prev[u] = true;
                }
                prev_clean = clean;
                if (lane == 0 && same != 0) atomicAdd(&pair_cnt[l - 1], static_cast<uint32_t>(same));
            }
#pragma unroll
            for (int a = 0; a < kLocAhead; ++a) cur[a] = nxt[a];
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < n_out; i += kTraceThreads) part[static_cast<size_t>(blockIdx.x) * n_out + i] = pair_cnt[i];
}

// One wavefront per output element j: the first `pairs` elements go to local_per_pair, the rest
// (present with home devices only) to away_per_layer.
__global__ __launch_bounds__(kWave) void locality_finalize_kernel(const uint32_t* __restrict__ part, int C, int pairs, int n_out,
                                                                   int64_t* __restrict__ local_per_pair,
                                                                   int64_t* __restrict__ away_per_layer)
{
    const int j = blockIdx.x;
    long long s = 0;
    for (int c = threadIdx.x; c < C; c += kWave) s += part[static_cast<size_t>(c) * n_out + j];
    s = wave_sum(s);
    if (threadIdx.x == 0) {
        if (j < pairs) local_per_pair[j] = s;
        else away_per_layer[j - pairs] = s;
    }
}

static int64_t locality_chunk(int64_t N, int vec)
{
    const int64_t sweep = static_cast<int64_t>(kTraceThreads) * vec;
    int64_t chunk = (N + kTargetWorkgroups - 1) / kTargetWorkgroups;  // about one workgroup per CU
    chunk = (chunk + sweep - 1) / sweep * sweep;
    if (chunk < sweep) chunk = sweep;
    const int64_t cap = (1ll << 31) / sweep * sweep;  // 32-bit partial counters
    return chunk > cap ? cap : chunk;
}

static int validate_trace_args(const char* fn, int L, int64_t N, int E)
{
    if (L < 1 || L > EXF_MAX_TRACE_LAYERS) return fail(EXF_ERR_BAD_SHAPE, "%s: L = %d outside [1,%d]", fn, L, EXF_MAX_TRACE_LAYERS);
    if (N < 0) return fail(EXF_ERR_BAD_SHAPE, "%s: N = %lld < 0", fn, static_cast<long long>(N));
    if (E < 1 || E > EXF_MAX_EXPERTS) return fail(EXF_ERR_BAD_SHAPE, "%s: E = %d outside [1,%d]", fn, E, EXF_MAX_EXPERTS);
    if (N >= (1ll << 40)) return fail(EXF_ERR_BAD_SHAPE, "%s: N must be below 2^40", fn);
    return EXF_OK;
}

template <typename Kern>
static int allow_large_lds(Kern kern, size_t bytes, const char* what)
{
    if (bytes <= 64 * 1024) return EXF_OK;
    hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                         static_cast<int>(bytes));
    if (err != hipSuccess) return fail(EXF_ERR_HIP, "%s: LDS attribute: %s", what, hipGetErrorString(err));
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

namespace exf {

// affinity_histogram and affinity_statistics: the same two launches.  With a placement every
// workgroup of the first launch also counts, per pair, the transitions of its finished histogram whose
// two experts share a device, and the second launch has one more workgroup per pair to add these up.
static int run_affinity(const char* fn, const int32_t* trace, const int32_t* placement, int L, int64_t N, int E, int64_t* counts,
                        int64_t* loads, float* cond_prob, int64_t* n_invalid, int64_t* local_per_pair, void* workspace,
                        size_t workspace_bytes, void* stream)
{
    const AffinityPlan p = make_affinity_plan(L, N, E, aligned16(trace));
    if (workspace_bytes < p.total_bytes) return fail(EXF_ERR_WORKSPACE_TOO_SMALL, "%s: workspace %zu < %zu bytes", fn, workspace_bytes, p.total_bytes);
    hipStream_t s = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    uint32_t* part_counts = reinterpret_cast<uint32_t*>(ws + p.off_counts);
    uint32_t* part_orphan_next = reinterpret_cast<uint32_t*>(ws + p.off_orphan_next);
    uint32_t* part_orphan_last = reinterpret_cast<uint32_t*>(ws + p.off_orphan_last);
    uint32_t* part_invalid = reinterpret_cast<uint32_t*>(ws + p.off_invalid);
    uint32_t* part_local = placement != nullptr ? reinterpret_cast<uint32_t*>(ws + p.off_local) : nullptr;
    if (p.C > 0) {
        const int c_pad = (p.C + kXcds - 1) / kXcds * kXcds;
        const unsigned grid = static_cast<unsigned>(c_pad) * p.Q;
        const size_t lds = (static_cast<size_t>(p.copies) * p.g * p.words + static_cast<size_t>(p.g) * E + E + 1 + p.g +
                            static_cast<size_t>(p.g + 1) * E) * sizeof(uint32_t);
        if (p.vec == 4) {
            if (int rc = allow_large_lds(affinity_partial_kernel<4>, lds, fn)) return rc;
            hipLaunchKernelGGL(affinity_partial_kernel<4>, dim3(grid), dim3(kTraceThreads), lds, s, trace, L, N, E, p.g, p.Q, p.copies,
                               p.words, p.chunk, p.C, part_counts, part_orphan_next, part_orphan_last, part_invalid, placement, part_local);
        } else {
            if (int rc = allow_large_lds(affinity_partial_kernel<1>, lds, fn)) return rc;
            hipLaunchKernelGGL(affinity_partial_kernel<1>, dim3(grid), dim3(kTraceThreads), lds, s, trace, L, N, E, p.g, p.Q, p.copies,
                               p.words, p.chunk, p.C, part_counts, part_orphan_next, part_orphan_last, part_invalid, placement, part_local);
        }
    }
    // rows of all pairs, then the loads of the final layer, the invalid tally and (with a placement) the
    // locality numerators of all pairs
    const unsigned fin_grid = static_cast<unsigned>(((L - 1) * E + kFinRowsPerWorkgroup - 1) / kFinRowsPerWorkgroup + E + 1 +
                                                   (placement != nullptr ? L - 1 : 0));
    hipLaunchKernelGGL(affinity_finalize_kernel, dim3(fin_grid), dim3(256), 0, s, part_counts, part_orphan_next, part_orphan_last,
                       part_invalid, p.C, p.Q, L, E, p.words, counts, loads, cond_prob, n_invalid, part_local, local_per_pair);
    return check_launch(fn);
}

}  // namespace exf

extern "C" int affinity_histogram(const int32_t* trace, int L, int64_t N, int E, int64_t* counts, int64_t* loads,
                                  float* cond_prob, int64_t* n_invalid, void* workspace, size_t workspace_bytes, void* stream)
{
    using namespace exf;
    if (int rc = validate_trace_args("affinity_histogram", L, N, E)) return rc;
    if (N > 0) EXF_REQUIRE_PTR(trace);
    if (L > 1) EXF_REQUIRE_PTR(counts);
    EXF_REQUIRE_PTR(workspace);
    return run_affinity("affinity_histogram", trace, nullptr, L, N, E, counts, loads, cond_prob, n_invalid, nullptr, workspace,
                        workspace_bytes, stream);
}

extern "C" size_t affinity_statistics_workspace_bytes(int L, int64_t N, int E) { return affinity_histogram_workspace_bytes(L, N, E); }

extern "C" int affinity_statistics(const int32_t* trace, const int32_t* placement, int L, int64_t N, int E, int G, int64_t* counts,
                                   int64_t* loads, float* cond_prob, int64_t* n_invalid, int64_t* local_per_pair, void* workspace,
                                   size_t workspace_bytes, void* stream)
{
    using namespace exf;
    if (int rc = validate_trace_args("affinity_statistics", L, N, E)) return rc;
    if (G < 1) return fail(EXF_ERR_BAD_SHAPE, "affinity_statistics: G = %d < 1", G);
    if (N > 0) EXF_REQUIRE_PTR(trace);
    EXF_REQUIRE_PTR(placement);
    if (L > 1) {
        EXF_REQUIRE_PTR(counts);
        EXF_REQUIRE_PTR(local_per_pair);
    }
    EXF_REQUIRE_PTR(workspace);
    return run_affinity("affinity_statistics", trace, placement, L, N, E, counts, loads, cond_prob, n_invalid, local_per_pair,
                        workspace, workspace_bytes, stream);
}

namespace exf {
struct MultihopPlan {
    int g, Q, copies, words, C, vec, pairs;
    int64_t chunk;
    size_t total_bytes;
};
static MultihopPlan make_multihop_plan(int L, int64_t N, int E, bool aligned)
{
    MultihopPlan p;
    p.pairs = L * (L - 1) / 2;
    p.words = (E * E + 1) / 2;
    const size_t hist_bytes = static_cast<size_t>(p.words) * sizeof(uint32_t);
    int g = static_cast<int>(kAffHistBudget / hist_bytes);
    if (g > kAffMaxGroup) g = kAffMaxGroup;
    if (g < 1) g = 1;
    p.g = g;
    p.copies = 1;
    while (p.copies < 16 && hist_bytes * g * (p.copies * 2) <= kAffHistBudget) p.copies *= 2;
    p.Q = 0;
    for (int l = 0; l + 1 < L; ++l) p.Q += (L - 1 - l + g - 1) / g;
    if (p.Q < 1) p.Q = 1;
    p.vec = (aligned && N % 4 == 0) ? 4 : 1;
    const int64_t sweep = static_cast<int64_t>(kTraceThreads) * p.vec;
    int c_target = kTargetWorkgroups / p.Q;
    if (c_target < 1) c_target = 1;
    int64_t chunk = (N + c_target - 1) / c_target;
    chunk = (chunk + sweep - 1) / sweep * sweep;
    if (chunk < sweep) chunk = sweep;
    if (chunk > kAffMaxChunk) chunk = kAffMaxChunk / sweep * sweep;
    p.chunk = chunk;
    p.C = static_cast<int>(N > 0 ? (N + chunk - 1) / chunk : 0);
    p.total_bytes = align_up(static_cast<size_t>(p.C > 0 ? p.C : 1) * (p.pairs > 0 ? p.pairs : 1) * p.words * sizeof(uint32_t), 256);
    return p;
}
}  // namespace exf

extern "C" size_t affinity_multihop_workspace_bytes(int L, int64_t N, int E)
{
    if (L < 1 || N < 0 || E < 1 || E > EXF_MAX_EXPERTS) return 0;
    const size_t a = exf::make_multihop_plan(L, N, E, true).total_bytes;
    const size_t b = exf::make_multihop_plan(L, N, E, false).total_bytes;
    return a > b ? a : b;
}

extern "C" int affinity_multihop(const int32_t* trace, int L, int64_t N, int E, int64_t* counts, float* cond_prob, void* workspace,
                                 size_t workspace_bytes, void* stream)
{
    using namespace exf;
    if (int rc = validate_trace_args("affinity_multihop", L, N, E)) return rc;
    if (L == 1) return EXF_OK;  // no pair, no output element
    if (N > 0) EXF_REQUIRE_PTR(trace);
    EXF_REQUIRE_PTR(counts);
    EXF_REQUIRE_PTR(workspace);
    const MultihopPlan p = make_multihop_plan(L, N, E, aligned16(trace));
    if (workspace_bytes < p.total_bytes)
        return fail(EXF_ERR_WORKSPACE_TOO_SMALL, "affinity_multihop: workspace %zu < %zu bytes", workspace_bytes, p.total_bytes);
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint32_t* part_counts = static_cast<uint32_t*>(workspace);
    if (p.C > 0) {
        const int c_pad = (p.C + kXcds - 1) / kXcds * kXcds;
        const int64_t grid = static_cast<int64_t>(c_pad) * p.Q;
        if (grid >= (1ll << 31)) return fail(EXF_ERR_BAD_SHAPE, "affinity_multihop: too many workgroups");
        const size_t lds = static_cast<size_t>(p.copies) * p.g * p.words * sizeof(uint32_t);
        if (p.vec == 4) {
            if (int rc = allow_large_lds(multihop_partial_kernel<4>, lds, "affinity_multihop")) return rc;
            hipLaunchKernelGGL(multihop_partial_kernel<4>, dim3(static_cast<unsigned>(grid)), dim3(kTraceThreads), lds, s, trace, L, N, E,
                               p.g, p.Q, p.copies, p.words, p.chunk, p.C, part_counts);
        } else {
            if (int rc = allow_large_lds(multihop_partial_kernel<1>, lds, "affinity_multihop")) return rc;
            hipLaunchKernelGGL(multihop_partial_kernel<1>, dim3(static_cast<unsigned>(grid)), dim3(kTraceThreads), lds, s, trace, L, N, E,
                               p.g, p.Q, p.copies, p.words, p.chunk, p.C, part_counts);
        }
    }
    // one wavefront per (pair, source expert) row: sums the chunks, forms the conditional probabilities
    // (the finalize kernel of the one-hop statistic, told that there are pairs+1 "layers" and no loads)
    const unsigned fin_grid = static_cast<unsigned>((p.pairs * E + kFinRowsPerWorkgroup - 1) / kFinRowsPerWorkgroup);
    hipLaunchKernelGGL(affinity_finalize_kernel, dim3(fin_grid), dim3(256), 0, s, part_counts, nullptr, nullptr, nullptr, p.C, 1,
                       p.pairs + 1, E, p.words, counts, nullptr, cond_prob, nullptr, nullptr, nullptr);
    return check_launch("affinity_multihop");
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
        if (vec == 4) {
            if (int rc = allow_large_lds(locality_partial_kernel<4, false>, lds, "placement_locality")) return rc;
            hipLaunchKernelGGL((locality_partial_kernel<4, false>), dim3(C), dim3(kTraceThreads), lds, s, trace, placement, nullptr, L, N,
                               E, chunk, part);
        } else {
            if (int rc = allow_large_lds(locality_partial_kernel<1, false>, lds, "placement_locality")) return rc;
            hipLaunchKernelGGL((locality_partial_kernel<1, false>), dim3(C), dim3(kTraceThreads), lds, s, trace, placement, nullptr, L, N,
                               E, chunk, part);
        }
    }
    hipLaunchKernelGGL(locality_finalize_kernel, dim3(L - 1), dim3(kWave), 0, s, part, C, L - 1, L - 1, local_per_pair, nullptr);
    return check_launch("placement_locality");
}

extern "C" size_t routing_transfers_workspace_bytes(int L, int64_t N)
{
    if (L < 1 || N < 0) return 0;
    const int64_t chunk = exf::locality_chunk(N, 1);  // the scalar plan has the most chunks
    const int64_t C = N > 0 ? (N + chunk - 1) / chunk : 0;
    return exf::align_up(static_cast<size_t>(C > 0 ? C : 1) * static_cast<size_t>(2 * L - 1) * sizeof(uint32_t), 256);
}

extern "C" int routing_transfers(const int32_t* trace, const int32_t* placement, const int32_t* home, int L, int64_t N, int E, int G,
                                 int64_t* local_per_pair, int64_t* away_per_layer, void* workspace, size_t workspace_bytes,
                                 void* stream)
{
    using namespace exf;
    if (int rc = validate_trace_args("routing_transfers", L, N, E)) return rc;
    if (G < 1) return fail(EXF_ERR_BAD_SHAPE, "routing_transfers: G = %d < 1", G);
    EXF_REQUIRE_PTR(placement);
    EXF_REQUIRE_PTR(away_per_layer);
    if (L > 1) EXF_REQUIRE_PTR(local_per_pair);
    EXF_REQUIRE_PTR(workspace);
    if (N > 0) {
        EXF_REQUIRE_PTR(trace);
        EXF_REQUIRE_PTR(home);
    }
    if (workspace_bytes < routing_transfers_workspace_bytes(L, N))
        return fail(EXF_ERR_WORKSPACE_TOO_SMALL, "routing_transfers: workspace %zu < %zu bytes", workspace_bytes,
                    routing_transfers_workspace_bytes(L, N));
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int vec = (aligned16(trace) && aligned16(home) && N % 4 == 0) ? 4 : 1;
    const int64_t chunk = locality_chunk(N, vec);
    const int C = static_cast<int>(N > 0 ? (N + chunk - 1) / chunk : 0);
    uint32_t* part = static_cast<uint32_t*>(workspace);
    const int n_out = 2 * L - 1;
    if (C > 0) {
        const size_t lds = (static_cast<size_t>(L) * E + n_out) * sizeof(int32_t);
        if (vec == 4) {
            if (int rc = allow_large_lds(locality_partial_kernel<4, true>, lds, "routing_transfers")) return rc;
            hipLaunchKernelGGL((locality_partial_kernel<4, true>), dim3(C), dim3(kTraceThreads), lds, s, trace, placement, home, L, N, E,
                               chunk, part);
        } else {
            if (int rc = allow_large_lds(locality_partial_kernel<1, true>, lds, "routing_transfers")) return rc;
            hipLaunchKernelGGL((locality_partial_kernel<1, true>), dim3(C), dim3(kTraceThreads), lds, s, trace, placement, home, L, N, E,
                               chunk, part);
        }
    }
    hipLaunchKernelGGL(locality_finalize_kernel, dim3(n_out), dim3(kWave), 0, s, part, C, L - 1, n_out, local_per_pair, away_per_layer);
    return check_launch("routing_transfers");
}
