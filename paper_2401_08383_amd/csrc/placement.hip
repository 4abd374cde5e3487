// Placement search driven by the co-routing statistic (Design, "Solving Affinity's duality by
// Integer Programming" and "Staged Experts Affinity").
//
// The integer program minimises the crossing transitions  sum_k sum_j R_{k,j}  under load balance
// (every part holds E/P experts of every layer) and exclusivity (every expert on one part).  With
// the E x E counts of affinity_histogram the objective of a map is
//     total - sum_l sum_{i,p} counts[l][i][p] * [part_l(i) == part_{l+1}(p)],
// so it is evaluated from 754 KB of counts instead of the trace.
//
//   placement_locality_from_counts : GPU, scores a BATCH of candidate maps against the counts.
//       One workgroup per (layer pair, slice of candidates) keeps the pair's E x E counts in LDS;
//       a wavefront takes one candidate at a time: lane p holds the part of expert p at layer l+1,
//       walks the E source experts (their parts broadcast by shuffle) and adds the counts of the
//       pairs that share a part; 64-bit integer arithmetic throughout, so the result is exact.
//   exf_placement_search           : host.  The paper names no solver; this one is
//       - exact when the number of balanced partitions of a layer is small: the objective is a
//         chain over layers, so a dynamic programme over (layer, partition) finds the optimum;
//       - otherwise layer by layer greedy (largest regret first) followed by pairwise-swap local
//         search with exact O(1) swap gains from per-expert inflow / outflow tables, over several
//         random restarts.
//       Two stages as in the paper: first experts -> nodes (crossings between nodes), then inside
//       every node its experts -> its GPUs, scored with the transitions that stay in the node.
#include <stdint.h>

#include <algorithm>
#include <numeric>
#include <vector>

#include "common.hpp"

namespace exf {

constexpr int kScoreThreads = 256;
constexpr int kScoreWaves = kScoreThreads / kWave;
constexpr int kScoreSlice = 64;  // candidates per workgroup

__global__ __launch_bounds__(kScoreThreads) void placement_score_kernel(const int64_t* __restrict__ counts,
                                                                         const int32_t* __restrict__ placements, int B, int L, int E,
                                                                         int64_t* __restrict__ local)
{
    extern __shared__ long long cnt_lds[];  // [E][E] counts of this layer pair
    const int l = blockIdx.y;  // layer pair on y (at most 255), candidate slices on x (up to 2^18)
    const int64_t* src = counts + static_cast<size_t>(l) * E * E;
    for (int i = threadIdx.x; i < E * E; i += kScoreThreads) cnt_lds[i] = src[i];
    __syncthreads();

    const int lane = lane_id();
    const int wave = threadIdx.x / kWave;
    const int b_end = min(B, (static_cast<int>(blockIdx.x) + 1) * kScoreSlice);
    int b = static_cast<int>(blockIdx.x) * kScoreSlice + wave;
    // parts of the candidate's experts at layers l (lane = source expert) and l+1 (lane = target expert);
    // the next candidate's two rows are requested before the current one is scored
    auto load_rows = [&](int cand, int& cur_row, int& nxt_row) {
        const int c = min(cand, B - 1);
        const int e = min(lane, E - 1);
        const int32_t* row = placements + (static_cast<size_t>(c) * L + l) * E;
        cur_row = row[e];
        nxt_row = row[E + e];
    };
    int part_l = 0, part_l1 = 0;
    if (b < b_end) load_rows(b, part_l, part_l1);
    while (b < b_end) {
        int next_l = 0, next_l1 = 0;
        load_rows(b + kScoreWaves, next_l, next_l1);
        long long acc = 0;
        for (int i = 0; i < E; ++i) {
            const int pi = __shfl(part_l, i, kWave);
            if (lane < E && pi == part_l1) acc += cnt_lds[i * E + lane];
        }
        acc = wave_sum(acc);
        if (lane == 0) local[static_cast<size_t>(b) * (L - 1) + l] = acc;
        part_l = next_l;
        part_l1 = next_l1;
        b += kScoreWaves;
    }
}

// ------------------------------------------------------------------------------------ host solver
namespace {

// counts of one sub-problem: n experts per layer, counts[l][i][p] for the L-1 pairs
struct Problem {
    int L, n, P;
    std::vector<int64_t> c;  // [(L-1)][n][n]
    int64_t at(int l, int i, int p) const { return c[(static_cast<size_t>(l) * n + i) * n + p]; }
};

int64_t score(const Problem& pb, const std::vector<int>& part)  // part [L][n]
{
    int64_t s = 0;
    for (int l = 0; l + 1 < pb.L; ++l)
        for (int i = 0; i < pb.n; ++i)
            for (int p = 0; p < pb.n; ++p)
                if (part[l * pb.n + i] == part[(l + 1) * pb.n + p]) s += pb.at(l, i, p);
    return s;
}

// all labelled balanced partitions of n experts into P parts, if there are at most `limit` of them
bool enumerate_partitions(int n, int P, size_t limit, std::vector<std::vector<int>>& out)
{
    const int cap = n / P;
    std::vector<int> cur, left(P, cap);
    bool ok = true;
    auto rec = [&](auto&& self, int e) -> void {
        if (!ok) return;
        if (e == n) {
            if (out.size() >= limit) {
                ok = false;
                return;
            }
            out.push_back(cur);
            return;
        }
        for (int p = 0; p < P; ++p)
            if (left[p] > 0) {
                left[p] -= 1;
                cur.push_back(p);
                self(self, e + 1);
                cur.pop_back();
                left[p] += 1;
            }
    };
    rec(rec, 0);
    return ok;
}

// exact optimum by dynamic programming over the chain of layers; returns false if the state space is too large
bool solve_exact(const Problem& pb, std::vector<int>& part)
{
    std::vector<std::vector<int>> parts;
    if (!enumerate_partitions(pb.n, pb.P, 128, parts)) return false;
    const int S = static_cast<int>(parts.size());
    const int n = pb.n;
    std::vector<int64_t> best(static_cast<size_t>(pb.L) * S, 0);
    std::vector<int> from(static_cast<size_t>(pb.L) * S, 0);
    for (int l = 1; l < pb.L; ++l) {
        for (int t = 0; t < S; ++t) {
            int64_t top = -1;
            int arg = 0;
            for (int s = 0; s < S; ++s) {
                int64_t v = best[static_cast<size_t>(l - 1) * S + s];
                for (int i = 0; i < n; ++i)
                    for (int p = 0; p < n; ++p)
                        if (parts[s][i] == parts[t][p]) v += pb.at(l - 1, i, p);
                if (v > top) {
                    top = v;
                    arg = s;
                }
            }
            best[static_cast<size_t>(l) * S + t] = top;
            from[static_cast<size_t>(l) * S + t] = arg;
        }
    }
    int t = 0;
    for (int s = 1; s < S; ++s)
        if (best[static_cast<size_t>(pb.L - 1) * S + s] > best[static_cast<size_t>(pb.L - 1) * S + t]) t = s;
    part.assign(static_cast<size_t>(pb.L) * n, 0);
    for (int l = pb.L - 1; l >= 0; --l) {
        for (int e = 0; e < n; ++e) part[l * n + e] = parts[t][e];
        t = from[static_cast<size_t>(l) * S + t];
    }
    return true;
}

struct Rng {  // splitmix64: the restarts must not depend on the C library's generator
    uint64_t s;
    uint64_t next()
    {
        uint64_t z = (s += 0x9e3779b97f4a7c15ull);
        z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
        z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
        return z ^ (z >> 31);
    }
    int below(int n) { return static_cast<int>(next() % static_cast<uint64_t>(n)); }
};

// layer l+1 from layer l: expert p gains  gain[p][g] = sum_{i on part g} counts[l][i][p]  on part g;
// experts are fixed one at a time, the one with the largest regret (best minus second-best open part) first
void greedy_next_layer(const Problem& pb, int l, std::vector<int>& part)
{
    const int n = pb.n, P = pb.P, cap = n / P;
    std::vector<int64_t> gain(static_cast<size_t>(n) * P, 0);
    for (int i = 0; i < n; ++i)
        for (int p = 0; p < n; ++p) gain[static_cast<size_t>(p) * P + part[l * n + i]] += pb.at(l, i, p);
    std::vector<int> left(P, cap);
    std::vector<char> done(n, 0);
    for (int step = 0; step < n; ++step) {
        int pick = -1, pick_part = 0;
        int64_t pick_regret = -1;
        for (int p = 0; p < n; ++p) {
            if (done[p]) continue;
            int64_t b1 = -1, b2 = -1;
            int a1 = 0;
            for (int g = 0; g < P; ++g) {
                if (left[g] == 0) continue;
                const int64_t v = gain[static_cast<size_t>(p) * P + g];
                if (v > b1) {
                    b2 = b1;
                    b1 = v;
                    a1 = g;
                } else if (v > b2) {
                    b2 = v;
                }
            }
            const int64_t regret = b2 < 0 ? b1 : b1 - b2;
            if (regret > pick_regret) {
                pick_regret = regret;
                pick = p;
                pick_part = a1;
            }
        }
        done[pick] = 1;
        left[pick_part] -= 1;
        part[(l + 1) * n + pick] = pick_part;
    }
}

// pairwise swaps inside a layer until none improves.  value[l][e][g] = transitions of expert e of layer
// l that stay local if e sits on part g (inflow from layer l-1 plus outflow to layer l+1); two experts
// of one layer never interact, so the gain of a swap is exact.
void local_search(const Problem& pb, std::vector<int>& part)
{
    const int L = pb.L, n = pb.n, P = pb.P;
    std::vector<int64_t> value(static_cast<size_t>(L) * n * P);
    auto rebuild_layer = [&](int l) {
        for (int e = 0; e < n; ++e)
            for (int g = 0; g < P; ++g) value[(static_cast<size_t>(l) * n + e) * P + g] = 0;
        if (l > 0)
            for (int i = 0; i < n; ++i)
                for (int e = 0; e < n; ++e) value[(static_cast<size_t>(l) * n + e) * P + part[(l - 1) * n + i]] += pb.at(l - 1, i, e);
        if (l + 1 < L)
            for (int e = 0; e < n; ++e)
                for (int p = 0; p < n; ++p) value[(static_cast<size_t>(l) * n + e) * P + part[(l + 1) * n + p]] += pb.at(l, e, p);
    };
    for (int l = 0; l < L; ++l) rebuild_layer(l);
    bool improved = true;
    for (int sweep = 0; improved && sweep < 1000; ++sweep) {
        improved = false;
        for (int l = 0; l < L; ++l) {
            for (int a = 0; a < n; ++a)
                for (int b = a + 1; b < n; ++b) {
                    const int ga = part[l * n + a], gb = part[l * n + b];
                    if (ga == gb) continue;
                    const int64_t* va = &value[(static_cast<size_t>(l) * n + a) * P];
                    const int64_t* vb = &value[(static_cast<size_t>(l) * n + b) * P];
                    const int64_t delta = (va[gb] + vb[ga]) - (va[ga] + vb[gb]);
                    if (delta > 0) {
                        part[l * n + a] = gb;
                        part[l * n + b] = ga;
                        if (l > 0) rebuild_layer(l - 1);
                        if (l + 1 < L) rebuild_layer(l + 1);
                        improved = true;
                    }
                }
        }
    }
}

void solve_heuristic(const Problem& pb, int restarts, uint64_t seed, std::vector<int>& best_part)
{
    const int n = pb.n, P = pb.P, cap = n / P;
    Rng rng{seed};
    int64_t best = -1;
    std::vector<int> part(static_cast<size_t>(pb.L) * n);
    for (int r = 0; r < std::max(restarts, 1); ++r) {
        std::vector<int> order(n);
        std::iota(order.begin(), order.end(), 0);
        if (r > 0)
            for (int i = n - 1; i > 0; --i) std::swap(order[i], order[rng.below(i + 1)]);  // first restart: contiguous
        for (int i = 0; i < n; ++i) part[order[i]] = i / cap;
        for (int l = 0; l + 1 < pb.L; ++l) greedy_next_layer(pb, l, part);
        local_search(pb, part);
        const int64_t s = score(pb, part);
        if (s > best) {
            best = s;
            best_part = part;
        }
    }
}

void solve(const Problem& pb, int restarts, uint64_t seed, std::vector<int>& part)
{
    if (pb.P == 1) {
        part.assign(static_cast<size_t>(pb.L) * pb.n, 0);
        return;
    }
    if (!solve_exact(pb, part)) solve_heuristic(pb, restarts, seed, part);
}

}  // namespace
}  // namespace exf

extern "C" int placement_locality_from_counts(const int64_t* counts, const int32_t* placements, int B, int L, int E,
                                              int64_t* local, void* stream)
{
    using namespace exf;
    if (L < 1 || L > EXF_MAX_TRACE_LAYERS) return fail(EXF_ERR_BAD_SHAPE, "placement_locality_from_counts: L = %d outside [1,%d]", L, EXF_MAX_TRACE_LAYERS);
    if (E < 1 || E > EXF_MAX_EXPERTS) return fail(EXF_ERR_BAD_SHAPE, "placement_locality_from_counts: E = %d outside [1,%d]", E, EXF_MAX_EXPERTS);
    if (B < 0 || B > (1 << 24)) return fail(EXF_ERR_BAD_SHAPE, "placement_locality_from_counts: B = %d outside [0,2^24]", B);
    if (B == 0 || L == 1) return EXF_OK;  // no candidate or no transition: no output element
    EXF_REQUIRE_PTR(counts);
    EXF_REQUIRE_PTR(placements);
    EXF_REQUIRE_PTR(local);
    const dim3 grid(static_cast<unsigned>((B + kScoreSlice - 1) / kScoreSlice), static_cast<unsigned>(L - 1));
    const size_t lds = static_cast<size_t>(E) * E * sizeof(long long);
    hipLaunchKernelGGL(placement_score_kernel, grid, dim3(kScoreThreads), lds, static_cast<hipStream_t>(stream), counts, placements, B, L,
                       E, local);
    return check_launch("placement_locality_from_counts");
}

extern "C" int exf_placement_search(const int64_t* counts_host, int L, int E, int G, int nodes, int restarts, uint64_t seed,
                                    int32_t* placement_host)
{
    using namespace exf;
    EXF_REQUIRE_PTR(placement_host);
    if (L < 1 || L > EXF_MAX_TRACE_LAYERS || E < 1 || E > EXF_MAX_EXPERTS)
        return fail(EXF_ERR_BAD_SHAPE, "exf_placement_search: L = %d, E = %d out of range", L, E);
    if (G < 1 || nodes < 1 || E % G != 0 || G % nodes != 0)
        return fail(EXF_ERR_BAD_SHAPE, "exf_placement_search: need nodes | G | E (E=%d G=%d nodes=%d)", E, G, nodes);
    if (L > 1) EXF_REQUIRE_PTR(counts_host);
    for (int l = 0; l + 1 < L; ++l)
        for (int i = 0; i < E * E; ++i)
            if (counts_host[static_cast<size_t>(l) * E * E + i] < 0)
                return fail(EXF_ERR_BAD_SHAPE, "exf_placement_search: negative count in layer pair %d", l);

    // stage 1: experts -> nodes
    Problem top{L, E, nodes, {}};
    top.c.assign(counts_host, counts_host + static_cast<size_t>(L > 1 ? L - 1 : 0) * E * E);
    std::vector<int> node_of;
    solve(top, restarts, seed, node_of);

    // stage 2: inside every node, its experts -> its GPUs, scored with the transitions that stay in the node
    const int per_node = G / nodes, n_sub = E / nodes;
    for (int nd = 0; nd < nodes; ++nd) {
        std::vector<int> members(static_cast<size_t>(L) * n_sub);  // expert ids of this node, per layer, ascending
        for (int l = 0; l < L; ++l) {
            int k = 0;
            for (int e = 0; e < E; ++e)
                if (node_of[l * E + e] == nd) members[l * n_sub + k++] = e;
        }
        Problem sub{L, n_sub, per_node, {}};
        sub.c.resize(static_cast<size_t>(L > 1 ? L - 1 : 0) * n_sub * n_sub);
        for (int l = 0; l + 1 < L; ++l)
            for (int i = 0; i < n_sub; ++i)
                for (int p = 0; p < n_sub; ++p)
                    sub.c[(static_cast<size_t>(l) * n_sub + i) * n_sub + p] =
                        counts_host[(static_cast<size_t>(l) * E + members[l * n_sub + i]) * E + members[(l + 1) * n_sub + p]];
        std::vector<int> gpu_of;
        solve(sub, restarts, seed + 0x1000u * static_cast<uint64_t>(nd + 1), gpu_of);
        for (int l = 0; l < L; ++l)
            for (int i = 0; i < n_sub; ++i) placement_host[static_cast<size_t>(l) * E + members[l * n_sub + i]] = nd * per_node + gpu_of[l * n_sub + i];
    }
    return EXF_OK;
}
