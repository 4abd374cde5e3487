/*
 * CPU oracle for the single-GPU hot path of context-coherent MoE inference with
 * inter-layer expert affinity (arXiv 2401.08383).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is the plain definition of every step, written out
 * as loops with fp64 arithmetic, so that a reader can check it against the paper by eye.
 * Only the tests, the smoke check and the benchmark's cpu_baseline leg may call it; the
 * GPU library shares no code, header, table or helper with this file.
 *
 * Every function below has at least one pin in the CPU test-suite (closed forms,
 * invariants, brute force, the paper's worked placement example); none is
 * "parity unpinned".
 *
 * Parallelism: an OpenMP `parallel for` over independent tokens / rows only (no
 * blocking, no reordering of any reduction).  Integer statistics are single-threaded.
 *
 * Conventions: row-major arrays; the reduction dimension is contiguous for every weight
 * (Wg [E,d], W1 [E_loc,f,d], W2 [E_loc,d,f]).  Activations and weights arrive as fp32
 * arrays (bf16 values are widened exactly by the caller) and are promoted to double
 * before any arithmetic.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------------------
 * Gate (Background "Gating Strategies": softmax-based gating; Challenges "Data Locality":
 * the gate decides each token's destination expert).
 * logits[t][e] = sum_c x[t][c] * Wg[e][c], c ascending.  No bias, no noise.
 * ---------------------------------------------------------------------------------- */
void ref_gate_logits(const float* x, const float* wg, int64_t T, int d, int E, double* logits)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        for (int e = 0; e < E; ++e) {
            double acc = 0.0;
            for (int c = 0; c < d; ++c)
                acc += (double)x[t * d + c] * (double)wg[(int64_t)e * d + c];
            logits[t * E + e] = acc;
        }
    }
}

/* Softmax over the E experts of each token: p = exp(l - max) / sum exp(l - max). */
void ref_softmax(const double* logits, int64_t T, int E, double* p)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        const double* l = logits + t * E;
        double m = l[0];
        for (int e = 1; e < E; ++e)
            if (l[e] > m) m = l[e];
        double s = 0.0;
        for (int e = 0; e < E; ++e) s += exp(l[e] - m);
        for (int e = 0; e < E; ++e) p[t * E + e] = exp(l[e] - m) / s;
    }
}

/* ------------------------------------------------------------------------------------
 * Top-k routing (Experimental setup: top-1 gating with variable token capacity, i.e. no
 * token is dropped or padded; Table 1 also carries top-2 volume formulas).
 * Selection is on the logits (order-equivalent to the probabilities), k times: the
 * largest logit not yet taken, the lowest expert id among equals.  Slot 0 is the best.
 * Weight: the softmax probability of the chosen expert; when renormalize != 0 and k > 1
 * the k weights are divided by their sum.
 * ---------------------------------------------------------------------------------- */
void ref_topk(const double* logits, int64_t T, int E, int k, int renormalize,
              int32_t* topk_idx, double* topk_w)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        const double* l = logits + t * E;
        double m = l[0];
        for (int e = 1; e < E; ++e)
            if (l[e] > m) m = l[e];
        double s = 0.0;
        for (int e = 0; e < E; ++e) s += exp(l[e] - m);

        int32_t taken[8];
        for (int j = 0; j < k; ++j) {
            int best = -1;
            for (int e = 0; e < E; ++e) {
                int used = 0;
                for (int q = 0; q < j; ++q)
                    if (taken[q] == e) used = 1;
                if (used) continue;
                if (best < 0 || l[e] > l[best]) best = e; /* strict > keeps the lowest id */
            }
            taken[j] = best;
            topk_idx[t * k + j] = best;
            topk_w[t * k + j] = exp(l[best] - m) / s;
        }
        if (renormalize && k > 1) {
            double z = 0.0;
            for (int j = 0; j < k; ++j) z += topk_w[t * k + j];
            for (int j = 0; j < k; ++j) topk_w[t * k + j] /= z;
        }
    }
}

/* ------------------------------------------------------------------------------------
 * Token dispatch (Challenges "Data Locality": tokens are grouped by the expert the gate
 * chose).  Assignments a = t*k + j are visited in ascending a and appended to the bucket
 * of their local expert; buckets are concatenated in expert order.  That is a stable
 * counting sort, so the permutation is unique.
 *   g = topk_idx[a];  g outside [0,E)           -> invalid, sorted_of_src[a] = -1
 *   e = expert_map ? expert_map[g] : g;  e < 0  -> not local,  sorted_of_src[a] = -1
 *   (e >= E_local is treated as invalid as well)
 * Returns the number of kept assignments (= offsets[E_local]).
 * ---------------------------------------------------------------------------------- */
int64_t ref_dispatch(const int32_t* topk_idx, const int32_t* expert_map, int64_t T, int k,
                     int E, int E_local, int32_t* src_of_sorted, int32_t* sorted_of_src,
                     int32_t* expert_counts, int32_t* expert_offsets, int64_t* n_invalid)
{
    const int64_t A = T * k;
    int64_t invalid = 0;
    int32_t* local = (int32_t*)malloc(sizeof(int32_t) * (size_t)(A > 0 ? A : 1));
    for (int e = 0; e < E_local; ++e) expert_counts[e] = 0;
    for (int64_t a = 0; a < A; ++a) {
        int32_t g = topk_idx[a];
        int32_t e = -1;
        if (g < 0 || g >= E) {
            ++invalid;
        } else {
            e = expert_map ? expert_map[g] : g;
            if (e >= E_local) { e = -1; ++invalid; }
            if (e < -1) e = -1;
        }
        local[a] = e;
        if (e >= 0) expert_counts[e] += 1;
    }
    expert_offsets[0] = 0;
    for (int e = 0; e < E_local; ++e) expert_offsets[e + 1] = expert_offsets[e] + expert_counts[e];
    int32_t* cursor = (int32_t*)malloc(sizeof(int32_t) * (size_t)(E_local > 0 ? E_local : 1));
    for (int e = 0; e < E_local; ++e) cursor[e] = expert_offsets[e];
    for (int64_t a = 0; a < A; ++a) {
        int32_t e = local[a];
        if (e < 0) { sorted_of_src[a] = -1; continue; }
        int32_t s = cursor[e]++;
        src_of_sorted[s] = (int32_t)a;
        sorted_of_src[a] = s;
    }
    int64_t kept = expert_offsets[E_local];
    free(cursor);
    free(local);
    if (n_invalid) *n_invalid = invalid;
    return kept;
}

/* x_sorted[s] = x[src_of_sorted[s] / k]  (a pure copy of token rows). */
void ref_gather_rows(const float* x, const int32_t* src_of_sorted, int64_t n_sorted, int k, int d,
                     float* x_sorted)
{
    for (int64_t s = 0; s < n_sorted; ++s) {
        int64_t t = src_of_sorted[s] / k;
        memcpy(x_sorted + s * d, x + t * d, sizeof(float) * (size_t)d);
    }
}

/* ------------------------------------------------------------------------------------
 * Expert FFN (Introduction / Challenges: every expert is a context-free feed-forward
 * network applied to the tokens routed to it).
 *   h[u] = act( sum_c x_s[c] * W1[e][u][c] + b1[e][u] ),   u < f
 *   y[v] =      sum_u h[u]  * W2[e][v][u] + b2[e][v],      v < d
 * act 0: GELU, exact form  z/2 * (1 + erf(z / sqrt 2));  act 1: tanh approximation
 *   z/2 * (1 + tanh( sqrt(2/pi) * (z + 0.044715 z^3) )).
 * The hidden vector stays in fp64.  Only the requested sorted rows are evaluated, so
 * the same routine serves full small cases and sampled rows of large ones; the expert of
 * row s is the e with offsets[e] <= s < offsets[e+1].
 * ---------------------------------------------------------------------------------- */
static double act_fn(double z, int act)
{
    if (act == 1) {
        const double c = 0.79788456080286535588; /* sqrt(2/pi) */
        return 0.5 * z * (1.0 + tanh(c * (z + 0.044715 * z * z * z)));
    }
    return 0.5 * z * (1.0 + erf(z * 0.70710678118654752440));
}

void ref_expert_ffn_rows(const float* x_sorted, const int32_t* expert_offsets, const float* w1,
                         const float* b1, const float* w2, const float* b2, int d, int f,
                         int E_local, int act, const int64_t* rows, int64_t n_rows, double* y)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < n_rows; ++r) {
        const int64_t s = rows[r];
        int e = -1;
        for (int q = 0; q < E_local; ++q)
            if (s >= expert_offsets[q] && s < expert_offsets[q + 1]) e = q;
        double* yr = y + r * d;
        if (e < 0) { /* row beyond the last bucket: no expert owns it */
            for (int v = 0; v < d; ++v) yr[v] = 0.0;
            continue;
        }
        const float* xs = x_sorted + s * d;
        const float* W1 = w1 + (int64_t)e * f * d;
        const float* W2 = w2 + (int64_t)e * d * f;
        double* h = (double*)malloc(sizeof(double) * (size_t)f);
        for (int u = 0; u < f; ++u) {
            double acc = 0.0;
            for (int c = 0; c < d; ++c) acc += (double)xs[c] * (double)W1[(int64_t)u * d + c];
            if (b1) acc += (double)b1[(int64_t)e * f + u];
            h[u] = act_fn(acc, act);
        }
        for (int v = 0; v < d; ++v) {
            double acc = 0.0;
            for (int u = 0; u < f; ++u) acc += h[u] * (double)W2[(int64_t)v * f + u];
            if (b2) acc += (double)b2[(int64_t)e * d + v];
            yr[v] = acc;
        }
        free(h);
    }
}

/* ------------------------------------------------------------------------------------
 * Gate-weighted combine (Background "Expert Model": a soft gate combines expert outputs).
 *   out[t] = sum_{j<k} w[t][j] * y_sorted[ sorted_of_src[t*k+j] ],  j ascending,
 * assignments whose sorted position is -1 contribute nothing.
 * ---------------------------------------------------------------------------------- */
void ref_combine(const double* y_sorted, const int32_t* sorted_of_src, const double* topk_w,
                 int64_t T, int d, int k, double* out)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        for (int c = 0; c < d; ++c) out[t * d + c] = 0.0;
        for (int j = 0; j < k; ++j) {
            int32_t s = sorted_of_src[t * k + j];
            if (s < 0) continue;
            double w = topk_w[t * k + j];
            for (int c = 0; c < d; ++c) out[t * d + c] += w * y_sorted[(int64_t)s * d + c];
        }
    }
}

/* ------------------------------------------------------------------------------------
 * Inter-layer expert affinity (Design "Modeling Inter-layer Expert Affinity", the
 * conditional-probability equation).  With hard top-1 routing a token's term is the
 * indicator of (expert i at layer l, expert p at layer l+1):
 *   counts[l][i][p] = #{ n : tr[l][n] = i and tr[l+1][n] = p },   l = 0 .. L-2
 *   loads[l][i]     = #{ n : tr[l][n] = i },                      l = 0 .. L-1
 * An id outside [0,E) is tallied in n_invalid; a transition with an invalid end is not
 * counted.  trace is layer-major [L][N].
 * ---------------------------------------------------------------------------------- */
void ref_affinity_counts(const int32_t* trace, int L, int64_t N, int E, int64_t* counts,
                         int64_t* loads, int64_t* n_invalid)
{
    int64_t invalid = 0;
    if (L > 1) memset(counts, 0, sizeof(int64_t) * (size_t)(L - 1) * E * E);
    if (loads) memset(loads, 0, sizeof(int64_t) * (size_t)L * E);
    for (int l = 0; l < L; ++l) {
        for (int64_t n = 0; n < N; ++n) {
            int32_t i = trace[(int64_t)l * N + n];
            if (i < 0 || i >= E) { ++invalid; continue; }
            if (loads) loads[(int64_t)l * E + i] += 1;
            if (l + 1 < L) {
                int32_t p = trace[(int64_t)(l + 1) * N + n];
                if (p < 0 || p >= E) continue;
                counts[((int64_t)l * E + i) * E + p] += 1;
            }
        }
    }
    if (n_invalid) *n_invalid = invalid;
}

/* Conditional probability P(expert p at layer l+1 | expert i at layer l): the count
 * divided by the number of tokens AT expert i of layer l that also have a valid next
 * expert (the row sum); an empty row is all zeros. */
void ref_cond_prob(const int64_t* counts, int L, int E, double* prob)
{
    for (int l = 0; l + 1 < L; ++l) {
        for (int i = 0; i < E; ++i) {
            const int64_t* row = counts + ((int64_t)l * E + i) * E;
            int64_t s = 0;
            for (int p = 0; p < E; ++p) s += row[p];
            for (int p = 0; p < E; ++p)
                prob[((int64_t)l * E + i) * E + p] = s > 0 ? (double)row[p] / (double)s : 0.0;
        }
    }
}

/* ------------------------------------------------------------------------------------
 * Locality of a placement (Design "Solving Affinity's duality by Integer Programming":
 * the objective sums, over tokens and the L-1 layer transitions, the indicator that the
 * token moves to an expert on another device; the evaluation reports the share of tokens
 * routed to an expert on their current GPU).
 *   local[l] = #{ n : placement[l][tr[l][n]] == placement[l+1][tr[l+1][n]] }
 * so the objective equals N_valid*(L-1) - sum_l local[l].  A transition with an invalid
 * expert id at either end is not counted.
 * ---------------------------------------------------------------------------------- */
void ref_placement_locality(const int32_t* trace, const int32_t* placement, int L, int64_t N,
                            int E, int64_t* local_per_pair)
{
    for (int l = 0; l + 1 < L; ++l) {
        int64_t c = 0;
        for (int64_t n = 0; n < N; ++n) {
            int32_t i = trace[(int64_t)l * N + n];
            int32_t p = trace[(int64_t)(l + 1) * N + n];
            if (i < 0 || i >= E || p < 0 || p >= E) continue;
            if (placement[(int64_t)l * E + i] == placement[(int64_t)(l + 1) * E + p]) c += 1;
        }
        local_per_pair[l] = c;
    }
}

/* The same numerators from the E x E counts: sum of counts over expert pairs that share a
 * device.  An independent route to the statistic. */
void ref_placement_locality_from_counts(const int64_t* counts, const int32_t* placement, int L,
                                        int E, int64_t* local_per_pair)
{
    for (int l = 0; l + 1 < L; ++l) {
        int64_t c = 0;
        for (int i = 0; i < E; ++i)
            for (int p = 0; p < E; ++p)
                if (placement[(int64_t)l * E + i] == placement[(int64_t)(l + 1) * E + p])
                    c += counts[((int64_t)l * E + i) * E + p];
        local_per_pair[l] = c;
    }
}

/* -------------------------------------------------------------------------------------
 * Cross-GPU token transfers of a routing trace (Design, "Token Context Coherence in Expert
 * Parallelism": the walk-through of the 3-layer example; Table "Comparison with state-of-the-art
 * GPT MoE optimization methods": p = ratio of tokens involved in the Alltoall).
 *   away[l]  = #{ n : placement[l][tr[l][n]] != home[n] }   tokens whose layer-l expert is not on
 *              the GPU that owns their request
 * Vanilla expert parallelism sends such a token out and back at every layer: 2 * sum_l away[l]
 * transfers.  With coherent contexts a token travels from its home to the first expert and then
 * only when consecutive experts sit on different GPUs: away[0] + sum_l (transitions - local[l])
 * with local[l] of ref_placement_locality.  Entries with an invalid expert id are not counted.
 * ---------------------------------------------------------------------------------- */
void ref_routing_away(const int32_t* trace, const int32_t* placement, const int32_t* home, int L,
                      int64_t N, int E, int64_t* away_per_layer)
{
    for (int l = 0; l < L; ++l) {
        int64_t c = 0;
        for (int64_t n = 0; n < N; ++n) {
            int32_t e = trace[(int64_t)l * N + n];
            if (e < 0 || e >= E) continue;
            if (placement[(int64_t)l * E + e] != home[n]) c += 1;
        }
        away_per_layer[l] = c;
    }
}

/* -------------------------------------------------------------------------------------
 * Forward communication volume (Table "Comparison with state-of-the-art GPT MoE optimization
 * methods"), in tokens.  G GPUs, N tokens per GPU, L MoE layers; p = ratio of tokens involved in
 * an Alltoall, p* = the same ratio with coherent contexts and an affinity placement.
 *   row "Deepspeed-MoE": top-1  2 G N L p        top-2  4 G N L p
 *   row "ExFlow":        top-1  G N (L p* + G)   top-2  G N (2 L p* + G)
 * The table's entries written out as they stand: vol[0..3] in that order.
 * ---------------------------------------------------------------------------------- */
void ref_comm_volume(int G, int64_t N, int L, double p, double p_star, double* vol)
{
    double g = (double)G, n = (double)N, l = (double)L;
    vol[0] = 2.0 * g * n * l * p;
    vol[1] = 4.0 * g * n * l * p;
    vol[2] = g * n * (l * p_star + g);
    vol[3] = g * n * (2.0 * l * p_star + g);
}

/* The two ratios of a trace (Design, "Token Context Coherence in Expert Parallelism"), by walking
 * every token as the walk-through does: a vanilla token leaves home (and returns) at every layer
 * whose expert is elsewhere; a coherent context moves when the GPU of its next expert differs from
 * where it is.  ratios[0] = p = away visits / (N L), ratios[1] = p* = moves / (N L).  Expert ids
 * must be valid. */
void ref_transfer_ratios(const int32_t* trace, const int32_t* placement, const int32_t* home, int L,
                         int64_t N, int E, double* ratios)
{
    int64_t away = 0, moves = 0;
    for (int64_t n = 0; n < N; ++n) {
        int32_t at = home[n];
        for (int l = 0; l < L; ++l) {
            int32_t gpu = placement[(int64_t)l * E + trace[(int64_t)l * N + n]];
            if (gpu != home[n]) away += 1;
            if (gpu != at) moves += 1;
            at = gpu;
        }
    }
    ratios[0] = (double)away / ((double)N * (double)L);
    ratios[1] = (double)moves / ((double)N * (double)L);
}

/* -------------------------------------------------------------------------------------
 * Affinity across several layers (appendix "Extend Expert Affinity to Cross Multiple Layers":
 * the affinity of layer l's experts to the experts of ALL following layers).  The same count
 * as ref_affinity_counts for every ordered pair of layers l < l':
 *   counts[p(l,l')][i][j] = #{ n : tr[l][n] == i and tr[l'][n] == j },  both ids valid,
 * pairs numbered source layer first:  p(l,l') = l*L - l*(l+1)/2 + (l' - l - 1).
 * ---------------------------------------------------------------------------------- */
void ref_affinity_counts_multihop(const int32_t* trace, int L, int64_t N, int E, int64_t* counts)
{
    int64_t p = 0;
    for (int l = 0; l < L; ++l)
        for (int m = l + 1; m < L; ++m, ++p) {
            int64_t* c = counts + p * E * E;
            for (int64_t i = 0; i < (int64_t)E * E; ++i) c[i] = 0;
            for (int64_t n = 0; n < N; ++n) {
                int32_t a = trace[(int64_t)l * N + n];
                int32_t b = trace[(int64_t)m * N + n];
                if (a < 0 || a >= E || b < 0 || b >= E) continue;
                c[(int64_t)a * E + b] += 1;
            }
        }
}
