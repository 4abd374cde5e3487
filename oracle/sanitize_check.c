/* Memory-safety driver for the CPU oracle (TEST INFRASTRUCTURE, like the oracle itself).
 *
 * Linked with moe_oracle.c into one executable that is built with
 *   gcc -O1 -g -fopenmp -fsanitize=address,undefined -fno-sanitize-recover=all
 * and calls every oracle function on small ragged shapes with exactly-sized heap buffers, including
 * the edge cases of the method (no tokens, one layer, invalid expert ids, experts mapped to -1,
 * empty experts, top-2).  Any out-of-bounds access, use of an uninitialised index or undefined
 * integer operation ends the run with a non-zero status.  It checks no values: the pins do that.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void ref_gate_logits(const float*, const float*, int64_t, int, int, double*);
void ref_softmax(const double*, int64_t, int, double*);
void ref_topk(const double*, int64_t, int, int, int, int32_t*, double*);
int64_t ref_dispatch(const int32_t*, const int32_t*, int64_t, int, int, int, int32_t*, int32_t*, int32_t*, int32_t*, int64_t*);
void ref_gather_rows(const float*, const int32_t*, int64_t, int, int, float*);
void ref_expert_ffn_rows(const float*, const int32_t*, const float*, const float*, const float*, const float*, int, int, int, int,
                         const int64_t*, int64_t, double*);
void ref_combine(const double*, const int32_t*, const double*, int64_t, int, int, double*);
void ref_affinity_counts(const int32_t*, int, int64_t, int, int64_t*, int64_t*, int64_t*);
void ref_cond_prob(const int64_t*, int, int, double*);
void ref_placement_locality(const int32_t*, const int32_t*, int, int64_t, int, int64_t*);
void ref_placement_locality_from_counts(const int64_t*, const int32_t*, int, int, int64_t*);
void ref_routing_away(const int32_t*, const int32_t*, const int32_t*, int, int64_t, int, int64_t*);
void ref_comm_volume(int, int64_t, int, double, double, double*);
void ref_transfer_ratios(const int32_t*, const int32_t*, const int32_t*, int, int64_t, int, double*);
void ref_affinity_counts_multihop(const int32_t*, int, int64_t, int, int64_t*);

static uint64_t state = 88172645463325252ull;
static uint32_t rnd(void)
{
    state ^= state << 13;
    state ^= state >> 7;
    state ^= state << 17;
    return (uint32_t)(state >> 16);
}
static float rndf(void) { return (float)(rnd() % 2001) / 1000.0f - 1.0f; }
static void* buf(size_t n, size_t elem) { return calloc(n ? n : 1, elem); } /* n = 0: a valid pointer nobody may read */
static float* fbuf(size_t n)
{
    float* p = buf(n, sizeof(float));
    for (size_t i = 0; i < n; ++i) p[i] = rndf();
    return p;
}

static void layer_case(int64_t T, int d, int f, int E, int E_local, int k, int with_map, int with_bias, int act, int bad_ids)
{
    const int64_t A = T * k;
    float *x = fbuf((size_t)T * d), *wg = fbuf((size_t)E * d);
    double *logits = buf((size_t)T * E, sizeof(double)), *prob = buf((size_t)T * E, sizeof(double));
    int32_t* idx = buf((size_t)A, sizeof(int32_t));
    double* w = buf((size_t)A, sizeof(double));
    ref_gate_logits(x, wg, T, d, E, logits);
    ref_softmax(logits, T, E, prob);
    ref_topk(logits, T, E, k, k > 1, idx, w);
    if (bad_ids)
        for (int64_t a = 0; a < A; a += 5) idx[a] = (a % 2) ? E + 3 : -1;
    int32_t* map = NULL;
    if (with_map) {
        map = buf((size_t)E, sizeof(int32_t));
        for (int e = 0; e < E; ++e) map[e] = (e % 3 == 2) ? -1 : e % E_local;
    }
    int32_t *src = buf((size_t)A, sizeof(int32_t)), *inv = buf((size_t)A, sizeof(int32_t));
    int32_t *cnt = buf((size_t)E_local, sizeof(int32_t)), *off = buf((size_t)E_local + 1, sizeof(int32_t));
    int64_t n_inv = 0;
    const int64_t kept = ref_dispatch(idx, map, T, k, E, E_local, src, inv, cnt, off, &n_inv);
    float* xs = buf((size_t)kept * d, sizeof(float));
    ref_gather_rows(x, src, kept, k, d, xs);
    float *w1 = fbuf((size_t)E_local * f * d), *w2 = fbuf((size_t)E_local * d * f);
    float *b1 = with_bias ? fbuf((size_t)E_local * f) : NULL, *b2 = with_bias ? fbuf((size_t)E_local * d) : NULL;
    int64_t* rows = buf((size_t)kept, sizeof(int64_t));
    for (int64_t s = 0; s < kept; ++s) rows[s] = kept - 1 - s; /* any order */
    double* y = buf((size_t)kept * d, sizeof(double));
    ref_expert_ffn_rows(xs, off, w1, b1, w2, b2, d, f, E_local, act, rows, kept, y);
    double* out = buf((size_t)T * d, sizeof(double));
    ref_combine(y, inv, w, T, d, k, out);
    free(x); free(wg); free(logits); free(prob); free(idx); free(w); free(map); free(src); free(inv); free(cnt); free(off);
    free(xs); free(w1); free(w2); free(b1); free(b2); free(rows); free(y); free(out);
}

static void trace_case(int L, int64_t N, int E, int G, int bad_ids)
{
    int32_t* tr = buf((size_t)L * N, sizeof(int32_t));
    for (int64_t i = 0; i < (int64_t)L * N; ++i) tr[i] = (int32_t)(rnd() % (uint32_t)E);
    int32_t* clean = buf((size_t)L * N, sizeof(int32_t));
    for (int64_t i = 0; i < (int64_t)L * N; ++i) clean[i] = tr[i];
    if (bad_ids)
        for (int64_t i = 0; i < (int64_t)L * N; i += 7) tr[i] = (i % 2) ? E : -5;
    int32_t* pl = buf((size_t)L * E, sizeof(int32_t));
    for (int i = 0; i < L * E; ++i) pl[i] = (int32_t)(rnd() % (uint32_t)G);
    int32_t* home = buf((size_t)N, sizeof(int32_t));
    for (int64_t n = 0; n < N; ++n) home[n] = (int32_t)(rnd() % (uint32_t)G);
    const int P = L > 1 ? L - 1 : 0;
    int64_t *counts = buf((size_t)P * E * E, sizeof(int64_t)), *loads = buf((size_t)L * E, sizeof(int64_t)), n_inv = 0;
    ref_affinity_counts(tr, L, N, E, counts, loads, &n_inv);
    ref_affinity_counts(tr, L, N, E, counts, NULL, NULL);
    double* prob = buf((size_t)P * E * E, sizeof(double));
    ref_cond_prob(counts, L, E, prob);
    int64_t *loc = buf((size_t)P, sizeof(int64_t)), *loc2 = buf((size_t)P, sizeof(int64_t)), *away = buf((size_t)L, sizeof(int64_t));
    ref_placement_locality(tr, pl, L, N, E, loc);
    ref_placement_locality_from_counts(counts, pl, L, E, loc2);
    ref_routing_away(tr, pl, home, L, N, E, away);
    int64_t* multi = buf((size_t)L * (L - 1) / 2 * E * E, sizeof(int64_t));
    ref_affinity_counts_multihop(tr, L, N, E, multi);
    if (N > 0) {
        double r[2];
        ref_transfer_ratios(clean, pl, home, L, N, E, r);
        double vol[4];
        ref_comm_volume(G, N, L, r[0], r[1], vol);
    }
    free(tr); free(clean); free(pl); free(home); free(counts); free(loads); free(prob); free(loc); free(loc2); free(away); free(multi);
}

int main(void)
{
    layer_case(37, 24, 40, 5, 5, 1, 0, 0, 0, 0);
    layer_case(61, 16, 24, 8, 3, 2, 1, 1, 1, 0);  /* top-2, experts mapped to -1, biases, tanh form */
    layer_case(29, 8, 12, 6, 6, 2, 0, 1, 0, 1);   /* ids outside [0,E) */
    layer_case(33, 8, 8, 8, 3, 1, 0, 0, 0, 0);    /* no map and fewer local experts than ids: the rest is invalid */
    layer_case(1, 4, 4, 1, 1, 1, 0, 0, 0, 0);     /* one token, one expert */
    layer_case(0, 8, 8, 4, 4, 1, 1, 0, 0, 0);     /* no tokens */
    layer_case(9, 8, 8, 64, 64, 2, 0, 0, 0, 0);   /* far more experts than tokens: empty experts */
    trace_case(4, 103, 7, 3, 0);
    trace_case(6, 57, 64, 8, 1);
    trace_case(1, 20, 4, 2, 0);                   /* one layer: no pair */
    trace_case(3, 0, 8, 4, 0);                    /* no tokens */
    trace_case(2, 1, 1, 1, 0);
    puts("oracle: sanitizer run clean");
    return 0;
}
