/*
 * exflow_moe.h — C ABI of the MI355X (gfx950) library for the single-GPU hot path of
 * context-coherent Mixture-of-Experts inference with inter-layer expert affinity
 * (arXiv 2401.08383).
 *
 * Three groups of calls:
 *   MoE expert layer  : moe_gate_topk -> moe_dispatch -> moe_expert_ffn -> moe_combine, or
 *                       moe_gate_topk -> moe_dispatch (index maps only) -> moe_expert_ffn_fused
 *   affinity statistic: affinity_histogram, placement_locality (both in one pass: affinity_statistics),
 *                       affinity_multihop, routing_transfers
 *   placement search  : placement_locality_from_counts (GPU scoring), exf_placement_search (host)
 *
 * Conventions that hold for every call
 *   - Returns EXF_OK (0) or a negative EXF_ERR_* code; exf_last_error() gives the text of the
 *     last failure on the calling thread.  No exception crosses the boundary.
 *   - All argument validation happens on the host BEFORE anything is enqueued, so a call that
 *     returns an error has launched nothing and touched no buffer.
 *   - Pointers are DEVICE pointers unless a comment says "host".  The caller owns every
 *     buffer; the library allocates nothing, frees nothing and keeps no pointer after the
 *     call returns.  Scratch memory is the caller's `workspace` (size from the matching
 *     *_workspace_bytes function, 256-byte aligned).
 *   - Arrays are dense row-major.  Activation / weight pointers must be 16-byte aligned and
 *     the reduction dimension is contiguous for every weight matrix.
 *   - Calls enqueue on `stream` (a hipStream_t passed as void*, NULL = the default stream)
 *     and return without synchronising; results are valid once the stream has been
 *     synchronised.  Data-dependent sizes (tokens per expert) never return to the host.
 *   - T == 0 / N == 0 is valid: nothing is read, counters and offsets are still written.
 *   - dt selects the storage type of activations and weights together: EXF_F32 or EXF_BF16.
 *     Accumulation is always fp32.
 *   - Expert ids that fall outside [0,E) in topk_idx or trace cannot be rejected on the host;
 *     the kernels skip them (see each call).
 */
#ifndef EXFLOW_MOE_H
#define EXFLOW_MOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EXF_OK 0
#define EXF_ERR_NULL_PTR (-1)
#define EXF_ERR_BAD_SHAPE (-2)
#define EXF_ERR_BAD_DTYPE (-3)
#define EXF_ERR_WORKSPACE_TOO_SMALL (-4)
#define EXF_ERR_HIP (-5)
#define EXF_ERR_NOT_IMPLEMENTED (-6)
#define EXF_ERR_MISALIGNED (-7)

#define EXF_F32 0
#define EXF_BF16 1

#define EXF_ACT_GELU_ERF 0  /* z/2 * (1 + erf(z/sqrt 2)) */
#define EXF_ACT_GELU_TANH 1 /* z/2 * (1 + tanh(sqrt(2/pi) (z + 0.044715 z^3))) */

#define EXF_MAX_EXPERTS 64   /* gate width E, local experts E_local and trace alphabet E */
#define EXF_MAX_TOPK 2
#define EXF_DISPATCH_STATIC_MAX_ASSIGNMENTS (1ll << 20)  /* largest T*k of moe_dispatch_static */
#define EXF_MAX_TRACE_LAYERS 256

/* Library version (major*10000 + minor*100 + patch). */
int exf_version(void);

/* Text of the last error raised on this thread ("" if none).  Host pointer, owned by the
 * library, valid until the next failing call on the same thread. */
const char* exf_last_error(void);

/* ---------------------------------------------------------------------------------------
 * moe_gate_topk — gate GEMM, softmax and top-k routing of one MoE layer.
 * (Background, "Gating Strategies and Optimizations": softmax-based gating; Challenges,
 *  "Data Locality": the gate decides each token's destination expert; Experimental setup:
 *  top-1 gating with variable token capacity — no token is dropped or padded.  Table 1
 *  carries the top-2 case.)
 *
 *   logits[t][e] = sum_c x[t][c] * w_gate[e][c]          (fp32 accumulation)
 *   p[t][:]      = softmax(logits[t][:])                 (fp32)
 *   slot j of token t = the j-th largest logit, ties to the LOWEST expert id; slot 0 is best
 *   topk_w[t][j] = p[t][e_j]                             if k == 1 or renormalize == 0
 *                = p[t][e_j] / sum_j' p[t][e_j']         otherwise
 *
 *   x        [T,d]  dt          w_gate [E,d] dt
 *   logits_out [T,E] fp32, may be NULL
 *   topk_idx [T,k] int32        topk_w [T,k] fp32
 * Shapes: T >= 0, 1 <= E <= EXF_MAX_EXPERTS, 1 <= k <= min(E, EXF_MAX_TOPK),
 *         d >= 8 and d % 8 == 0 (bf16) / d % 4 == 0 (fp32).  Inputs must be finite.
 * ------------------------------------------------------------------------------------- */
int moe_gate_topk(const void* x, const void* w_gate, int64_t T, int d, int E, int k,
                  int renormalize, int dt, float* logits_out, int32_t* topk_idx, float* topk_w,
                  void* stream);

/* Selection and weights only, from given fp32 logits [T,E] (same rule as above).  Because
 * it starts from stored logits its indices are a pure function of its input. */
int moe_topk_from_logits(const float* logits, int64_t T, int E, int k, int renormalize,
                         int32_t* topk_idx, float* topk_w, void* stream);

/* ---------------------------------------------------------------------------------------
 * moe_dispatch — group the token-to-expert assignments by expert ("token dispatch",
 * Challenges, "Data Locality") as a STABLE counting sort, and gather the token rows into
 * expert-contiguous order.
 *
 * Assignment a = t*k + j carries global expert id g = topk_idx[a].
 *   local id e = expert_map ? expert_map[g] : g.
 *   g outside [0,E), e < 0 (expert lives on another GPU) or e >= E_local: the assignment is
 *   not kept, sorted_of_src[a] = -1.
 * Kept assignments are ordered by (e, a).  With S = number kept = expert_offsets[E_local]:
 *   expert_counts  [E_local]    tokens per local expert
 *   expert_offsets [E_local+1]  exclusive scan of the counts
 *   src_of_sorted  [A]          sorted position s -> a           (entries s >= S untouched)
 *   sorted_of_src  [A]          a -> sorted position or -1
 *   x_sorted       [A,d] dt     x_sorted[s] = x[src_of_sorted[s] / k]   (rows s >= S untouched);
 *                               may be NULL to skip the row gather (then x may be NULL too)
 * Shapes: A = T*k < 2^31, 1 <= k <= EXF_MAX_TOPK, 1 <= E_local <= EXF_MAX_EXPERTS, E >= 1,
 *         d % 8 == 0 (bf16) / d % 4 == 0 (fp32).
 * expert_map [E] int32 or NULL (identity: e = g, so an id >= E_local is not kept).
 * workspace: moe_dispatch_workspace_bytes(T, k, E_local) bytes.
 * ------------------------------------------------------------------------------------- */
size_t moe_dispatch_workspace_bytes(int64_t T, int k, int E_local);
int moe_dispatch(const void* x, const int32_t* topk_idx, const int32_t* expert_map, int64_t T, int d,
                 int k, int E, int E_local, int dt, void* x_sorted, int32_t* src_of_sorted,
                 int32_t* sorted_of_src, int32_t* expert_counts, int32_t* expert_offsets,
                 void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * moe_dispatch_static — moe_dispatch for callers that cannot allocate or supply scratch memory:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, outputs and validation as moe_dispatch without the workspace pair; the per-chunk
 * expert counts live in a device array built into the library (256 KiB per GPU, held until the
 * process ends).  Limit: T*k <= EXF_DISPATCH_STATIC_MAX_ASSIGNMENTS, EXF_ERR_BAD_SHAPE beyond it.
 * The call allocates and frees nothing.  All calls on one GPU share that array: calls that overlap
 * on one GPU (different streams, different threads) race and must be serialised by the caller;
 * successive calls on one stream are safe, nothing has to be cleared in between.
 * ------------------------------------------------------------------------------------- */
int moe_dispatch_static(const void* x, const int32_t* topk_idx, const int32_t* expert_map, int64_t T,
                        int d, int k, int E, int E_local, int dt, void* x_sorted,
                        int32_t* src_of_sorted, int32_t* sorted_of_src, int32_t* expert_counts,
                        int32_t* expert_offsets, void* stream);

/* ---------------------------------------------------------------------------------------
 * moe_expert_ffn — every local expert applies its feed-forward network to the rows routed
 * to it (Introduction and Challenges: experts are context-free FFNs).
 *
 * For sorted row s with expert_offsets[e] <= s < expert_offsets[e+1]:
 *   h[u] = act( sum_c x_sorted[s][c] * w1[e][u][c] + b1[e][u] )     u < f
 *   y[s][v] =   sum_u h[u] * w2[e][v][u] + b2[e][v]                 v < d
 * Rows s >= expert_offsets[E_local] are not written.  expert_offsets is read on the device;
 * the host never learns the per-expert sizes.  A must be an upper bound on
 * expert_offsets[E_local] (normally T*k).
 *
 *   x_sorted [A,d] dt;  w1 [E_local,f,d] dt;  w2 [E_local,d,f] dt;
 *   b1 [E_local,f] dt or NULL;  b2 [E_local,d] dt or NULL;  y_sorted [A,d] dt.
 * bf16: the hidden activations are rounded to bf16 once, between the two contractions.
 * Shapes: d, f multiples of 64 (bf16) / 4 (fp32); 1 <= E_local <= EXF_MAX_EXPERTS.
 * workspace: moe_expert_ffn_workspace_bytes(A, d, f, E_local, dt) bytes (the hidden activations of
 * A rows of f values; bf16: in a layout of the library's own in which every expert starts on a 32-row
 * boundary - A + 32 E_local rows -, plus 16 MiB for the partial sums of remainder tiles that are cut
 * along the reduction).
 * ------------------------------------------------------------------------------------- */
size_t moe_expert_ffn_workspace_bytes(int64_t A, int d, int f, int E_local, int dt);
int moe_expert_ffn(const void* x_sorted, const int32_t* expert_offsets, const void* w1, const void* b1,
                   const void* w2, const void* b2, int64_t A, int d, int f, int E_local, int act,
                   int dt, void* y_sorted, void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * moe_expert_ffn_fused — expert FFN and gate-weighted combine on the tokens where they lie
 * (the same mathematics as moe_expert_ffn followed by moe_combine; Background, "Expert Model").
 * The first contraction reads row src_of_sorted[s] / k of x for sorted row s, so moe_dispatch
 * can be called with x_sorted = NULL (index-only) and no sorted copy of the activations exists.
 * With k = 1 the second contraction multiplies its fp32 result by the token's gate weight and
 * writes it to the token's own row of `out` (one rounding to dt); rows of tokens whose
 * assignment was not kept (sorted_of_src[t] < 0) are set to zero.  With k > 1 the second
 * contraction writes sorted rows into the workspace and the combine kernel follows.
 *
 *   out[t][:] = sum_{j<k, sorted_of_src[t*k+j] >= 0} topk_w[t][j] * FFN_{e(t,j)}( x[t][:] )
 *
 *   x [T,d] dt;  src_of_sorted [T*k], sorted_of_src [T*k], expert_offsets [E_local+1] as
 *   written by moe_dispatch;  topk_w [T,k] fp32;  weights and biases as for moe_expert_ffn;
 *   out [T,d] dt, must not overlap x.  Shapes as for moe_expert_ffn (d, f multiples of 64 for
 *   bf16, of 4 for fp32).
 * workspace: moe_expert_ffn_fused_workspace_bytes(T, k, d, f, E_local, dt) bytes.
 * ------------------------------------------------------------------------------------- */
size_t moe_expert_ffn_fused_workspace_bytes(int64_t T, int k, int d, int f, int E_local, int dt);
int moe_expert_ffn_fused(const void* x, const int32_t* src_of_sorted, const int32_t* sorted_of_src,
                         const float* topk_w, const int32_t* expert_offsets, const void* w1,
                         const void* b1, const void* w2, const void* b2, int64_t T, int k, int d, int f,
                         int E_local, int act, int dt, void* out, void* workspace,
                         size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * moe_combine — gate-weighted combination of the expert outputs (Background, "Expert
 * Model": a soft gate combines the experts' outputs).
 *   out[t][:] = sum_{j<k} topk_w[t][j] * y_sorted[ sorted_of_src[t*k+j] ][:]   (j ascending,
 *   fp32 accumulation, one rounding to dt); assignments with position -1 contribute nothing.
 *   y_sorted [A,d] dt; sorted_of_src [T*k] int32; topk_w [T,k] fp32; out [T,d] dt.
 * ------------------------------------------------------------------------------------- */
int moe_combine(const void* y_sorted, const int32_t* sorted_of_src, const float* topk_w, int64_t T,
                int d, int k, int dt, void* out, void* stream);

/* ---------------------------------------------------------------------------------------
 * affinity_histogram — inter-layer expert affinity from a routing trace (Design, "Modeling
 * Inter-layer Expert Affinity", the conditional-probability equation; the heat-map figure).
 *
 *   trace [L,N] int32, layer-major: trace[l][n] = expert of token n at MoE layer l (top-1).
 *   counts[l][i][p] = #{ n : trace[l][n] = i and trace[l+1][n] = p }       int64 [L-1,E,E]
 *   loads [l][i]    = #{ n : trace[l][n] = i }                             int64 [L,E], may be NULL
 *   cond_prob[l][i][p] = counts[l][i][p] / sum_p' counts[l][i][p'], 0 for an empty row
 *                        — P(expert p at layer l+1 | expert i at layer l)  fp32 [L-1,E,E], may be NULL
 *   n_invalid[0]    = number of trace entries outside [0,E)                int64 [1], may be NULL
 * A transition with an invalid id at either end is not counted.  Outputs are overwritten,
 * not accumulated.  Shapes: 1 <= L <= EXF_MAX_TRACE_LAYERS, N >= 0, 1 <= E <= EXF_MAX_EXPERTS.
 * workspace: affinity_histogram_workspace_bytes(L, N, E) bytes.
 * ------------------------------------------------------------------------------------- */
size_t affinity_histogram_workspace_bytes(int L, int64_t N, int E);
int affinity_histogram(const int32_t* trace, int L, int64_t N, int E, int64_t* counts, int64_t* loads,
                       float* cond_prob, int64_t* n_invalid, void* workspace, size_t workspace_bytes,
                       void* stream);

/* ---------------------------------------------------------------------------------------
 * affinity_multihop — the co-routing counts of EVERY ordered layer pair l < m (appendix "Extend
 * Expert Affinity to Cross Multiple Layers": a layer's expert affinity to all following layers).
 *   counts     int64 [L(L-1)/2, E, E]  counts[p(l,m)][i][j] = #{ n : trace[l][n] == i and
 *                                      trace[m][n] == j }, both ids valid; pairs numbered source
 *                                      layer first: p(l,m) = l*L - l*(l+1)/2 + (m - l - 1)
 *   cond_prob  fp32, same shape, optional (NULL): counts / row sum, 0 for an empty row
 * Nothing is written when L == 1.  Shapes as affinity_histogram.
 * workspace: affinity_multihop_workspace_bytes(L, N, E) bytes (per-chunk partial histograms).
 * ------------------------------------------------------------------------------------- */
size_t affinity_multihop_workspace_bytes(int L, int64_t N, int E);
int affinity_multihop(const int32_t* trace, int L, int64_t N, int E, int64_t* counts, float* cond_prob,
                      void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * placement_locality — how many layer-to-layer transitions stay on the device that holds
 * the token, for a given expert-to-device placement (Design, "Solving Affinity's duality by
 * Integer Programming": the objective sums the crossing indicators R over tokens and the
 * L-1 transitions; Evaluation, "Reduced Cross-GPU Token Routing": the share of tokens routed
 * to experts on their current GPU).
 *
 *   placement [L,E] int32: device (GPU or node) of expert e at layer l, any value in [0,G).
 *   local_per_pair[l] = #{ n : placement[l][trace[l][n]] == placement[l+1][trace[l+1][n]] }
 *                                                                           int64 [L-1]
 * so the objective equals N*(L-1) - sum(local_per_pair) and the locality fraction is
 * sum(local_per_pair) / (N*(L-1)), both formed by the caller.  Transitions with an invalid
 * expert id are not counted.  The map is scored as given; exf_check_placement tests the
 * load-balance and exclusivity constraints.
 * workspace: placement_locality_workspace_bytes(L, N) bytes.
 * ------------------------------------------------------------------------------------- */
size_t placement_locality_workspace_bytes(int L, int64_t N);
int placement_locality(const int32_t* trace, const int32_t* placement, int L, int64_t N, int E, int G,
                       int64_t* local_per_pair, void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * affinity_statistics — affinity_histogram and the locality numerators of placement_locality
 * from ONE pass over the trace (same passages as those two calls).  The locality numerator of a
 * layer pair is a function of its co-routing counts,
 *   local_per_pair[l] = sum_{i,p} counts[l][i][p] * [ placement[l][i] == placement[l+1][p] ],
 * so the launch that sums the per-chunk histograms adds it up as well and the trace is not read
 * a second time.  Outputs, shapes and the treatment of invalid ids are those of the two calls;
 * loads, cond_prob and n_invalid may be NULL; local_per_pair [L-1] int64 is overwritten.
 * workspace: affinity_statistics_workspace_bytes(L, N, E) bytes.
 * ------------------------------------------------------------------------------------- */
size_t affinity_statistics_workspace_bytes(int L, int64_t N, int E);
int affinity_statistics(const int32_t* trace, const int32_t* placement, int L, int64_t N, int E, int G,
                        int64_t* counts, int64_t* loads, float* cond_prob, int64_t* n_invalid,
                        int64_t* local_per_pair, void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * routing_transfers — the cross-GPU token transfers of a routing trace under a placement
 * (Design, "Token Context Coherence in Expert Parallelism": the walk-through that counts 4 and 6
 * transfers for vanilla expert parallelism against 3 and 1 with coherent contexts; the table
 * "Comparison with state-of-the-art GPT MoE optimization methods": p, the ratio of tokens
 * involved in the Alltoall).  One pass over the trace yields
 *   local_per_pair[l]  as placement_locality                                    int64 [L-1]
 *   away_per_layer[l] = #{ n : placement[l][trace[l][n]] != home[n] }           int64 [L]
 * where home [N] int32 (device) is the GPU that owns the request of token n (any values).
 * Vanilla expert parallelism moves 2 * sum_l away_per_layer[l] tokens; with coherent contexts
 * the count is away_per_layer[0] + sum_l (valid transitions of pair l - local_per_pair[l]).
 * Entries with an invalid expert id are not counted.  (The per-destination send buffer itself
 * is moe_dispatch with expert_map = the placement row of the layer and E_local = G: rows come
 * out grouped by destination GPU, stable, with the send counts in expert_counts.)
 * workspace: routing_transfers_workspace_bytes(L, N) bytes.  local_per_pair may be NULL if L == 1.
 * ------------------------------------------------------------------------------------- */
size_t routing_transfers_workspace_bytes(int L, int64_t N);
int routing_transfers(const int32_t* trace, const int32_t* placement, const int32_t* home, int L,
                      int64_t N, int E, int G, int64_t* local_per_pair, int64_t* away_per_layer,
                      void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * exf_comm_volume — the forward communication volume model of the table "Comparison with
 * state-of-the-art GPT MoE optimization methods" (host helper, pure arithmetic).
 *   G   GPUs of the expert-parallel group          N  tokens per GPU
 *   L   MoE layers                                 p  ratio of tokens that take part in an Alltoall
 *   p_star  the same ratio under context-coherent expert parallelism with an affinity placement
 * volumes_host (HOST, out, 4 doubles, in tokens):
 *   [0] vanilla expert parallelism, top-1 gating   2 * G * N * L * p       (out and back per layer)
 *   [1] vanilla, top-2 gating                      4 * G * N * L * p
 *   [2] context-coherent, top-1                    G * N * (L * p_star + G)  (one Alltoall per layer
 *                                                   plus the AllGather of the contexts: the + G term)
 *   [3] context-coherent, top-2                    G * N * (2 * L * p_star + G)
 * Requires G >= 1, N >= 0, L >= 1, 0 <= p, p_star <= 1; EXF_ERR_BAD_SHAPE otherwise.
 *
 * exf_transfer_ratios — p and p_star of a trace from the counters routing_transfers returns (HOST
 * copies), for a trace of `tokens` tokens without invalid ids (Design, "Token Context Coherence in
 * Expert Parallelism": vanilla moves a token out and back whenever its expert is not at home, a
 * coherent context moves from home to its first expert and then only between GPUs that differ):
 *   p      = sum_l away_per_layer[l] / (tokens * L)
 *   p_star = (away_per_layer[0] + sum_l (tokens - local_per_pair[l])) / (tokens * L)
 * so that 2*G*N*L*p and G*N*L*p_star with G*N = tokens are exactly the two transfer counts.
 * local_per_pair_host may be NULL when L == 1.  tokens >= 1, L >= 1.
 * ------------------------------------------------------------------------------------- */
int exf_comm_volume(int G, int64_t N, int L, double p, double p_star, double* volumes_host);
int exf_transfer_ratios(const int64_t* away_per_layer_host, const int64_t* local_per_pair_host, int L,
                        int64_t tokens, double* p_host, double* p_star_host);

/* Host helper: placement is a HOST array [L,E].  Returns EXF_OK iff every entry is in [0,G)
 * and every device holds exactly E/G experts of every layer (the load-balance and
 * exclusivity constraints of the integer program); EXF_ERR_BAD_SHAPE otherwise. */
int exf_check_placement(const int32_t* placement_host, int L, int E, int G);

/* ---------------------------------------------------------------------------------------
 * Placement search driven by the statistic (Design, "Solving Affinity's duality by Integer
 * Programming": minimise the crossing transitions under the load-balance and exclusivity
 * constraints; "Staged Experts Affinity": first between nodes, then between the GPUs of a node).
 * In terms of the co-routing counts a map keeps
 *     local[l] = sum_{i,p} counts[l][i][p] * [ placement[l][i] == placement[l+1][p] ]
 * transitions of layer pair l local; the objective of the integer program is the total number
 * of counted transitions minus sum_l local[l].
 *
 * placement_locality_from_counts (GPU): scores a batch of B candidate maps.
 *   counts      device int64 [L-1,E,E]   (as written by affinity_histogram)
 *   placements  device int32 [B,L,E]     any values; maps are scored as given
 *   local       device int64 [B,L-1]     out; exact integer sums
 *   Nothing is written when B == 0 or L == 1.  1 <= L <= EXF_MAX_TRACE_LAYERS,
 *   1 <= E <= EXF_MAX_EXPERTS, 0 <= B <= 2^24.  Asynchronous on `stream`, no workspace.
 *
 * exf_placement_search (host): counts_host is a HOST array [L-1,E,E] of non-negative counts;
 *   placement_host [L,E] (HOST, out) receives the GPU of every expert, GPUs numbered so that node
 *   = gpu / (G / nodes).  Requires nodes | G | E.  Stage 1 partitions the experts of every layer
 *   over the nodes, stage 2 partitions every node's experts over its GPUs using the transitions
 *   that stay inside the node.  A stage is solved exactly (dynamic programme over the chain of
 *   layers) when a layer has at most 128 balanced partitions, otherwise by a greedy
 *   layer-by-layer assignment refined by pairwise swaps, best of `restarts` (>= 1) starts drawn
 *   from `seed`.  The result always satisfies exf_check_placement.  Deterministic for given
 *   arguments.  The paper names no solver; this one is this library's own.
 * ------------------------------------------------------------------------------------- */
int placement_locality_from_counts(const int64_t* counts, const int32_t* placements, int B, int L,
                                   int E, int64_t* local, void* stream);
int exf_placement_search(const int64_t* counts_host, int L, int E, int G, int nodes, int restarts,
                         uint64_t seed, int32_t* placement_host);

#ifdef __cplusplus
}
#endif
#endif /* EXFLOW_MOE_H */
