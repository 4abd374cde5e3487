// moe_gate_topk / moe_topk_from_logits: gate GEMM + softmax + top-k routing.
//
// The gate contraction is skinny (N = E <= 64 outputs per token) and therefore bound by the
// HBM read of x.  bf16: one workgroup takes TB = 16*MT tokens; its NW wavefronts split the
// reduction dimension, each accumulating a [E x TB] block with 16x16x32 bf16 MFMA (experts on
// the MFMA row axis, tokens on the column axis, so that a token's logits sit in 4 lanes).
// The wavefronts' partial blocks are summed through LDS in a fixed order, then one thread per
// token does softmax and selection in fp32.  fp32 inputs (tiny configuration) use one
// wavefront per token with wavefront reductions.
#include <math.h>

#include "common.hpp"

namespace exf {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;

struct Route {
    int i0, i1;
    float w0, w1;
};

// Softmax weights of the selected experts from the two best logits and sum exp(l - l0).
__device__ __forceinline__ void route_weights(Route& r, float l0, float l1, float sum_exp, int k, int renormalize)
{
    if (k == 1) {
        r.w0 = 1.0f / sum_exp;
        r.w1 = 0.0f;
    } else {
        const float t = expf(l1 - l0);
        if (renormalize) {
            const float z = 1.0f + t;
            r.w0 = 1.0f / z;
            r.w1 = t / z;
        } else {
            r.w0 = 1.0f / sum_exp;
            r.w1 = t / sum_exp;
        }
    }
}

// Sequential routing of one token; logit(e) returns its e-th fp32 logit.
template <typename F>
__device__ __forceinline__ Route route_sequential(F logit, int E, int k, int renormalize)
{
    Route r;
    float l0 = logit(0);
    r.i0 = 0;
    for (int e = 1; e < E; ++e) {
        const float v = logit(e);
        if (v > l0) {  // strict: the lowest id wins a tie
            l0 = v;
            r.i0 = e;
        }
    }
    float l1 = 0.0f;
    r.i1 = -1;
    if (k > 1) {
        for (int e = 0; e < E; ++e) {
            if (e == r.i0) continue;
            const float v = logit(e);
            if (r.i1 < 0 || v > l1) {
                l1 = v;
                r.i1 = e;
            }
        }
    }
    float s = 0.0f;
    for (int e = 0; e < E; ++e) s += expf(logit(e) - l0);
    route_weights(r, l0, l1, s, k, renormalize);
    return r;
}

// Wavefront routing: lane e holds logit e (lanes >= E hold -inf).  Every lane returns the result.
__device__ __forceinline__ void wave_argmax(float& v, int& i)
{
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
        const float ov = __shfl_xor(v, off, kWave);
        const int oi = __shfl_xor(i, off, kWave);
        if (ov > v || (ov == v && oi < i)) {
            v = ov;
            i = oi;
        }
    }
}

__device__ __forceinline__ Route route_wave(float my_logit, int E, int k, int renormalize)
{
    const int lane = lane_id();
    const bool live = lane < E;
    Route r;
    float v = live ? my_logit : -INFINITY;
    int i = live ? lane : kWave + lane;
    wave_argmax(v, i);
    const float l0 = v;
    r.i0 = i;
    float l1 = 0.0f;
    r.i1 = -1;
    if (k > 1) {
        v = (live && lane != r.i0) ? my_logit : -INFINITY;
        i = (live && lane != r.i0) ? lane : kWave + lane;
        wave_argmax(v, i);
        l1 = v;
        r.i1 = i;
    }
    const float s = wave_sum(live ? expf(my_logit - l0) : 0.0f);
    route_weights(r, l0, l1, s, k, renormalize);
    return r;
}

__device__ __forceinline__ void store_route(const Route& r, int64_t t, int k, int32_t* __restrict__ topk_idx,
                                            float* __restrict__ topk_w)
{
    topk_idx[t * k] = r.i0;
    topk_w[t * k] = r.w0;
    if (k > 1) {
        topk_idx[t * k + 1] = r.i1;
        topk_w[t * k + 1] = r.w1;
    }
}

// ------------------------------------------------------------------------------------------
// Routing from stored logits: one wavefront per token, lane e reads logits[t][e].
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void topk_from_logits_kernel(const float* __restrict__ logits, int64_t T, int E, int k,
                                                                int renormalize, int32_t* __restrict__ topk_idx,
                                                                float* __restrict__ topk_w)
{
    const int lane = lane_id();
    const int64_t waves = static_cast<int64_t>(gridDim.x) * (blockDim.x / kWave);
    for (int64_t t = static_cast<int64_t>(blockIdx.x) * (blockDim.x / kWave) + threadIdx.x / kWave; t < T; t += waves) {
        const float l = lane < E ? logits[t * E + lane] : 0.0f;
        const Route r = route_wave(l, E, k, renormalize);
        if (lane == 0) store_route(r, t, k, topk_idx, topk_w);
    }
}

// ------------------------------------------------------------------------------------------
// fp32 gate: one wavefront per token; lanes split the reduction dimension.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void gate_f32_kernel(const float* __restrict__ x, const float* __restrict__ wg, int64_t T,
                                                        int d, int E, int k, int renormalize,
                                                        float* __restrict__ logits_out, int32_t* __restrict__ topk_idx,
                                                        float* __restrict__ topk_w)
{
    const int lane = lane_id();
    const int64_t waves = static_cast<int64_t>(gridDim.x) * (blockDim.x / kWave);
    for (int64_t t = static_cast<int64_t>(blockIdx.x) * (blockDim.x / kWave) + threadIdx.x / kWave; t < T; t += waves) {
        const float* xr = x + t * d;
        float mine = 0.0f;
        for (int e = 0; e < E; ++e) {
            const float* wr = wg + static_cast<int64_t>(e) * d;
            float acc = 0.0f;
            for (int c = lane * 4; c < d; c += kWave * 4) {
                const float4 a = *reinterpret_cast<const float4*>(xr + c);
                const float4 b = *reinterpret_cast<const float4*>(wr + c);
                acc = fmaf(a.x, b.x, acc);
                acc = fmaf(a.y, b.y, acc);
                acc = fmaf(a.z, b.z, acc);
                acc = fmaf(a.w, b.w, acc);
            }
            acc = wave_sum(acc);
            if (lane == e) mine = acc;
        }
        if (logits_out != nullptr && lane < E) logits_out[t * E + lane] = mine;
        const Route r = route_wave(mine, E, k, renormalize);
        if (lane == 0) store_route(r, t, k, topk_idx, topk_w);
    }
}

// ------------------------------------------------------------------------------------------
// bf16 gate on the matrix cores.
//   MFMA 16x16x32: A operand lane l = W_gate[expert 16*nt + l%16][k0 + 8*(l/16) .. +7]
//                  B operand lane l = x[token 16*mt + l%16][k0 + 8*(l/16) .. +7]
//                  D lane l, v     = logits(expert 16*nt + 4*(l/16) + v, token 16*mt + l%16)
// ------------------------------------------------------------------------------------------
template <int MT, int NT, int NW>
__global__ __launch_bounds__(NW * 64) void gate_bf16_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ wg,
                                                             int64_t T, int d, int E, int k, int renormalize,
                                                             float* __restrict__ logits_out,
                                                             int32_t* __restrict__ topk_idx, float* __restrict__ topk_w)
{
    constexpr int TB = MT * 16;       // tokens per workgroup
    constexpr int EP = NT * 16;       // padded expert count
    constexpr int TBP = TB + 1;       // padded row of the LDS blocks
    constexpr int SLOTS = NW > 1 ? NW - 1 : 1;
    __shared__ float part[SLOTS][EP][TBP];

    const int lane = lane_id();
    const int wave = threadIdx.x / kWave;
    const int64_t t0 = static_cast<int64_t>(blockIdx.x) * TB;
    const int r16 = lane & 15;
    const int kq = (lane >> 4) * 8;

    // this wavefront's share of the 32-wide reduction steps
    const int steps = (d + 31) / 32;
    const int per = (steps + NW - 1) / NW;
    const int s_begin = wave * per;
    const int s_end = min(steps, s_begin + per);

    const bf16_t* xrow[MT];
    const bf16_t* wrow[NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int64_t t = min(t0 + mt * 16 + r16, T - 1);
        xrow[mt] = x + t * d;
    }
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int e = min(nt * 16 + r16, E - 1);
        wrow[nt] = wg + static_cast<int64_t>(e) * d;
    }

    f32x4_t acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    const bf16x8_t zero8 = {};
#pragma unroll 4  // the loads of four steps go out together: a short batch is a chain of memory round trips otherwise
    for (int s = s_begin; s < s_end; ++s) {
        const int c = s * 32 + kq;
        const bool ok = c < d;  // d % 8 == 0: a group of 8 is entirely inside or outside
        const int cc = ok ? c : 0;
        bf16x8_t a[NT], b[MT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) a[nt] = *reinterpret_cast<const bf16x8_t*>(wrow[nt] + cc);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) b[mt] = *reinterpret_cast<const bf16x8_t*>(xrow[mt] + cc);
        if (!ok) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) b[mt] = zero8;
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[nt], b[mt], acc[mt][nt], 0, 0, 0);
    }

    // sum the wavefronts' partial blocks in a fixed order: slots hold waves 1..NW-1, wave 0 adds them
    if (wave > 0) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    part[wave - 1][nt * 16 + (lane >> 4) * 4 + v][mt * 16 + r16] = acc[mt][nt][v];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int e = nt * 16 + (lane >> 4) * 4 + v;
                    const int tt = mt * 16 + r16;
                    float sum = acc[mt][nt][v];
                    for (int w = 1; w < NW; ++w) sum += part[w - 1][e][tt];
                    part[0][e][tt] = sum;  // same lane read this element: no cross-lane hazard
                }
    }
    __syncthreads();

    if (logits_out != nullptr) {
        const int64_t tokens_here = min(static_cast<int64_t>(TB), T - t0);
        const int n = static_cast<int>(tokens_here) * E;
        float* dst = logits_out + t0 * E;
        for (int i = threadIdx.x; i < n; i += NW * 64) dst[i] = part[0][i % E][i / E];
    }
    if (E > 16) {  // many experts: a wavefront per token, lane e holds expert e
        for (int tt = wave; tt < TB; tt += NW) {
            const int64_t t = t0 + tt;
            if (t < T) {  // (the same for every lane of the wavefront)
                const Route r = route_wave(part[0][min(lane, E - 1)][tt], E, k, renormalize);
                if (lane == 0) store_route(r, t, k, topk_idx, topk_w);
            }
        }
        return;
    }
    for (int tt = threadIdx.x; tt < TB; tt += NW * 64) {
        const int64_t t = t0 + tt;
        if (t < T) {
            const Route r = route_sequential([&](int e) { return part[0][e][tt]; }, E, k, renormalize);
            store_route(r, t, k, topk_idx, topk_w);
        }
    }
}

// ------------------------------------------------------------------------------------------
// bf16 gate with W_gate resident in LDS (used whenever the padded weight fits): a persistent
// workgroup copies W_gate into LDS once (row per expert, 16-byte pieces XOR-swizzled so that the
// 16 lanes of an MFMA row group hit 16 different bank groups); after that every wavefront streams
// its own 16-token tiles over the full reduction dimension - x is read from HBM exactly once, there is no cross-wavefront
// reduction and no barrier in the loop.  A token's logits end up in 4 lanes (l, l^16, l^32,
// l^48), so softmax and top-k need two shuffle steps.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void pick_better(float& v, int& i, float ov, int oi)
{
    if (ov > v || (ov == v && oi < i)) {
        v = ov;
        i = oi;
    }
}

template <int NT, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void gate_bf16_lds_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ wg,
                                                                    int64_t T, int d, int E, int k, int renormalize,
                                                                    float* __restrict__ logits_out, int32_t* __restrict__ topk_idx,
                                                                    float* __restrict__ topk_w)
{
    constexpr int EP = NT * 16;
    // [EP][d/8] 16-byte pieces, row e = expert e (rows past E are zero); inside a row piece c sits at
    // position c ^ (e & swz): the 16 lanes of an MFMA row group (16 consecutive experts, same c) then
    // read 16 different 16-byte bank groups, while the copy from global memory stays row-contiguous.
    extern __shared__ uint4 wlds[];
    const int chunks = d / 8;
    const int swz = min(15, (chunks & -chunks) - 1);  // the XOR must stay inside the row
    const int lane = lane_id();
    const int wave = threadIdx.x / kWave;
    const int r16 = lane & 15, g = lane >> 4;
    const int64_t n_tiles = (T + 15) / 16;
    const int steps = (chunks + 3) / 4;
    const bf16x8_t zero8 = {};
    const int64_t stride = static_cast<int64_t>(gridDim.x) * WAVES;
    int64_t tile = static_cast<int64_t>(blockIdx.x) * WAVES + wave;
    const bool has_work = tile < n_tiles;  // (a wavefront without a tile still helps with the copy)

    // The wavefront walks the batches (PF steps of 32 reduction elements) of its tiles as ONE
    // stream: the PF 16-byte loads of the next batch - of the next tile, if this one is finished -
    // are issued before the MFMAs of the current batch.  Inside a tile the loads are unconditional
    // (indices past the end are clamped; the operand is zeroed when it is used) and a scheduling barrier
    // keeps them in front of the MFMAs, so PF loads per lane are in flight while the matrix cores work;
    // left to itself the compiler sinks every load down to its MFMA.
    constexpr int PF = 4;
    typedef __attribute__((__vector_size__(4 * sizeof(int)))) int i32x4_v;
    auto issue = [&](int64_t tl, int s0, i32x4_v(&b)[PF]) {
        const int64_t t = min(min(tl, n_tiles - 1) * 16 + r16, T - 1);
        const bf16_t* xrow = x + t * d;
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            const int c = min((s0 + u) * 4 + g, chunks - 1);
            b[u] = __builtin_nontemporal_load(reinterpret_cast<const i32x4_v*>(xrow + c * 8));  // x is streamed once
        }
    };
    // DEPTH batches per wavefront are in flight.  With eight or more wavefronts two are enough: at one
    // token tile per wavefront (the launch shape up to 256 * 16 tiles) the batch loop ends when the
    // last x bytes arrive from HBM, however early they were asked for, and more batches in flight
    // only delayed the weight copy.  Four wavefronts keep too little in flight that way (measured:
    // 6 % slower than with four batches and sixteen copy loads per thread).
    constexpr int DEPTH = WAVES <= 4 ? 4 : 2;
    i32x4_v ring[DEPTH][PF];
    int64_t issue_tile = tile;  // issue cursor: the batch the next loads belong to
    int issue_s0 = 0;
    auto issue_next = [&](i32x4_v(&b)[PF]) {
        if (issue_tile >= n_tiles) return;  // past this wavefront's last tile: nothing will read the batch
        issue(issue_tile, issue_s0, b);
        issue_s0 += PF;
        if (issue_s0 >= steps) {
            issue_s0 = 0;
            issue_tile += stride;
        }
    };
    // W_gate -> LDS, FB 16-byte loads in flight per thread (a plain loop runs one at a time).  The
    // loads of the first round are issued first and the first x batches right behind them, so both
    // travel at once and the weights, which every wavefront waits for, arrive first.
    const uint4* wg16 = reinterpret_cast<const uint4*>(wg);
    const int total = EP * chunks, valid = E * chunks;
    constexpr int FB = WAVES <= 4 ? 16 : 8;
    auto fill_store = [&](int i, const uint4& v) {
        if (i >= total) return;
        const int e = i / chunks, c = i - e * chunks;
        wlds[e * chunks + (c ^ (e & swz))] = i < valid ? v : uint4{0u, 0u, 0u, 0u};
    };
    {
        uint4 v[FB];
#pragma unroll
        for (int u = 0; u < FB; ++u) v[u] = wg16[min(static_cast<int>(threadIdx.x) + u * WAVES * 64, valid - 1)];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q = 0; q < DEPTH - 1; ++q) issue_next(ring[q]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < FB; ++u) fill_store(threadIdx.x + u * WAVES * 64, v[u]);
    }
    for (int base = threadIdx.x + WAVES * 64 * FB; base < total; base += WAVES * 64 * FB) {
        uint4 v[FB];
#pragma unroll
        for (int u = 0; u < FB; ++u) v[u] = wg16[min(base + u * WAVES * 64, valid - 1)];
#pragma unroll
        for (int u = 0; u < FB; ++u) fill_store(base + u * WAVES * 64, v[u]);
    }
    __syncthreads();
    if (!has_work) return;
    int s0 = 0;
    f32x4_t acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    bool done = false;
    while (!done) {
#pragma unroll
      for (int q = 0; q < DEPTH; ++q) {
        if (done) break;
        i32x4_v(&cur)[PF] = ring[q];
        const bool last_batch = s0 + PF >= steps;
        const int64_t tile_next = last_batch ? tile + stride : tile;
        const int s0_next = last_batch ? 0 : s0 + PF;
        issue_next(ring[(q + DEPTH - 1) % DEPTH]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            const int c = (s0 + u) * 4 + g;
            bf16x8_t bv;
            __builtin_memcpy(&bv, &cur[u], sizeof(bv));
            if (c >= chunks) bv = zero8;
            const int cl = min(c, chunks - 1);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const uint4 wv = wlds[(nt * 16 + r16) * chunks + (cl ^ (r16 & swz))];
                bf16x8_t a;
                __builtin_memcpy(&a, &wv, sizeof(a));
                acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bv, acc[nt], 0, 0, 0);
            }
        }
        if (last_batch) {
        // this lane: token tile*16 + r16, experts nt*16 + 4g + v (ascending in (nt, v))
        float l0 = -INFINITY;
        int i0 = 2 * kWave;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int e = nt * 16 + 4 * g + v;
                if (e < E) pick_better(l0, i0, acc[nt][v], e);
            }
        pick_better(l0, i0, __shfl_xor(l0, 16, kWave), __shfl_xor(i0, 16, kWave));
        pick_better(l0, i0, __shfl_xor(l0, 32, kWave), __shfl_xor(i0, 32, kWave));
        float l1 = -INFINITY;
        int i1 = 2 * kWave;
        if (k > 1) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int e = nt * 16 + 4 * g + v;
                    if (e < E && e != i0) pick_better(l1, i1, acc[nt][v], e);
                }
            pick_better(l1, i1, __shfl_xor(l1, 16, kWave), __shfl_xor(i1, 16, kWave));
            pick_better(l1, i1, __shfl_xor(l1, 32, kWave), __shfl_xor(i1, 32, kWave));
        }
        float se = 0.0f;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (nt * 16 + 4 * g + v < E) se += expf(acc[nt][v] - l0);
        se += __shfl_xor(se, 16, kWave);
        se += __shfl_xor(se, 32, kWave);
        const int64_t tok = tile * 16 + r16;
        if (tok < T) {
            if (logits_out != nullptr) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int e = nt * 16 + 4 * g + v;
                        if (e < E) logits_out[tok * E + e] = acc[nt][v];
                    }
            }
            if (g == 0) {
                Route r;
                r.i0 = i0;
                r.i1 = i1;
                route_weights(r, l0, l1, se, k, renormalize);
                store_route(r, tok, k, topk_idx, topk_w);
            }
        }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        if (tile_next >= n_tiles) done = true;
        }  // last batch of the tile
        tile = tile_next;
        s0 = s0_next;
      }
    }
}

constexpr size_t kGateLdsLimit = 128 * 1024;

template <int NT>
static int launch_gate_bf16_lds(const void* x, const void* wg, int64_t T, int d, int E, int k, int renormalize, float* logits_out,
                                int32_t* topk_idx, float* topk_w, hipStream_t stream)
{
    const size_t lds = static_cast<size_t>(NT) * 16 * d * 2;
    const int64_t n_tiles = (T + 15) / 16;
    // persistent workgroups, one per CU (more when the weight copy is small); 4 to 16 wavefronts
    // each, chosen so that about 256 workgroups take part
    const int per_cu = static_cast<int>(lds <= 32 * 1024 ? 4 : (lds <= 64 * 1024 ? 2 : 1));
    const int waves = n_tiles >= 256 * 16 ? 16 : (n_tiles >= 256 * 8 ? 8 : 4);
    int64_t blocks = (n_tiles + waves - 1) / waves;
    if (blocks > 256 * per_cu) blocks = 256 * per_cu;
#define EXF_LAUNCH_GATE_LDS(W)                                                                                                   \
    do {                                                                                                                        \
        auto kern = gate_bf16_lds_kernel<NT, W>;                                                                                \
        if (lds > 64 * 1024) {                                                                                                  \
            hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, \
                                                 static_cast<int>(lds));                                                       \
            if (err != hipSuccess) return fail(EXF_ERR_HIP, "moe_gate_topk: LDS attribute: %s", hipGetErrorString(err));         \
        }                                                                                                                       \
        hipLaunchKernelGGL(kern, dim3(static_cast<unsigned>(blocks)), dim3(W * 64), lds, stream, static_cast<const bf16_t*>(x),  \
                           static_cast<const bf16_t*>(wg), T, d, E, k, renormalize, logits_out, topk_idx, topk_w);              \
    } while (0)
    if (waves == 16) EXF_LAUNCH_GATE_LDS(16);
    else if (waves == 8) EXF_LAUNCH_GATE_LDS(8);
    else EXF_LAUNCH_GATE_LDS(4);
#undef EXF_LAUNCH_GATE_LDS
    return EXF_OK;
}

template <int MT, int NT, int NW>
static void launch_gate_bf16(const void* x, const void* wg, int64_t T, int d, int E, int k, int renormalize,
                             float* logits_out, int32_t* topk_idx, float* topk_w, hipStream_t stream)
{
    const int64_t blocks = (T + MT * 16 - 1) / (MT * 16);
    hipLaunchKernelGGL((gate_bf16_kernel<MT, NT, NW>), dim3(static_cast<unsigned>(blocks)), dim3(NW * 64), 0, stream,
                       static_cast<const bf16_t*>(x), static_cast<const bf16_t*>(wg), T, d, E, k, renormalize, logits_out,
                       topk_idx, topk_w);
}

template <int NT>
static void dispatch_gate_bf16(const void* x, const void* wg, int64_t T, int d, int E, int k, int renormalize,
                               float* logits_out, int32_t* topk_idx, float* topk_w, hipStream_t stream)
{
    // Tokens per workgroup: as many as still leave >= 512 workgroups (2 per CU); a short batch
    // with a long reduction dimension gets 16 wavefronts per workgroup instead.
    if (T >= 64 * 512)
        launch_gate_bf16<4, NT, 4>(x, wg, T, d, E, k, renormalize, logits_out, topk_idx, topk_w, stream);
    else if (T >= 32 * 512)
        launch_gate_bf16<2, NT, 4>(x, wg, T, d, E, k, renormalize, logits_out, topk_idx, topk_w, stream);
    else if (T >= 16 * 128 || d < 2048)
        launch_gate_bf16<1, NT, 4>(x, wg, T, d, E, k, renormalize, logits_out, topk_idx, topk_w, stream);
    else
        launch_gate_bf16<1, NT, 16>(x, wg, T, d, E, k, renormalize, logits_out, topk_idx, topk_w, stream);
}

static int validate_topk_args(const char* fn, int64_t T, int E, int k)
{
    if (T < 0) return fail(EXF_ERR_BAD_SHAPE, "%s: T = %lld < 0", fn, static_cast<long long>(T));
    if (E < 1 || E > EXF_MAX_EXPERTS) return fail(EXF_ERR_BAD_SHAPE, "%s: E = %d outside [1,%d]", fn, E, EXF_MAX_EXPERTS);
    if (k < 1 || k > EXF_MAX_TOPK || k > E)
        return fail(EXF_ERR_BAD_SHAPE, "%s: k = %d outside [1,min(E,%d)]", fn, k, EXF_MAX_TOPK);
    if (T * k >= (1ll << 31)) return fail(EXF_ERR_BAD_SHAPE, "%s: T*k must be below 2^31", fn);
    return EXF_OK;
}

}  // namespace exf

extern "C" int moe_gate_topk(const void* x, const void* w_gate, int64_t T, int d, int E, int k, int renormalize, int dt,
                             float* logits_out, int32_t* topk_idx, float* topk_w, void* stream)
{
    using namespace exf;
    if (dt != EXF_F32 && dt != EXF_BF16) return fail(EXF_ERR_BAD_DTYPE, "moe_gate_topk: dt = %d", dt);
    if (int rc = validate_topk_args("moe_gate_topk", T, E, k)) return rc;
    const int gran = dt == EXF_BF16 ? 8 : 4;
    if (d < gran || d % gran != 0)
        return fail(EXF_ERR_BAD_SHAPE, "moe_gate_topk: d = %d must be a positive multiple of %d", d, gran);
    if (T == 0) return EXF_OK;
    EXF_REQUIRE_PTR(x);
    EXF_REQUIRE_PTR(w_gate);
    EXF_REQUIRE_PTR(topk_idx);
    EXF_REQUIRE_PTR(topk_w);
    EXF_REQUIRE_ALIGNED(x);
    EXF_REQUIRE_ALIGNED(w_gate);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dt == EXF_F32) {
        const int64_t blocks = (T + 3) / 4;
        hipLaunchKernelGGL(gate_f32_kernel, dim3(static_cast<unsigned>(blocks < 65536 ? blocks : 65536)), dim3(256), 0, s,
                           static_cast<const float*>(x), static_cast<const float*>(w_gate), T, d, E, k, renormalize,
                           logits_out, topk_idx, topk_w);
    } else {
        const int nt = (E + 15) / 16;
        // long batches: W_gate resident in LDS; short ones: the split-K kernel (more workgroups)
        if (static_cast<size_t>(nt) * 16 * d * 2 <= kGateLdsLimit && T >= 16384) {
            int rc = EXF_OK;
            switch (nt) {
                case 1: rc = launch_gate_bf16_lds<1>(x, w_gate, T, d, E, k, renormalize, logits_out, topk_idx, topk_w, s); break;
                case 2: rc = launch_gate_bf16_lds<2>(x, w_gate, T, d, E, k, renormalize, logits_out, topk_idx, topk_w, s); break;
                case 3: rc = launch_gate_bf16_lds<3>(x, w_gate, T, d, E, k, renormalize, logits_out, topk_idx, topk_w, s); break;
                default: rc = launch_gate_bf16_lds<4>(x, w_gate, T, d, E, k, renormalize, logits_out, topk_idx, topk_w, s); break;
            }
            if (rc != EXF_OK) return rc;
            return check_launch("moe_gate_topk");
        }
        switch (nt) {
            case 1: dispatch_gate_bf16<1>(x, w_gate, T, d, E, k, renormalize, logits_out, topk_idx, topk_w, s); break;
            case 2: dispatch_gate_bf16<2>(x, w_gate, T, d, E, k, renormalize, logits_out, topk_idx, topk_w, s); break;
            case 3: dispatch_gate_bf16<3>(x, w_gate, T, d, E, k, renormalize, logits_out, topk_idx, topk_w, s); break;
            default: dispatch_gate_bf16<4>(x, w_gate, T, d, E, k, renormalize, logits_out, topk_idx, topk_w, s); break;
        }
    }
    return check_launch("moe_gate_topk");
}

extern "C" int moe_topk_from_logits(const float* logits, int64_t T, int E, int k, int renormalize, int32_t* topk_idx,
                                    float* topk_w, void* stream)
{
    using namespace exf;
    if (int rc = validate_topk_args("moe_topk_from_logits", T, E, k)) return rc;
    if (T == 0) return EXF_OK;
    EXF_REQUIRE_PTR(logits);
    EXF_REQUIRE_PTR(topk_idx);
    EXF_REQUIRE_PTR(topk_w);
    const int64_t blocks = (T + 3) / 4;
    hipLaunchKernelGGL(topk_from_logits_kernel, dim3(static_cast<unsigned>(blocks < 65536 ? blocks : 65536)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), logits, T, E, k, renormalize, topk_idx, topk_w);
    return check_launch("moe_topk_from_logits");
}
