// moe_expert_ffn: grouped expert FFN  y = act(x W1^T + b1) W2^T + b2  over expert-contiguous rows.
//
// Two launches of one grouped "NT" GEMM kernel  C[rows of e, N] = A[rows, K] * B_e[N, K]^T
// (both operands have the reduction dimension contiguous): the first with the bias+GELU
// epilogue writing the hidden activations [A,f] to the workspace, the second writing y.
// The per-expert row ranges are read from expert_offsets ON THE DEVICE: the grid is sized for
// the worst case (ceil(A/MT) + E_local row tiles) and every workgroup locates its own
// (expert, row tile, column tile) with a wavefront scan; surplus workgroups exit at once.
//
// bf16 kernel (gfx950 matrix cores)
//   - macro tile MT x NT x KT, WM x WN wavefronts, each owning (MT/WM) x (NT/WN) as 32x32 MFMA
//     tiles (v_mfma_f32_32x32x16_bf16, fp32 accumulators).
//   - global -> LDS with direct-to-LDS 16-byte loads (no staging registers), STAGES-deep ring,
//     one workgroup barrier per K tile.  A direct-to-LDS load writes 64 lanes x 16 B
//     contiguously, so the LDS layout is fixed; bank conflicts on the MFMA operand reads are
//     avoided by choosing WHICH 16-byte chunk of a row each lane fetches (XOR swizzle applied on
//     the global side).
//   - the weight tile feeds the MFMA row axis and the activation tile the column axis, so a lane
//     ends up with 4 consecutive output columns of one row -> 8-byte bf16 stores.
//   - workgroup -> tile order: consecutive ids go round-robin to the 8 XCDs, so id%8 selects the
//     XCD and every XCD walks a contiguous range of tiles ordered (expert, column tile, row tile):
//     the workgroups resident on one XCD share an expert's activation rows and a few weight
//     panels in that XCD's L2.
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

// erf by the rational-exponential formula 7.1.26 of Abramowitz & Stegun (|error| <= 1.5e-7),
// enough for a result that is rounded to bf16 next.
__device__ __forceinline__ float gelu_erf_fast(float z)
{
    const float x = fabsf(z) * 0.70710678118654752440f;
    const float t = __frcp_rn(fmaf(0.3275911f, x, 1.0f));
    float p = fmaf(1.061405429f, t, -1.453152027f);
    p = fmaf(p, t, 1.421413741f);
    p = fmaf(p, t, -0.284496736f);
    p = fmaf(p, t, 0.254829592f);
    const float erfc_abs = p * t * __expf(-x * x);      // 1 - erf(|z|/sqrt2)
    const float erf_signed = copysignf(1.0f - erfc_abs, z);
    return 0.5f * z * (1.0f + erf_signed);
}
// z/2 (1 + tanh u) = z / (1 + exp(-2u))
__device__ __forceinline__ float gelu_tanh_fast(float z)
{
    const float u = 0.79788456080286535588f * (z + 0.044715f * z * z * z);
    return z * __frcp_rn(1.0f + __expf(-2.0f * u));
}

enum Epilogue { kEpiNone = 0, kEpiGeluErf = 1, kEpiGeluTanh = 2 };

// ---------------------------------------------------------------------------- tile lookup
struct Tile2D {
    int expert;
    int row_begin, row_end;
    int n_tile;
};

// Tiles ordered (expert, column tile, row tile); `idx` is the position in that order.
__device__ __forceinline__ bool locate_tile(const int32_t* __restrict__ offsets, int E_local, int mt, int n_tiles, int max_rows,
                                            int xcd, int slot, Tile2D& out)
{
    const int lane = lane_id();
    int lo = 0, hi = 0;
    if (lane < E_local) {
        lo = min(max(offsets[lane], 0), max_rows);
        hi = min(max(offsets[lane + 1], lo), max_rows);
    }
    const int row_tiles = (hi - lo + mt - 1) / mt;
    const int tiles = row_tiles * n_tiles;
    const int incl = wave_inclusive_scan(tiles);
    const int excl = incl - tiles;
    const int total = __shfl(incl, kWave - 1, kWave);
    const int per_xcd = (total + kXcdCount - 1) / kXcdCount;
    const int idx = xcd * per_xcd + slot;
    if (slot >= per_xcd || idx >= total) return false;
    const unsigned long long m = __ballot(lane < E_local && idx >= excl && idx < incl);
    if (m == 0ull) return false;
    const int src = __ffsll(static_cast<long long>(m)) - 1;
    const int e_lo = __shfl(lo, src, kWave);
    const int e_hi = __shfl(hi, src, kWave);
    const int e_rt = __shfl(row_tiles, src, kWave);
    const int r = idx - __shfl(excl, src, kWave);
    out.expert = src;
    out.n_tile = r / e_rt;
    out.row_begin = e_lo + (r % e_rt) * mt;
    out.row_end = min(out.row_begin + mt, e_hi);
    return true;
}

// ---------------------------------------------------------------------------- bf16 MFMA kernel
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <int MT, int NT, int KT, int STAGES, int WM, int WN, int EPI>
__global__ __launch_bounds__(WM* WN * 64) void grouped_gemm_bf16_kernel(const bf16_t* __restrict__ act,     // [A,K]
                                                                         const int32_t* __restrict__ offsets,
                                                                         const bf16_t* __restrict__ weight,  // [E_local,N,K]
                                                                         const bf16_t* __restrict__ bias,    // [E_local,N] or null
                                                                         int max_rows, int K, int N, int E_local,
                                                                         bf16_t* __restrict__ out)           // [A,N]
{
    constexpr int NWAVES = WM * WN;
    constexpr int RB = KT * 2;              // bytes per tile row
    constexpr int CPR = RB / 16;            // 16-byte chunks per tile row
    constexpr int RPI = 1024 / RB;          // tile rows covered by one wavefront-wide direct-to-LDS load
    constexpr int GROUPS = (MT + NT) / RPI; // load instructions per K tile (whole workgroup)
    constexpr int LPW = GROUPS / NWAVES;    // ... per wavefront
    constexpr int STAGE_BYTES = (MT + NT) * RB;
    constexpr int WTM = MT / WM, WTN = NT / WN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int KSTEPS = KT / 16;
    static_assert(KT == 32 || KT == 64, "row swizzle is written for 64- and 128-byte tile rows");
    static_assert(GROUPS % NWAVES == 0 && MT % RPI == 0 && NT % RPI == 0, "tile must split evenly over the wavefronts");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wavefront tile is made of 32x32 MFMA tiles");
    static_assert((STAGES - 1) * LPW < 64, "outstanding loads must fit the vmcnt counter");

    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    const int lane = lane_id();
    const int wave = threadIdx.x / kWave;
    const int wm = wave / WN, wn = wave % WN;

    Tile2D tile;
    const int n_tiles = (N + NT - 1) / NT;
    if (!locate_tile(offsets, E_local, MT, n_tiles, max_rows, blockIdx.x % kXcdCount, blockIdx.x / kXcdCount, tile)) return;
    const int n0 = tile.n_tile * NT;
    const bf16_t* wexp = weight + static_cast<size_t>(tile.expert) * N * K;

    // ---- per-lane source pointers of this wavefront's direct-to-LDS loads -------------------
    // Group gi covers tile rows [gi*RPI, gi*RPI+RPI); lane -> row gi*RPI + lane/CPR and the
    // 16-byte chunk (lane%CPR) ^ swizzle(row) of that row; it lands at LDS byte gi*1024 + lane*16.
    const bf16_t* src[LPW];
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
        const int gi = wave + i * NWAVES;
        const int row = gi * RPI + lane / CPR;  // row inside the stage: activation rows first, then weight rows
        const int swz = (KT == 64) ? (row & 7) : ((row >> 1) & 3);
        const int chunk = (lane % CPR) ^ swz;
        if (row < MT) {
            const int r = min(tile.row_begin + row, tile.row_end - 1);  // rows past the tile end re-read the last valid row
            src[i] = act + static_cast<size_t>(r) * K + chunk * 8;
        } else {
            const int r = min(n0 + row - MT, N - 1);
            src[i] = wexp + static_cast<size_t>(r) * K + chunk * 8;
        }
    }

    // ---- per-lane LDS byte offsets of the MFMA operand reads -------------------------------
    // operand row = base + lane%32; K step ks uses logical chunk 2*ks + lane/32
    int frag_off[KSTEPS];
    {
        const int row = lane & 31;
        const int swz = (KT == 64) ? (row & 7) : ((row >> 1) & 3);
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) frag_off[ks] = row * RB + (((2 * ks + (lane >> 5)) ^ swz) * 16);
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

    const int nk = K / KT;
    auto issue = [&](int kt) {
        unsigned char* stage = smem + (kt % STAGES) * STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const int gi = wave + i * NWAVES;
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(src[i] + static_cast<size_t>(kt) * KT),
                (__attribute__((address_space(3))) void*)(stage + gi * 1024), 16, 0, 0);
        }
    };

#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s)
        if (s < nk) issue(s);

    for (int kt = 0; kt < nk; ++kt) {
        // K tile kt must have landed; up to STAGES-2 younger tiles may still be in flight
        const int younger = min(nk - 1, kt + STAGES - 2) - kt;
        if constexpr (STAGES >= 4) {
            if (younger >= 2) wait_vmcnt<2 * LPW>();
            else if (younger == 1) wait_vmcnt<LPW>();
            else wait_vmcnt<0>();
        } else if constexpr (STAGES == 3) {
            if (younger >= 1) wait_vmcnt<LPW>();
            else wait_vmcnt<0>();
        } else {
            wait_vmcnt<0>();
        }
        __syncthreads();  // everyone's share of tile kt is in LDS, and everyone is done reading tile kt-1
        if (kt + STAGES - 1 < nk) issue(kt + STAGES - 1);

        const unsigned char* stage = smem + (kt % STAGES) * STAGE_BYTES;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            bf16x8_t fa[TN], fb[TM];
#pragma unroll
            for (int a = 0; a < TN; ++a)
                fa[a] = *reinterpret_cast<const bf16x8_t*>(stage + wgt_base + a * 32 * RB + frag_off[ks]);
#pragma unroll
            for (int b = 0; b < TM; ++b)
                fb[b] = *reinterpret_cast<const bf16x8_t*>(stage + act_base + b * 32 * RB + frag_off[ks]);
#pragma unroll
            for (int a = 0; a < TN; ++a)
#pragma unroll
                for (int b = 0; b < TM; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
        }
    }

    // ---- epilogue: lane holds, for output row m = .. + lane%32, columns n = .. + 8*g + 4*(lane/32) + r ----
    const bf16_t* bexp = bias != nullptr ? bias + static_cast<size_t>(tile.expert) * N : nullptr;
#pragma unroll
    for (int b = 0; b < TM; ++b) {
        const int m = tile.row_begin + wm * WTM + b * 32 + (lane & 31);
        if (m >= tile.row_end) continue;
        bf16_t* orow = out + static_cast<size_t>(m) * N;
#pragma unroll
        for (int a = 0; a < TN; ++a) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = n0 + wn * WTN + a * 32 + g * 8 + (lane >> 5) * 4;
                if (n >= N) continue;  // N % 4 == 0: a group of four is entirely inside or outside
                float v[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float z = acc[a][b][g * 4 + r];
                    if (bexp != nullptr) z += bf16_to_f32(bexp[n + r]);
                    if constexpr (EPI == kEpiGeluErf) z = gelu_erf_fast(z);
                    if constexpr (EPI == kEpiGeluTanh) z = gelu_tanh_fast(z);
                    v[r] = z;
                }
                uint2 packed;
                packed.x = pack_bf16x2(v[0], v[1]);
                packed.y = pack_bf16x2(v[2], v[3]);
                *reinterpret_cast<uint2*>(orow + n) = packed;
            }
        }
    }
}

// ---------------------------------------------------------------------------- fp32 kernel
template <int EPI>
__global__ __launch_bounds__(256) void grouped_gemm_f32_kernel(const float* __restrict__ act, const int32_t* __restrict__ offsets,
                                                                const float* __restrict__ weight, const float* __restrict__ bias,
                                                                int max_rows, int K, int N, int E_local, float* __restrict__ out)
{
    constexpr int MT = 64, NT = 64, KT = 16;
    __shared__ float As[KT][MT + 4];
    __shared__ float Bs[KT][NT + 4];
    const TileRef tile = locate_row_tile(offsets, E_local, MT, blockIdx.x, max_rows);
    if (tile.expert < 0) return;
    const int n0 = blockIdx.y * NT;
    const float* wexp = weight + static_cast<size_t>(tile.expert) * N * K;
    const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
    const int lrow = threadIdx.x / 4, lk = (threadIdx.x % 4) * 4;
    const float* arow = act + static_cast<size_t>(min(tile.row_begin + lrow, tile.row_end - 1)) * K;
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
        float v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float z = acc[i][j];
            if (bexp != nullptr) z += bexp[n + j];
            if constexpr (EPI == kEpiGeluErf) z = gelu_erf_exact(z);
            if constexpr (EPI == kEpiGeluTanh) z = gelu_tanh_exact(z);
            v[j] = z;
        }
        *reinterpret_cast<float4*>(out + static_cast<size_t>(m) * N + n) = make_float4(v[0], v[1], v[2], v[3]);
    }
}

// ---------------------------------------------------------------------------- host launchers
template <int MT, int NT, int KT, int STAGES, int WM, int WN>
static int launch_bf16(const void* act, const int32_t* offsets, const void* weight, const void* bias, int64_t A, int K, int N,
                       int E_local, int epi, void* out, hipStream_t stream)
{
    constexpr size_t lds = static_cast<size_t>(STAGES) * (MT + NT) * KT * 2;
    const int64_t row_tiles = (A + MT - 1) / MT + E_local;
    const int64_t n_tiles = (N + NT - 1) / NT;
    const int64_t ub = row_tiles * n_tiles;
    const int64_t grid = (ub + kXcdCount - 1) / kXcdCount * kXcdCount;
    if (grid >= (1ll << 31)) return fail(EXF_ERR_BAD_SHAPE, "moe_expert_ffn: too many tiles");
#define EXF_LAUNCH_BF16(EPI)                                                                                                    \
    do {                                                                                                                        \
        auto kern = grouped_gemm_bf16_kernel<MT, NT, KT, STAGES, WM, WN, EPI>;                                                  \
        if (lds > 64 * 1024) {                                                                                                  \
            hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, \
                                                 static_cast<int>(lds));                                                       \
            if (err != hipSuccess) return fail(EXF_ERR_HIP, "moe_expert_ffn: LDS attribute: %s", hipGetErrorString(err));       \
        }                                                                                                                       \
        hipLaunchKernelGGL(kern, dim3(static_cast<unsigned>(grid)), dim3(WM* WN * 64), lds, stream,                              \
                           static_cast<const bf16_t*>(act), offsets, static_cast<const bf16_t*>(weight),                        \
                           static_cast<const bf16_t*>(bias), static_cast<int>(A), K, N, E_local, static_cast<bf16_t*>(out));    \
    } while (0)
    if (epi == kEpiNone) EXF_LAUNCH_BF16(kEpiNone);
    else if (epi == kEpiGeluErf) EXF_LAUNCH_BF16(kEpiGeluErf);
    else EXF_LAUNCH_BF16(kEpiGeluTanh);
#undef EXF_LAUNCH_BF16
    return EXF_OK;
}

static int launch_f32(const void* act, const int32_t* offsets, const void* weight, const void* bias, int64_t A, int K, int N,
                      int E_local, int epi, void* out, hipStream_t stream)
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
        hipLaunchKernelGGL(grouped_gemm_f32_kernel<kEpiNone>, grid, dim3(256), 0, stream, a, offsets, w, b, static_cast<int>(A), K, N, E_local, o);
    else if (epi == kEpiGeluErf)
        hipLaunchKernelGGL(grouped_gemm_f32_kernel<kEpiGeluErf>, grid, dim3(256), 0, stream, a, offsets, w, b, static_cast<int>(A), K, N, E_local, o);
    else
        hipLaunchKernelGGL(grouped_gemm_f32_kernel<kEpiGeluTanh>, grid, dim3(256), 0, stream, a, offsets, w, b, static_cast<int>(A), K, N, E_local, o);
    return EXF_OK;
}

}  // namespace exf

extern "C" size_t moe_expert_ffn_workspace_bytes(int64_t A, int d, int f, int E_local, int dt)
{
    (void)d;
    (void)E_local;
    if (A < 0 || f < 1 || (dt != EXF_F32 && dt != EXF_BF16)) return 0;
    const size_t elem = dt == EXF_BF16 ? 2 : 4;
    return exf::align_up(static_cast<size_t>(A > 0 ? A : 1) * static_cast<size_t>(f) * elem, 256);
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
        rc = launch_bf16<128, 128, 64, 2, 2, 2>(x_sorted, expert_offsets, w1, b1, A, d, f, E_local, epi, workspace, s);
        if (rc == EXF_OK)
            rc = launch_bf16<128, 128, 64, 2, 2, 2>(workspace, expert_offsets, w2, b2, A, f, d, E_local, kEpiNone, y_sorted, s);
    }
    if (rc != EXF_OK) return rc;
    return check_launch("moe_expert_ffn");
}
