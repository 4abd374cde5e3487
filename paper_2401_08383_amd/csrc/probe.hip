// Measurement probes: a plain streaming copy (calibrates HBM counters and gives the achievable
// copy bandwidth), a register-resident MFMA loop (achievable bf16 matrix-core rate) and a bare GEMM
// K loop over caller-supplied operands (what the matrix cores sustain while operands stream through
// LDS - which depends on the operand VALUES: the chip holds a power limit, not a clock).
#include "common.hpp"
#include "exflow_probe.h"

namespace exf {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

__global__ __launch_bounds__(256) void probe_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int64_t n)
{
    const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
    int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    for (; i + 3 * stride < n; i += 4 * stride) {
        uint4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = load_stream16(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < 4; ++u) store_stream16(dst + i + u * stride, v[u]);
    }
    for (; i < n; i += stride) dst[i] = src[i];
}

// Every wavefront issues `iters` rounds of four independent 32x32x16 bf16 MFMAs.
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, float* __restrict__ out)
{
    bf16x8_t a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = static_cast<__bf16>(1.0f + 0.001f * static_cast<float>(threadIdx.x % 7 + i));
        b[i] = static_cast<__bf16>(0.5f + 0.001f * static_cast<float>(threadIdx.x % 5 + i));
    }
    f32x16_t c0 = {}, c1 = {}, c2 = {}, c3 = {};
    for (int it = 0; it < iters; ++it) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
    out[static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x] = s;
}

// A bare K loop: 256 workgroups (one per compute unit) of 4 wavefronts walk 256x256 output tiles of
// 8 "experts" (1024 x 1024 activations, 4096 x 1024 weights each, bf16, reduction contiguous) with
// 256x256x64 K tiles: direct-to-LDS loads of the next K tile spread between the MFMAs of the
// current one, two LDS stages, XOR-swizzled 16-byte chunks, one barrier per K tile, 128x128 per
// wavefront (16 MFMAs per K step).  No epilogue; a checksum keeps the loop alive.
__device__ __forceinline__ void probe_dma_16B(const unsigned char* base, uint32_t voff, uint32_t lds_addr)
{
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1\n" : : "v"(voff), "s"(base), "s"(lds_addr) : "memory");
#else
    (void)base; (void)voff; (void)lds_addr;
#endif
}
__device__ __forceinline__ const unsigned char* probe_uniform(const unsigned char* p)
{
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v));
    const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v >> 32));
    return reinterpret_cast<const unsigned char*>((static_cast<uint64_t>(hi) << 32) | lo);
}
constexpr int kLoopExperts = 8, kLoopRows = 1024, kLoopCols = 4096, kLoopK = 1024;
constexpr size_t kLoopActBytes = static_cast<size_t>(kLoopExperts) * kLoopRows * kLoopK * 2;
constexpr size_t kLoopWgtBytes = static_cast<size_t>(kLoopExperts) * kLoopCols * kLoopK * 2;

__global__ __launch_bounds__(256, 1) void probe_gemm_loop_kernel(const unsigned char* __restrict__ act,
                                                                  const unsigned char* __restrict__ wgt, int passes,
                                                                  float* __restrict__ out)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    constexpr int RB = 128, STAGE = 512 * RB, ROW = kLoopK * 2;  // LDS tile row, stage, operand row in bytes
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    f32x16_t acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
    int frag_off[4];
    {
        const int row = lane & 31, swz = (row >> 1) & 7;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) frag_off[ks] = row * RB + (((2 * ks + (lane >> 5)) ^ swz) * 16);
    }
    const int act_base = wm * 128 * RB, wgt_base = (256 + wn * 128) * RB;
    // wavefronts 0,1 load the 256 activation rows of a K tile, wavefronts 2,3 the 256 weight rows
    uint32_t off[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int row = ((wave & 1) * 16 + i) * 8 + lane / 8;
        off[i] = row * ROW + ((lane % 8) ^ ((row >> 1) & 7)) * 16;
    }
    const uint32_t smem_addr = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) unsigned char*)smem));
    const uint32_t my_lds = (wave < 2 ? 0 : 256 * RB) + (wave & 1) * 16 * 1024;
    const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
    int it = 0;
    for (int pass = 0; pass < passes; ++pass) {
        for (int half = 0; half < 2; ++half) {
            const int s2 = slot + half * 32;                          // 64 tiles per XCD and pass
            const int t = ((s2 / 32) * 8 + xcd) * 32 + s2 % 32;       // chunks of 32 consecutive tiles per XCD
            const int e = t / 64, in_e = t % 64;
            const int ct = (in_e / 32) * 8 + (in_e % 32) / 4, rt = in_e % 4;  // blocks of 4 row x 8 column tiles
            const unsigned char* my_base =
                probe_uniform(wave < 2 ? act + (static_cast<size_t>(e) * kLoopRows + rt * 256) * ROW
                                       : wgt + (static_cast<size_t>(e) * kLoopCols + ct * 256) * ROW);
#pragma unroll
            for (int i = 0; i < 16; ++i) probe_dma_16B(my_base, off[i], smem_addr + (it & 1) * STAGE + my_lds + i * 1024);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            for (int kt = 0; kt < kLoopK / 64; ++kt, ++it) {
                const unsigned char* stage = smem + (it & 1) * STAGE;
                const uint32_t dst = smem_addr + ((it + 1) & 1) * STAGE + my_lds;
                const unsigned char* gsrc = my_base + (kt + 1) * 128;
                const unsigned char* pw = stage + wgt_base;
                const unsigned char* pa = stage + act_base;
                bf16x8_t fa[2][4], fb[2][4];
#pragma unroll
                for (int a = 0; a < 4; ++a) fa[0][a] = *reinterpret_cast<const bf16x8_t*>(pw + a * 32 * RB + frag_off[0]);
#pragma unroll
                for (int b = 0; b < 4; ++b) fb[0][b] = *reinterpret_cast<const bf16x8_t*>(pa + b * 32 * RB + frag_off[0]);
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    const int cur = ks & 1, nxt = cur ^ 1;
#pragma unroll
                    for (int m = 0; m < 16; ++m) {
                        if (ks < 3 && m % 2 == 0) {
                            const int r = m / 2;
                            if (r < 4) fa[nxt][r] = *reinterpret_cast<const bf16x8_t*>(pw + r * 32 * RB + frag_off[ks < 3 ? ks + 1 : 0]);
                            else fb[nxt][r - 4] = *reinterpret_cast<const bf16x8_t*>(pa + (r - 4) * 32 * RB + frag_off[ks < 3 ? ks + 1 : 0]);
                        }
                        acc[m / 4][m % 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][m / 4], fb[cur][m % 4], acc[m / 4][m % 4], 0, 0, 0);
                        __builtin_amdgcn_sched_barrier(0);
                        if (kt + 1 < kLoopK / 64 && ks < 2 && (m & 1)) {
                            const int i = ks * 8 + m / 2;
                            probe_dma_16B(gsrc, off[i], dst + i * 1024);
                            __builtin_amdgcn_sched_barrier(0);
                        }
                    }
                }
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                __syncthreads();
            }
        }
    }
    float s = 0;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) s += acc[a][b][0];
    out[static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x] = s;
}

}  // namespace exf

extern "C" int exf_probe_copy(void* dst, const void* src, size_t bytes, void* stream)
{
    using namespace exf;
    if (bytes == 0) return EXF_OK;
    EXF_REQUIRE_PTR(dst);
    EXF_REQUIRE_PTR(src);
    EXF_REQUIRE_ALIGNED(dst);
    EXF_REQUIRE_ALIGNED(src);
    if (bytes % 16 != 0) return fail(EXF_ERR_BAD_SHAPE, "exf_probe_copy: bytes must be a multiple of 16");
    const int64_t n = static_cast<int64_t>(bytes / 16);
    int64_t blocks = (n + 256 * 4 - 1) / (256 * 4);
    if (blocks > kStreamWorkgroups) blocks = kStreamWorkgroups;
    hipLaunchKernelGGL(probe_copy_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4*>(src), static_cast<uint4*>(dst), n);
    return check_launch("exf_probe_copy");
}

extern "C" int exf_probe_mfma(int workgroups, int iters, float* out, void* stream)
{
    using namespace exf;
    if (workgroups < 1 || workgroups > 65536 || iters < 1) return fail(EXF_ERR_BAD_SHAPE, "exf_probe_mfma: bad launch shape");
    EXF_REQUIRE_PTR(out);
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(stream), iters, out);
    return check_launch("exf_probe_mfma");
}

extern "C" size_t exf_probe_gemm_loop_bytes(void) { return exf::kLoopActBytes + exf::kLoopWgtBytes; }

extern "C" int exf_probe_gemm_loop(const void* operands, size_t bytes, int passes, float* out, void* stream)
{
    using namespace exf;
    if (passes < 1 || passes > 100000) return fail(EXF_ERR_BAD_SHAPE, "exf_probe_gemm_loop: passes = %d", passes);
    if (bytes < kLoopActBytes + kLoopWgtBytes)
        return fail(EXF_ERR_WORKSPACE_TOO_SMALL, "exf_probe_gemm_loop: %zu < %zu operand bytes", bytes, kLoopActBytes + kLoopWgtBytes);
    EXF_REQUIRE_PTR(operands);
    EXF_REQUIRE_PTR(out);
    EXF_REQUIRE_ALIGNED(operands);
    constexpr int lds = 2 * 512 * 128;
    hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(probe_gemm_loop_kernel),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (err != hipSuccess) return fail(EXF_ERR_HIP, "exf_probe_gemm_loop: LDS attribute: %s", hipGetErrorString(err));
    const unsigned char* base = static_cast<const unsigned char*>(operands);
    hipLaunchKernelGGL(probe_gemm_loop_kernel, dim3(256), dim3(256), lds, static_cast<hipStream_t>(stream), base, base + kLoopActBytes,
                       passes, out);
    return check_launch("exf_probe_gemm_loop");
}
