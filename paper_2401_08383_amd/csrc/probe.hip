// Measurement probes: a plain streaming copy (calibrates HBM counters and gives the achievable
// copy bandwidth) and a register-resident MFMA loop (achievable bf16 matrix-core rate).
#include "common.hpp"

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
