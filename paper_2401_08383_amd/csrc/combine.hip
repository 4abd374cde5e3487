// moe_combine: out[t] = sum_j topk_w[t][j] * y_sorted[sorted_of_src[t*k+j]], fp32 accumulation,
// one rounding to the storage type.  A pure stream: every thread owns 16-byte chunks of output
// rows; all the loads of an unrolled group are issued before the arithmetic.
#include "common.hpp"

namespace exf {

template <int K, bool BF16>
__global__ __launch_bounds__(256) void combine_kernel(const uint4* __restrict__ y, const int32_t* __restrict__ sorted_of_src,
                                                       const float* __restrict__ topk_w, int64_t T, int vec_per_row, int64_t A,
                                                       uint4* __restrict__ out)
{
    constexpr int U = 4;
    const int64_t total = T * vec_per_row;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
    for (int64_t i0 = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i0 < total; i0 += U * stride) {
        uint4 v[U][K];
        float w[U][K];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = i0 + u * stride;
            const bool live = i < total;
            const int64_t t = live ? i / vec_per_row : 0;
            const int c = live ? static_cast<int>(i - t * vec_per_row) : 0;
#pragma unroll
            for (int j = 0; j < K; ++j) {
                const int s = live ? sorted_of_src[t * K + j] : -1;
                const bool ok = s >= 0 && s < A;
                w[u][j] = ok ? topk_w[t * K + j] : 0.0f;
                v[u][j] = ok ? y[static_cast<int64_t>(s) * vec_per_row + c] : uint4{0u, 0u, 0u, 0u};
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = i0 + u * stride;
            if (i >= total) continue;
            uint4 r;
            if constexpr (BF16) {
                float acc[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) acc[q] = 0.0f;
#pragma unroll
                for (int j = 0; j < K; ++j) {
                    const uint32_t p[4] = {v[u][j].x, v[u][j].y, v[u][j].z, v[u][j].w};
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        acc[2 * q] = fmaf(w[u][j], __uint_as_float(p[q] << 16), acc[2 * q]);
                        acc[2 * q + 1] = fmaf(w[u][j], __uint_as_float(p[q] & 0xffff0000u), acc[2 * q + 1]);
                    }
                }
                r.x = pack_bf16x2(acc[0], acc[1]);
                r.y = pack_bf16x2(acc[2], acc[3]);
                r.z = pack_bf16x2(acc[4], acc[5]);
                r.w = pack_bf16x2(acc[6], acc[7]);
            } else {
                float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int j = 0; j < K; ++j) {
                    acc[0] = fmaf(w[u][j], __uint_as_float(v[u][j].x), acc[0]);
                    acc[1] = fmaf(w[u][j], __uint_as_float(v[u][j].y), acc[1]);
                    acc[2] = fmaf(w[u][j], __uint_as_float(v[u][j].z), acc[2]);
                    acc[3] = fmaf(w[u][j], __uint_as_float(v[u][j].w), acc[3]);
                }
                r = uint4{__float_as_uint(acc[0]), __float_as_uint(acc[1]), __float_as_uint(acc[2]), __float_as_uint(acc[3])};
            }
            out[i] = r;
        }
    }
}

}  // namespace exf

extern "C" int moe_combine(const void* y_sorted, const int32_t* sorted_of_src, const float* topk_w, int64_t T, int d, int k,
                           int dt, void* out, void* stream)
{
    using namespace exf;
    if (dt != EXF_F32 && dt != EXF_BF16) return fail(EXF_ERR_BAD_DTYPE, "moe_combine: dt = %d", dt);
    if (T < 0) return fail(EXF_ERR_BAD_SHAPE, "moe_combine: T = %lld < 0", static_cast<long long>(T));
    if (k < 1 || k > EXF_MAX_TOPK) return fail(EXF_ERR_BAD_SHAPE, "moe_combine: k = %d outside [1,%d]", k, EXF_MAX_TOPK);
    if (T * k >= (1ll << 31)) return fail(EXF_ERR_BAD_SHAPE, "moe_combine: T*k must be below 2^31");
    const int gran = dt == EXF_BF16 ? 8 : 4;
    if (d < gran || d % gran != 0)
        return fail(EXF_ERR_BAD_SHAPE, "moe_combine: d = %d must be a positive multiple of %d", d, gran);
    if (T == 0) return EXF_OK;
    EXF_REQUIRE_PTR(y_sorted);
    EXF_REQUIRE_PTR(sorted_of_src);
    EXF_REQUIRE_PTR(topk_w);
    EXF_REQUIRE_PTR(out);
    EXF_REQUIRE_ALIGNED(y_sorted);
    EXF_REQUIRE_ALIGNED(out);
    const int vec_per_row = d / gran;
    const int64_t A = T * k;
    const int64_t total = T * vec_per_row;
    int64_t blocks = (total + 256 * 4 - 1) / (256 * 4);
    if (blocks > 256 * 16) blocks = 256 * 16;
    const dim3 grid(static_cast<unsigned>(blocks)), block(256);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint4* y = static_cast<const uint4*>(y_sorted);
    uint4* o = static_cast<uint4*>(out);
    if (dt == EXF_BF16) {
        if (k == 1)
            hipLaunchKernelGGL((combine_kernel<1, true>), grid, block, 0, s, y, sorted_of_src, topk_w, T, vec_per_row, A, o);
        else
            hipLaunchKernelGGL((combine_kernel<2, true>), grid, block, 0, s, y, sorted_of_src, topk_w, T, vec_per_row, A, o);
    } else {
        if (k == 1)
            hipLaunchKernelGGL((combine_kernel<1, false>), grid, block, 0, s, y, sorted_of_src, topk_w, T, vec_per_row, A, o);
        else
            hipLaunchKernelGGL((combine_kernel<2, false>), grid, block, 0, s, y, sorted_of_src, topk_w, T, vec_per_row, A, o);
    }
    return check_launch("moe_combine");
}
