// moe_combine: out[t] = sum_j topk_w[t][j] * y_sorted[sorted_of_src[t*k+j]], fp32 accumulation,
// one rounding to the storage type.  A pure stream over the rows.
#include "common.hpp"

namespace exf {

// Rows are handled in batches of `row_batch` (at most 16) consecutive output rows per wavefront: the lanes first
// fetch the batch's source positions and weights with one coalesced load each (so the
// data-dependent addresses are known before any row data is requested), then the wavefront
// streams the batch as a flat sequence of 16-byte chunks, four per lane in flight.
template <int K, bool BF16>
__global__ __launch_bounds__(256) void combine_kernel(const uint4* __restrict__ y, const int32_t* __restrict__ sorted_of_src,
                                                       const float* __restrict__ topk_w, int64_t T, int vec_per_row, int64_t A,
                                                       int row_batch, uint4* __restrict__ out)
{
    constexpr int U = 4;
    const int lane = lane_id();
    const int64_t n_batches = (T + row_batch - 1) / row_batch;
    const int64_t n_waves = static_cast<int64_t>(gridDim.x) * (blockDim.x / kWave);
    const float rcp = 1.0f / static_cast<float>(vec_per_row);
    for (int64_t b = static_cast<int64_t>(blockIdx.x) * (blockDim.x / kWave) + threadIdx.x / kWave; b < n_batches; b += n_waves) {
        const int64_t t0 = b * row_batch;
        const int rows = static_cast<int>(min(static_cast<int64_t>(row_batch), T - t0));
        int pos[K];
        float wt[K];
#pragma unroll
        for (int j = 0; j < K; ++j) {  // lane r < rows holds the K assignments of token t0 + r
            const int s = lane < rows ? sorted_of_src[(t0 + lane) * K + j] : -1;
            const bool ok = s >= 0 && s < A;
            pos[j] = ok ? s : -1;
            wt[j] = ok ? topk_w[(t0 + lane) * K + j] : 0.0f;
        }
        // weighted sum of the K source chunks of one output chunk, rounded once to the storage type
        auto reduce_chunk = [&](const uint4(&vj)[K], const float(&wj)[K]) -> uint4 {
            uint4 r;
            if constexpr (BF16) {
                float acc[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) acc[q] = 0.0f;
#pragma unroll
                for (int j = 0; j < K; ++j) {
                    const uint32_t p[4] = {vj[j].x, vj[j].y, vj[j].z, vj[j].w};
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        acc[2 * q] = fmaf(wj[j], __uint_as_float(p[q] << 16), acc[2 * q]);
                        acc[2 * q + 1] = fmaf(wj[j], __uint_as_float(p[q] & 0xffff0000u), acc[2 * q + 1]);
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
                    acc[0] = fmaf(wj[j], __uint_as_float(vj[j].x), acc[0]);
                    acc[1] = fmaf(wj[j], __uint_as_float(vj[j].y), acc[1]);
                    acc[2] = fmaf(wj[j], __uint_as_float(vj[j].z), acc[2]);
                    acc[3] = fmaf(wj[j], __uint_as_float(vj[j].w), acc[3]);
                }
                r = uint4{__float_as_uint(acc[0]), __float_as_uint(acc[1]), __float_as_uint(acc[2]), __float_as_uint(acc[3])};
            }
            return r;
        };
        const int total = rows * vec_per_row;
        constexpr int kPass = kWave * U;  // output chunks the wavefront produces per pass
        if (total % kPass == 0) {
            // Every lane has a chunk in every pass: no condition anywhere near the loads (a dropped
            // assignment reads row 0 and is zeroed afterwards), and the loads of the next pass are issued
            // before this pass is reduced and stored.
            const int n_pass = total / kPass;
            auto load_pass = [&](int pass, uint4(&v)[U][K], float(&w)[U][K]) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int c = pass * kPass + u * kWave + lane;
                    const int r = row_of_chunk(c, vec_per_row, rcp);
                    const int col = c - r * vec_per_row;
#pragma unroll
                    for (int j = 0; j < K; ++j) {
                        const int s = __shfl(pos[j], r, kWave);
                        w[u][j] = __shfl(wt[j], r, kWave);
                        v[u][j] = load_stream16(y + static_cast<int64_t>(max(s, 0)) * vec_per_row + col);
                        if (s < 0) v[u][j] = uint4{0u, 0u, 0u, 0u};
                    }
                }
            };
            auto store_pass = [&](int pass, const uint4(&v)[U][K], const float(&w)[U][K]) {
#pragma unroll
                for (int u = 0; u < U; ++u)
                    store_stream16(out + t0 * vec_per_row + pass * kPass + u * kWave + lane, reduce_chunk(v[u], w[u]));
            };
            uint4 cur[U][K], nxt[U][K];
            float wcur[U][K], wnxt[U][K];
            load_pass(0, cur, wcur);
            for (int pass = 0; pass + 1 < n_pass; ++pass) {
                load_pass(pass + 1, nxt, wnxt);
                store_pass(pass, cur, wcur);
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int j = 0; j < K; ++j) {
                        cur[u][j] = nxt[u][j];
                        wcur[u][j] = wnxt[u][j];
                    }
            }
            store_pass(n_pass - 1, cur, wcur);
            continue;
        }
        for (int c0 = lane; c0 < total; c0 += kWave * U) {  // ragged batch: every chunk checked
            uint4 v[U][K];
            float w[U][K];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = c0 + u * kWave;
                const bool live = c < total;
                const int r = live ? row_of_chunk(c, vec_per_row, rcp) : 0;
                const int col = c - r * vec_per_row;
#pragma unroll
                for (int j = 0; j < K; ++j) {
                    const int s = __shfl(pos[j], r, kWave);
                    w[u][j] = __shfl(wt[j], r, kWave);
                    v[u][j] = (live && s >= 0) ? load_stream16(y + static_cast<int64_t>(s) * vec_per_row + col) : uint4{0u, 0u, 0u, 0u};
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = c0 + u * kWave;
                if (c >= total) continue;
                const uint4 r = reduce_chunk(v[u], w[u]);
                store_stream16(out + t0 * vec_per_row + c, r);
            }
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
    const int row_batch = row_batch_for(T);
    int64_t blocks = ((T + row_batch - 1) / row_batch + 3) / 4;  // four wavefronts (row batches) per workgroup
    if (blocks > kStreamWorkgroups) blocks = kStreamWorkgroups;
    const dim3 grid(static_cast<unsigned>(blocks)), block(256);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint4* y = static_cast<const uint4*>(y_sorted);
    uint4* o = static_cast<uint4*>(out);
    if (dt == EXF_BF16) {
        if (k == 1)
            hipLaunchKernelGGL((combine_kernel<1, true>), grid, block, 0, s, y, sorted_of_src, topk_w, T, vec_per_row, A, row_batch, o);
        else
            hipLaunchKernelGGL((combine_kernel<2, true>), grid, block, 0, s, y, sorted_of_src, topk_w, T, vec_per_row, A, row_batch, o);
    } else {
        if (k == 1)
            hipLaunchKernelGGL((combine_kernel<1, false>), grid, block, 0, s, y, sorted_of_src, topk_w, T, vec_per_row, A, row_batch, o);
        else
            hipLaunchKernelGGL((combine_kernel<2, false>), grid, block, 0, s, y, sorted_of_src, topk_w, T, vec_per_row, A, row_batch, o);
    }
    return check_launch("moe_combine");
}
