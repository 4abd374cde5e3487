// Shared host/device helpers of the gfx950 library: error reporting, bf16 conversion,
// wavefront primitives.  Nothing here is used by the CPU checker.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "exflow_moe.h"

namespace exf {

// ---- host side ---------------------------------------------------------------------------
// Records a formatted message for exf_last_error() on this thread and returns `code`.
int fail(int code, const char* fmt, ...);
// Maps the pending HIP launch error (if any) to EXF_ERR_HIP.
int check_launch(const char* what);

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

#define EXF_REQUIRE_PTR(p)                                                        \
    do {                                                                          \
        if ((p) == nullptr) return ::exf::fail(EXF_ERR_NULL_PTR, "%s: %s is NULL", __func__, #p); \
    } while (0)
#define EXF_REQUIRE_ALIGNED(p)                                                    \
    do {                                                                          \
        if (!::exf::aligned16(p))                                                 \
            return ::exf::fail(EXF_ERR_MISALIGNED, "%s: %s is not 16-byte aligned", __func__, #p); \
    } while (0)

constexpr int kWave = 64;  // CDNA wavefront width

// ---- device side -------------------------------------------------------------------------
typedef uint16_t bf16_t;  // storage only; arithmetic is fp32

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(static_cast<uint32_t>(b) << 16); }

// Round-to-nearest-even; inputs are finite by contract (NaN is quieted).
__device__ __forceinline__ bf16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<bf16_t>((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return static_cast<bf16_t>(u >> 16);
}

// Two floats -> two bf16 in one register (gfx950 has a packed round-to-nearest-even convert).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2_v;
    typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_v;
    const f32x2_v f = {lo, hi};
    const bf16x2_v b = __builtin_convertvector(f, bf16x2_v);
    uint32_t u;
    __builtin_memcpy(&u, &b, sizeof(u));
    return u;
}

// 16-byte streaming accesses: data that is touched once should not displace reusable lines.
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4_v;
__device__ __forceinline__ uint4 load_stream16(const uint4* p)
{
    const u32x4_v v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_v*>(p));
    return uint4{v[0], v[1], v[2], v[3]};
}
__device__ __forceinline__ void store_stream16(uint4* p, uint4 x)
{
    const u32x4_v v = {x.x, x.y, x.z, x.w};
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4_v*>(p));
}

// Launch width of the pure streaming kernels: a grid-stride loop over about two workgroups per
// CU sustained the highest HBM rate when measured (many more workgroups were slower).
constexpr int kStreamWorkgroups = 512;

// Row batches of the gather / combine streams (see combine.hip): rows per wavefront batch, chosen
// so that about 2048 wavefronts have work (a short batch keeps a small problem parallel, a long
// one amortises the index fetch), and the row a flat chunk index falls in: c / vec_per_row
// through a float reciprocal with one correction step (c < 2^24).
inline int row_batch_for(int64_t rows)
{
    int b = 16;
    while (b > 1 && rows / b < 2048) b >>= 1;
    return b;
}
__device__ __forceinline__ int row_of_chunk(int c, int vec_per_row, float rcp)
{
    int q = static_cast<int>(static_cast<float>(c) * rcp);
    const int r = c - q * vec_per_row;
    if (r < 0) q -= 1;
    else if (r >= vec_per_row) q += 1;
    return q;
}

__device__ __forceinline__ int lane_id() { return static_cast<int>(threadIdx.x) & (kWave - 1); }

template <typename T>
__device__ __forceinline__ T wave_sum(T v)
{
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// Inclusive prefix sum across the 64 lanes of a wavefront, on the cross-lane data path of the vector
// ALU (a shuffle goes through the LDS pipeline and costs a round trip of its own per step; a tile
// lookup runs several scans in a row before a workgroup can request its first operand).  Steps 1-4 add
// the lanes 1, 2, 4 and 8 to the right inside every row of 16 lanes (zero shifted in at a row's
// start), step 5 adds lane 15 of rows 0 and 2 to rows 1 and 3, step 6 lane 31 to rows 2 and 3.
__device__ __forceinline__ int wave_inclusive_scan(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);  // row_bcast:15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);  // row_bcast:31 into rows 2 and 3
    return v;
}

// Value of `v` in lane `src`, where src is the same in every lane (read on the scalar path).
__device__ __forceinline__ int wave_read_lane(int v, int src)
{
    return __builtin_amdgcn_readlane(v, __builtin_amdgcn_readfirstlane(src));
}

// Which expert owns row-tile `tile` when every expert's rows [off[e], off[e+1]) are cut into
// tiles of `mt` rows (tiles never straddle experts)?  Every lane of the calling wavefront
// returns the same answer.  e = -1 if `tile` is beyond the last tile.  E_local <= 64;
// max_rows is the row capacity of the activation buffers.
struct TileRef {
    int expert;     // local expert id or -1
    int row_begin;  // first sorted row of the tile
    int row_end;    // one past the last valid sorted row of the tile
    int total;      // total number of row tiles over all experts
};

__device__ __forceinline__ TileRef locate_row_tile(const int32_t* __restrict__ offsets, int E_local, int mt, int tile,
                                                   int max_rows)
{
    const int lane = lane_id();
    int lo = 0, hi = 0;
    if (lane < E_local) {  // clamped so that a corrupt offsets array can never index past the buffers
        lo = min(max(offsets[lane], 0), max_rows);
        hi = min(max(offsets[lane + 1], lo), max_rows);
    }
    const int cnt = hi - lo;
    const int tiles = cnt > 0 ? (cnt + mt - 1) / mt : 0;
    const int incl = wave_inclusive_scan(tiles);
    const int excl = incl - tiles;
    const bool mine = (lane < E_local) && (tile >= excl) && (tile < incl);
    const unsigned long long m = __ballot(mine);
    TileRef r;
    r.total = wave_read_lane(incl, kWave - 1);
    if (m == 0ull) {
        r.expert = -1;
        r.row_begin = 0;
        r.row_end = 0;
        return r;
    }
    const int src = __ffsll(static_cast<long long>(m)) - 1;
    const int e_lo = wave_read_lane(lo, src);
    const int e_hi = wave_read_lane(hi, src);
    const int e_excl = wave_read_lane(excl, src);
    r.expert = src;
    r.row_begin = e_lo + (tile - e_excl) * mt;
    r.row_end = min(r.row_begin + mt, e_hi);
    return r;
}

}  // namespace exf
