// Host-only part of the C ABI: error text, version, placement constraint check, communication volume model.
#include <cstdarg>
#include <cstdio>
#include <vector>

#include "common.hpp"

namespace exf {

static thread_local char g_error[512] = "";

int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
    return code;
}

int check_launch(const char* what)
{
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return fail(EXF_ERR_HIP, "%s: %s", what, hipGetErrorString(err));
    return EXF_OK;
}

}  // namespace exf

extern "C" int exf_version(void) { return 100; }

extern "C" const char* exf_last_error(void) { return exf::g_error; }

extern "C" int exf_check_placement(const int32_t* placement_host, int L, int E, int G)
{
    EXF_REQUIRE_PTR(placement_host);
    if (L < 1 || E < 1 || G < 1 || E % G != 0)
        return exf::fail(EXF_ERR_BAD_SHAPE, "exf_check_placement: need L,E,G >= 1 and G | E (L=%d E=%d G=%d)", L, E, G);
    std::vector<int> held(static_cast<size_t>(G));
    for (int l = 0; l < L; ++l) {
        for (int p = 0; p < G; ++p) held[p] = 0;
        for (int e = 0; e < E; ++e) {
            const int32_t p = placement_host[static_cast<size_t>(l) * E + e];
            if (p < 0 || p >= G)
                return exf::fail(EXF_ERR_BAD_SHAPE, "exf_check_placement: layer %d expert %d on device %d outside [0,%d)", l, e, p, G);
            held[p] += 1;
        }
        for (int p = 0; p < G; ++p)
            if (held[p] != E / G)
                return exf::fail(EXF_ERR_BAD_SHAPE, "exf_check_placement: layer %d device %d holds %d experts, expected %d", l, p,
                                 held[p], E / G);
    }
    return EXF_OK;
}

// Table "Comparison with state-of-the-art GPT MoE optimization methods": forward communication in tokens.
extern "C" int exf_comm_volume(int G, int64_t N, int L, double p, double p_star, double* volumes_host)
{
    EXF_REQUIRE_PTR(volumes_host);
    if (G < 1 || N < 0 || L < 1) return exf::fail(EXF_ERR_BAD_SHAPE, "exf_comm_volume: need G >= 1, N >= 0, L >= 1 (G=%d N=%lld L=%d)", G, static_cast<long long>(N), L);
    if (!(p >= 0.0 && p <= 1.0) || !(p_star >= 0.0 && p_star <= 1.0))
        return exf::fail(EXF_ERR_BAD_SHAPE, "exf_comm_volume: ratios must lie in [0,1] (p=%g p_star=%g)", p, p_star);
    const double resident = static_cast<double>(G) * static_cast<double>(N);  // tokens of the whole group
    const double hops = resident * L;                                        // (token, layer) visits
    const double gather = resident * G;                                      // every context copied to every GPU
    volumes_host[0] = 2.0 * hops * p;
    volumes_host[1] = 4.0 * hops * p;
    volumes_host[2] = hops * p_star + gather;
    volumes_host[3] = 2.0 * hops * p_star + gather;
    return EXF_OK;
}

extern "C" int exf_transfer_ratios(const int64_t* away_per_layer_host, const int64_t* local_per_pair_host, int L, int64_t tokens,
                                   double* p_host, double* p_star_host)
{
    EXF_REQUIRE_PTR(away_per_layer_host);
    EXF_REQUIRE_PTR(p_host);
    EXF_REQUIRE_PTR(p_star_host);
    if (L < 1 || tokens < 1) return exf::fail(EXF_ERR_BAD_SHAPE, "exf_transfer_ratios: need L >= 1 and tokens >= 1 (L=%d tokens=%lld)", L, static_cast<long long>(tokens));
    if (L > 1) EXF_REQUIRE_PTR(local_per_pair_host);
    int64_t away = 0, moved = 0;
    for (int l = 0; l < L; ++l) {
        const int64_t a = away_per_layer_host[l];
        if (a < 0 || a > tokens) return exf::fail(EXF_ERR_BAD_SHAPE, "exf_transfer_ratios: away_per_layer[%d] = %lld outside [0,tokens]", l, static_cast<long long>(a));
        away += a;
    }
    moved = away_per_layer_host[0];
    for (int l = 0; l + 1 < L; ++l) {
        const int64_t loc = local_per_pair_host[l];
        if (loc < 0 || loc > tokens) return exf::fail(EXF_ERR_BAD_SHAPE, "exf_transfer_ratios: local_per_pair[%d] = %lld outside [0,tokens]", l, static_cast<long long>(loc));
        moved += tokens - loc;
    }
    const double visits = static_cast<double>(tokens) * L;
    *p_host = static_cast<double>(away) / visits;
    *p_star_host = static_cast<double>(moved) / visits;
    return EXF_OK;
}
