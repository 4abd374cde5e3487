// Host-only part of the C ABI: error text, version, placement constraint check.
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
