// Host build of the device's fp64 exponential, compared with libm over the
// range the verification kernels use (non-positive arguments).
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <random>

#include "exp64.h"
#include "exp_table.h"

static int64_t ulp_diff(double a, double b) {
    int64_t ia, ib;
    std::memcpy(&ia, &a, 8);
    std::memcpy(&ib, &b, 8);
    return ia > ib ? ia - ib : ib - ia;
}

int main() {
    std::mt19937_64 rng(20241003355ull);
    std::uniform_real_distribution<double> near(-60.0, 0.0), far(-745.0, 0.0);
    int64_t worst = 0;
    long n_diff = 0, n = 0;
    for (int i = 0; i < 2000000; ++i) {
        double d = (i & 1) ? near(rng) : far(rng);
        if (i % 3 == 0) d = (double)(float)d;  // differences of fp32 logits
        const int64_t u = ulp_diff(lantern::exp_nonpos(d), std::exp(d));
        worst = u > worst ? u : worst;
        n_diff += u != 0;
        ++n;
    }
    // the table-driven exponential, also for the positive arguments it accepts
    std::uniform_real_distribution<double> pos(0.0, 50.0);
    int64_t worst_tab = 0;
    long n_diff_tab = 0;
    for (int i = 0; i < 3000000; ++i) {
        double d = (i % 3 == 0) ? near(rng) : (i % 3 == 1) ? far(rng) : pos(rng);
        if (i % 4 == 0) d = (double)(float)d;
        const int64_t u = ulp_diff(lantern::exp_tab(d, lantern::EXP_TABLE_HILO), std::exp(d));
        worst_tab = u > worst_tab ? u : worst_tab;
        n_diff_tab += u != 0;
    }
    // the short form on its range: the same values as exp_tab, bit for bit
    long n_core_diff = 0;
    std::uniform_real_distribution<double> core(-700.0, 60.0);
    for (int i = 0; i < 2000000; ++i) {
        double d = core(rng);
        if (i % 4 == 0) d = (double)(float)d;
        n_core_diff += lantern::exp_tab_core(d, reinterpret_cast<const unsigned char*>(lantern::EXP_TABLE_HILO)) != lantern::exp_tab(d, lantern::EXP_TABLE_HILO);
    }
    n_core_diff += lantern::exp_tab_core(-700.0, reinterpret_cast<const unsigned char*>(lantern::EXP_TABLE_HILO)) != lantern::exp_tab(-700.0, lantern::EXP_TABLE_HILO);
    n_core_diff += lantern::exp_tab_core(0.0, reinterpret_cast<const unsigned char*>(lantern::EXP_TABLE_HILO)) != 1.0;
    const bool specials_tab = n_core_diff == 0 && lantern::exp_tab(0.0, lantern::EXP_TABLE_HILO) == 1.0 &&
                              lantern::exp_tab(-INFINITY, lantern::EXP_TABLE_HILO) == 0.0 &&
                              lantern::exp_tab(-1e300, lantern::EXP_TABLE_HILO) == 0.0 &&
                              lantern::exp_tab(NAN, lantern::EXP_TABLE_HILO) == 0.0 &&
                              lantern::exp_tab(-745.1, lantern::EXP_TABLE_HILO) == std::exp(-745.1);
    const bool specials = lantern::exp_nonpos(0.0) == 1.0 && lantern::exp_nonpos(-INFINITY) == 0.0 &&
                          lantern::exp_nonpos(-800.0) == 0.0 && lantern::exp_nonpos(-1e300) == 0.0 &&
                          lantern::exp_nonpos(-745.1) == std::exp(-745.1);
    std::printf("%lld %ld %ld %d %lld %ld %d\n", (long long)worst, n_diff, n, specials ? 1 : 0, (long long)worst_tab,
                n_diff_tab, specials_tab ? 1 : 0);
    return 0;
}
