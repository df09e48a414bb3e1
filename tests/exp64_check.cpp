// Host build of the device's fp64 exponential, compared with libm over the
// range the verification kernels use (non-positive arguments).
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <random>

#include "exp64.h"

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
    const bool specials = lantern::exp_nonpos(0.0) == 1.0 && lantern::exp_nonpos(-INFINITY) == 0.0 &&
                          lantern::exp_nonpos(-800.0) == 0.0 && lantern::exp_nonpos(-1e300) == 0.0 &&
                          lantern::exp_nonpos(-745.1) == std::exp(-745.1);
    std::printf("%lld %ld %ld %d\n", (long long)worst, n_diff, n, specials ? 1 : 0);
    return 0;
}
