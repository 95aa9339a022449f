// Driver for running the library's host-only arithmetic (Theorem 1 in closed form, the parameter
// selections) under AddressSanitizer and UndefinedBehaviorSanitizer.  Built by
// tests/test_sanitizers.py from csrc/recall.cpp and csrc/select_params.cpp, which contain no
// GPU code.  Reads lines "N K target max_kprime bucket_multiple" and prints what the two
// selections and the closed form return, for the test to compare with the ordinary library.
#include <cstdint>
#include <cstdio>

#include "../../include/atk.h"

int main() {
    long long N;
    int K, maxkp, mult;
    double target;
    while (std::scanf("%lld %d %lf %d %d", &N, &K, &target, &maxkp, &mult) == 5) {
        int kp = -1, b = -1, kp2 = -1, b2 = -1;
        double r = -1.0, r2 = -1.0;
        const int s1 = atk_select_params(N, K, target, maxkp, mult, &kp, &b, &r);
        const int s2 = atk_mips_select_params(N, K, target, &kp2, &b2, &r2);
        const double e = (s1 == 0 && b >= 1 && N % b == 0) ? atk_expected_recall(N, b, K, kp) : -1.0;
        std::printf("%d %d %d %.17g %d %d %d %.17g %.17g\n", s1, kp, b, r, s2, kp2, b2, r2, e);
    }
    return 0;
}
