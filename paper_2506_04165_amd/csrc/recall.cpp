// Host-side closed form of the expected recall (Theorem 1), in double precision.
//
//   E[recall] = 1 - (B/K) * sum_{r=K'+1}^{min(K, N/B)} (r-K') C(K,r) C(N-K, N/B-r) / C(N, N/B)
//
// Each term is a hypergeometric probability; it is evaluated as exp of a sum of log-gamma
// values so that N up to 2^31 poses no overflow problem.
#include <cmath>
#include <cstdint>

#include "../../include/atk.h"

namespace {
double log_choose(double n, double k) {
    return std::lgamma(n + 1.0) - std::lgamma(k + 1.0) - std::lgamma(n - k + 1.0);
}
}  // namespace

extern "C" double atk_expected_recall(int64_t N, int64_t B, int64_t K, int64_t Kprime) {
    if (N <= 0 || B < 1 || N % B != 0 || K < 1 || K > N || Kprime < 1) return -1.0;
    const int64_t n = N / B;   // bucket size
    const int64_t rmax = K < n ? K : n;
    const double log_den = log_choose((double)N, (double)n);
    double excess = 0.0;       // E[max(0, X - K')], X = top-K elements landing in one bucket
    for (int64_t r = Kprime + 1; r <= rmax; ++r) {
        if (n - r > N - K) continue;   // C(N-K, n-r) = 0
        const double logp = log_choose((double)K, (double)r) +
                            log_choose((double)(N - K), (double)(n - r)) - log_den;
        excess += (double)(r - Kprime) * std::exp(logp);
    }
    double recall = 1.0 - (double)B / (double)K * excess;
    if (recall < 0.0) recall = 0.0;
    if (recall > 1.0) recall = 1.0;
    return recall;
}
