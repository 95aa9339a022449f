// Choice of (K', B) for a recall target (Section 6.3 last paragraph, appendix on parameter
// selection): among the legal configurations whose expected recall (Theorem 1) reaches the
// target, take the one with the fewest stage-1 survivors B*K'; on equal B*K' the smaller K'.
//
// Differences from the paper's sweep, all deliberate:
//   * the expectation is evaluated in closed form (atk_expected_recall) instead of by Monte
//     Carlo, so the answer is deterministic;
//   * "legal" means what these kernels run well: B divides N, B is a multiple of
//     `bucket_multiple` (64 = one wavefront by default; the paper's 128 is a TPU lane
//     constraint), K' <= N/B, K <= B*K', and K' <= max_kprime (the ceiling below which
//     stage 1 stays memory-bound on this chip: 4 for fp32, 8 for bf16);
//   * for fixed K' the recall grows with B, so the smallest sufficient B is found by
//     walking the divisors in ascending order and stopping at the first that qualifies.
#include <algorithm>
#include <cstdint>
#include <vector>

#include "../../include/atk.h"
#include "select_params.h"

extern "C" int atk_select_params(int64_t N, int K, double recall_target, int max_kprime,
                                 int bucket_multiple, int* Kprime_out, int* B_out,
                                 double* expected_recall_out) {
    return atk::select_params_impl(N, K, recall_target, max_kprime, bucket_multiple, nullptr, nullptr,
                                   Kprime_out, B_out, expected_recall_out);
}

int atk::select_params_impl(int64_t N, int K, double recall_target, int max_kprime, int bucket_multiple,
                            RunsFn runs, void* ctx, int* Kprime_out, int* B_out,
                            double* expected_recall_out) {
    if (N <= 0 || N > 0x7fffffffLL - 0xffff || K < 1 || K > N || !Kprime_out || !B_out) return ATK_INVALID_ARG;
    if (!(recall_target > 0.0) || recall_target > 1.0 || max_kprime < 1 || bucket_multiple < 1)
        return ATK_INVALID_ARG;

    // divisors of N that are multiples of bucket_multiple, ascending
    std::vector<int64_t> buckets;
    for (int64_t d = 1; d * d <= N; ++d) {
        if (N % d) continue;
        if (d % bucket_multiple == 0) buckets.push_back(d);
        const int64_t e = N / d;
        if (e != d && e % bucket_multiple == 0) buckets.push_back(e);
    }
    std::sort(buckets.begin(), buckets.end());

    int64_t best_elems = -1;
    int best_kp = 0;
    int64_t best_b = 0;
    double best_recall = 0.0;
    for (int kp = 1; kp <= max_kprime && kp <= K; ++kp) {
        for (int64_t B : buckets) {
            if (B * kp < K) continue;                 // stage 2 needs at least K survivors
            if (kp > N / B) break;                    // buckets only get shorter from here on
            if (best_elems >= 0 && B * kp >= best_elems) break;   // cannot improve any more
            if (runs && !runs(ctx, kp, B)) continue;
            const double r = atk_expected_recall(N, B, K, kp);
            if (r >= recall_target) {
                best_elems = B * kp; best_kp = kp; best_b = B; best_recall = r;
                break;
            }
        }
    }
    if (best_elems < 0) {
        // no approximate configuration reaches the target: K' = K with a single bucket is the
        // exact Top-K (recall 1)
        *Kprime_out = K; *B_out = 1;
        if (expected_recall_out) *expected_recall_out = 1.0;
        return ATK_OK;
    }
    *Kprime_out = best_kp;
    *B_out = (int)best_b;
    if (expected_recall_out) *expected_recall_out = best_recall;
    return ATK_OK;
}

// Fusion-aware choice for atk_mips_approx_topk (the paper's conclusion leaves "fusion-aware
// parameter selection" open).  In the fused kernel the list update is what costs: every score
// pays about 5K'-2 vector operations whatever B is, and the survivors are small next to the
// matrix product.  So the rule is the reverse of the unfused one: the smallest K' for which some
// legal B reaches the target, and for that K' the smallest such B.  Legal here: B divides N, B a
// multiple of 32 (a slab of the kernel), K' <= min(4, N/B), K <= B*K' <= 16384.
// Returns ATK_UNSUPPORTED when no legal configuration reaches the target.
extern "C" int atk_mips_select_params(int64_t N, int K, double recall_target, int* Kprime_out,
                                      int* B_out, double* expected_recall_out) {
    if (N <= 0 || N > 0x7fffffffLL - 0xffff || K < 1 || K > N || !Kprime_out || !B_out) return ATK_INVALID_ARG;
    if (!(recall_target > 0.0) || recall_target > 1.0) return ATK_INVALID_ARG;
    std::vector<int64_t> buckets;
    for (int64_t d = 1; d * d <= N; ++d) {
        if (N % d) continue;
        if (d % 32 == 0) buckets.push_back(d);
        const int64_t e = N / d;
        if (e != d && e % 32 == 0) buckets.push_back(e);
    }
    std::sort(buckets.begin(), buckets.end());
    for (int kp = 1; kp <= 4 && kp <= K; ++kp) {
        for (int64_t B : buckets) {
            if (B * kp > 16384) break;
            if (B * kp < K) continue;
            if (kp > N / B) break;
            const double r = atk_expected_recall(N, B, K, kp);
            if (r >= recall_target) {
                *Kprime_out = kp; *B_out = (int)B;
                if (expected_recall_out) *expected_recall_out = r;
                return ATK_OK;
            }
        }
    }
    return ATK_UNSUPPORTED;
}
