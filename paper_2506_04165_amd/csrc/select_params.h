// Host-only parameter sweep shared by the public selection entry points; see select_params.cpp.
#pragma once
#include <stdint.h>

namespace atk {

// `runs(ctx, K', B)`: whether the caller can run this configuration (NULL: every legal one).
using RunsFn = bool (*)(void* ctx, int Kprime, int64_t B);

// The sweep behind atk_select_params, restricted to configurations that `runs` accepts.
int select_params_impl(int64_t N, int K, double recall_target, int max_kprime, int bucket_multiple,
                       RunsFn runs, void* ctx, int* Kprime_out, int* B_out, double* expected_recall_out);

}  // namespace atk
