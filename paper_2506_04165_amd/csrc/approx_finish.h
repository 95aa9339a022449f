// Second launch of the split path: merges the per-segment partial lists of every bucket and
// runs stage 2.  See approx_finish.hip.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace atk {

struct FinishParams {
    const uint64_t* part_keys;   // [rows, nseg, K', B] keys written by the streaming launch
    const void* values;          // the input, only read to tell -0.0 from +0.0
    int64_t row_stride;
    int rows, K, Kprime, B, nseg;
    uint32_t flip;               // the order-reversing mask the keys were built under (0: Top-K), see ApproxParams
    int Cpad;                    // power of two >= B*K'
    void* out_vals;
    int32_t* out_idx;
};

// dtype: 0 fp32, 1 bf16 (and fp16, same order of bit patterns), 3 int32, 4 uint32, or this
// value for keys whose values are binary32 scores with no stored array behind them
// (`values` is not read; out_vals is float)
constexpr int kFinishScores = 100;

// KP: compiled list length (>= Kprime), one of 1,2,3,4,6,8,16,32
hipError_t launch_finish(const FinishParams& p, int dtype, int KP, hipStream_t stream);

// Stage 2 by ranking (slab route): see rank_finish_kernel.
struct RankFinishParams {
    const uint64_t* runs;        // [rows, nruns, 1 << log_run] keys, every run sorted (greatest first), zeros last
    const void* values;          // the input, only read to tell -0.0 from +0.0
    int64_t row_stride;
    int rows, K, nruns, log_run;
    int log_head;                // the first H = 1 << log_head keys of every run are held in LDS; H <= run length,
                                 // H >= ceil(K / nruns) when that is at most the run length, H >= 2
    int runs_per_wg;             // runs whose keys one workgroup ranks (grid: ceil(nruns / runs_per_wg) x rows)
    uint32_t flip;
    void* out_vals;
    int32_t* out_idx;
};
constexpr int kRankMaxHeadKeys = 12288;  // keys of a row's run heads (nruns << log_head) that the kernel holds in LDS
hipError_t launch_rank_finish(const RankFinishParams& p, int dtype, hipStream_t stream);

}  // namespace atk
