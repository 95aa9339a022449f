// Exact Top-K launcher (radix selection + LDS sort); see topk_exact.hip.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace atk {

constexpr int kRegRowVectors = 8;     // 16-byte vectors of a short row a thread keeps in registers
constexpr int kRegRowThreads = 256;   // ... in a workgroup of this many threads

struct TopkParams {
    const void* values;       // [rows, row_stride] elements of the given dtype
    const int32_t* payload;   // optional [rows, row_stride] original indices (survivor mode)
    int64_t row_stride;
    const void* orig_values;  // survivor mode: the rows the survivors were taken from ...
    int64_t orig_stride;      // ... and their stride (read only to tell -0.0 from +0.0)
    int rows, N, K;
    uint32_t flip;            // 0: the K greatest; min-K: the order-reversing mask of the element type, xor-ed
                              // onto every loaded pattern and again onto every pattern written out
    int cap;                  // LDS key buffer capacity (power of two, >= 1024, > K)
    int onepass;              // try the single pass with a rising threshold first (needs K <= 1024,
                              // cap >= 1024 + one round of the workgroup, cap <= 16 * threads)
    int reg_row;              // short aligned rows (N <= 256 threads x 8 vectors of 16 bytes, N a multiple of the
                              // vector length, 256 threads, no payload): keep the row in registers
    const int32_t* row_mask;  // optional [rows]: only rows with a non-zero entry are done, the others' outputs stay
    void* out_vals;
    int32_t* out_idx;
};

hipError_t launch_topk_exact(const TopkParams& p, int dtype, int threads, hipStream_t stream);

}  // namespace atk
