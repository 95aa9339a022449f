// Vector-ALU throughput probe (the paper's appendix "Estimating peak VPU throughput", redone
// for this chip): two streaming kernels with a tunable number of dependent integer operations
// per element.  Timing them over a large array shows a flat memory-bound region followed by a
// linear compute-bound one; the slope of the latter is the vector throughput (gamma of
// Section 2.3) and with it the ridge point "vector operations per 4 bytes" that bounds how
// large K' can be before stage 1 stops being memory-bound.
//
//   kind 0 "fibonacci": out[i] = y_n where (x, y) -> (y, x + y) is applied `ops` times,
//                       reading x[i] and y[i] (ops additions per two words read, one written)
//   kind 1 "squaring":  out[i] = x[i] squared `ops` times (ops multiplications per word read)
// int32 arithmetic wraps around.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/atk.h"

namespace {

template <int KIND>
__global__ void __launch_bounds__(256) valu_probe_kernel(const uint32_t* __restrict__ x,
                                                         const uint32_t* __restrict__ y,
                                                         uint32_t* __restrict__ out, size_t n, int ops) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        uint32_t a = x[i];
        if (KIND == 0) {
            uint32_t b = y[i];
            int k = 0;
            for (; k + 4 <= ops; k += 4) {      // four steps: (a,b) -> (b,a+b) -> ...
                a += b; b += a; a += b; b += a;
            }
            // after an even number of steps the pair is (a, b); finish the remainder
            for (; k < ops; ++k) { const uint32_t c = a + b; a = b; b = c; }
            out[i] = b;
        } else {
            int k = 0;
            for (; k + 4 <= ops; k += 4) { a *= a; a *= a; a *= a; a *= a; }
            for (; k < ops; ++k) a *= a;
            out[i] = a;
        }
    }
}

}  // namespace

extern "C" int atk_valu_probe(int kind, const void* x, const void* y, void* out, size_t n_words,
                              int ops, void* stream) {
    if ((kind != 0 && kind != 1) || !x || !out || (kind == 0 && !y) || ops < 0) return ATK_INVALID_ARG;
    if (((uintptr_t)x | (uintptr_t)y | (uintptr_t)out) % 4) return ATK_INVALID_ARG;
    if (n_words == 0) return ATK_OK;
    const int block = 256;
    size_t want = (n_words + block - 1) / block;
    const int grid = (int)(want < 256 * 32 ? want : 256 * 32);     // 32 workgroups per CU at most
    if (kind == 0)
        hipLaunchKernelGGL(valu_probe_kernel<0>, dim3(grid), dim3(block), 0, (hipStream_t)stream,
                           (const uint32_t*)x, (const uint32_t*)y, (uint32_t*)out, n_words, ops);
    else
        hipLaunchKernelGGL(valu_probe_kernel<1>, dim3(grid), dim3(block), 0, (hipStream_t)stream,
                           (const uint32_t*)x, (const uint32_t*)y, (uint32_t*)out, n_words, ops);
    return hipGetLastError() == hipSuccess ? ATK_OK : ATK_HIP_ERROR;
}
