// Read-only streaming probe: the measured bandwidth ceiling that the streaming kernels are held
// against (the beta of Section 2.3's runtime model, as this chip delivers it to a kernel that
// does nothing but read).  It reads a buffer once with the same instruction the stage-1 kernel
// streams rows with -- non-temporal 16-byte buffer loads, every workgroup walking a contiguous
// piece; one workgroup of 512 threads per CU with four loads in flight per lane measured fastest of
// the shapes tried, 6.5 TB/s on 256 MB and 7.1 TB/s on 1 GiB -- and folds the words of every piece into a checksum word
// of its own (no atomics: nothing but the loads takes time) so that the loads cannot be dropped
// and the result can be checked.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/atk.h"
#include "atk_device.h"

namespace {

constexpr int kThreads = 512;
constexpr int kInFlight = 4;                 // 16-byte loads issued before the first is used

__global__ void __launch_bounds__(kThreads) read_probe_kernel(const char* data, size_t n_vec,
                                                             size_t vec_per_wg, uint32_t* out) {
    const size_t first = (size_t)blockIdx.x * vec_per_wg;
    const size_t count = first < n_vec ? (n_vec - first < vec_per_wg ? n_vec - first : vec_per_wg) : 0;
    const atk::buffer_rsrc rs = atk::make_rsrc(data + first * 16);      // a piece is below 4 GiB
    uint32_t acc = 0;
    size_t i = threadIdx.x;
    for (; i + (size_t)(kInFlight - 1) * kThreads < count; i += (size_t)kInFlight * kThreads) {
        uint4 v[kInFlight];
#pragma unroll
        for (int u = 0; u < kInFlight; ++u)
            v[u] = atk::buffer_load<16>::run(rs, (uint32_t)((i + (size_t)u * kThreads) * 16), 0);
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < count; i += kThreads) {
        const uint4 v = atk::buffer_load<16>::run(rs, (uint32_t)(i * 16), 0);
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    for (int o = atk::kWave / 2; o >= 1; o >>= 1) acc ^= (uint32_t)__shfl_xor((int)acc, o, atk::kWave);
    __shared__ uint32_t wave_acc[kThreads / atk::kWave];
    if ((threadIdx.x & (atk::kWave - 1)) == 0) wave_acc[threadIdx.x / atk::kWave] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t all = 0;
        for (int w = 0; w < kThreads / atk::kWave; ++w) all ^= wave_acc[w];
        out[blockIdx.x] ^= all;          // this workgroup's own word
    }
}

}  // namespace

extern "C" int atk_read_probe(const void* data, size_t bytes, void* checksum, void* stream) {
    if (!checksum || (uintptr_t)checksum % 4) return ATK_INVALID_ARG;
    if (bytes == 0) return ATK_OK;
    if (!data || (uintptr_t)data % 16 || bytes % 16) return ATK_INVALID_ARG;
    const size_t n_vec = bytes / 16;
    // as many pieces as checksum words (one workgroup per CU); a piece stays below what a 32-bit
    // offset reaches
    const size_t grid = ATK_READ_PROBE_WORDS;
    const size_t vec_per_wg = (n_vec + grid - 1) / grid;
    if (vec_per_wg * 16 >= ((size_t)1 << 31)) return ATK_UNSUPPORTED;
    hipLaunchKernelGGL(read_probe_kernel, dim3((unsigned)grid), dim3(kThreads), 0, (hipStream_t)stream,
                       (const char*)data, n_vec, vec_per_wg, (uint32_t*)checksum);
    return hipGetLastError() == hipSuccess ? ATK_OK : ATK_HIP_ERROR;
}
