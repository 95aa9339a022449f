// Finish of the split path.  When a batch has too few rows to fill the chip, every row is cut
// into segments that separate workgroups stream (Section 6.1 Steps 1-2 on a part of each
// bucket); what is left to do per row is
//   * Step 2 proper: per bucket, the K' greatest of the union of its per-segment lists.  One
//     thread owns a bucket, reads the nseg*K' keys (coalesced across buckets) and keeps the
//     K' greatest in registers.  Keys carry the index, so ties need no special care;
//   * Steps 3-4: the B*K' merged keys go to LDS; radix selection thins them out, one wavefront
//     sorts what is left in registers and writes the first K.
#include "approx_finish.h"
#include <type_traits>
#include "atk_device.h"
#include "select_sort.h"

namespace atk {
namespace {

template <typename DT, int KP>
__global__ void __launch_bounds__(1024) approx_finish_kernel(FinishParams p) {
    extern __shared__ uint64_t cand[];
    const int tid = threadIdx.x, T = blockDim.x;
    const int row = blockIdx.x;
    const int C = p.B * p.Kprime;
    for (int i = C + tid; i < p.Cpad; i += T) cand[i] = 0;
    const uint64_t* part = p.part_keys + (size_t)row * p.nseg * p.Kprime * p.B;
    // The nseg*K' keys of a bucket lie B apart: key j of bucket b is part[j*B + b].  Sixteen
    // loads are issued before any key is used, so that their latencies overlap (one row can be
    // all the work there is): sixteen keys of one bucket, or four keys of four buckets when a
    // bucket has few.
    const int per_bucket = p.nseg * p.Kprime;
    auto merge_tile = [&](auto nb_tag) {
        constexpr int NB = decltype(nb_tag)::value, NK = 16 / NB;
        for (int b0 = tid; b0 < p.B; b0 += T * NB) {
            uint64_t top[NB][KP];
#pragma unroll
            for (int v = 0; v < NB; ++v)
#pragma unroll
                for (int j = 0; j < KP; ++j) top[v][j] = 0;
            for (int j0 = 0; j0 < per_bucket; j0 += NK) {
                uint64_t in[NB][NK];
#pragma unroll
                for (int v = 0; v < NB; ++v)
#pragma unroll
                    for (int u = 0; u < NK; ++u) {
                        const int b = b0 + v * T;
                        in[v][u] = (b < p.B && j0 + u < per_bucket) ? part[(size_t)(j0 + u) * p.B + b] : 0;
                    }
#pragma unroll
                for (int v = 0; v < NB; ++v)
#pragma unroll
                    for (int u = 0; u < NK; ++u) {
                        const uint64_t key = in[v][u];
                        bool c[KP];
#pragma unroll
                        for (int j = 0; j < KP; ++j) c[j] = key > top[v][j];
#pragma unroll
                        for (int j = KP - 1; j >= 1; --j)
                            top[v][j] = c[j - 1] ? top[v][j - 1] : (c[j] ? key : top[v][j]);
                        top[v][0] = c[0] ? key : top[v][0];
                    }
            }
#pragma unroll
            for (int v = 0; v < NB; ++v) {
                const int b = b0 + v * T;
#pragma unroll
                for (int j = 0; j < KP; ++j)
                    if (b < p.B && j < p.Kprime) cand[b * p.Kprime + j] = top[v][j];
            }
        }
    };
    if constexpr (KP <= 4) {
        if (per_bucket <= 4) merge_tile(std::integral_constant<int, 4>{});
        else merge_tile(std::integral_constant<int, 1>{});
    } else {
        merge_tile(std::integral_constant<int, 1>{});
    }
    __syncthreads();
    const char* rowp = (const char*)p.values + (size_t)row * p.row_stride * elem<DT>::size;
    wg_topk_from_lds<DT>(cand, p.Cpad, p.K, cand + p.Cpad, rowp, p.out_vals, p.out_idx,
                         (int64_t)row * p.K, p.flip);
}

template <typename DT>
hipError_t launch_for(const FinishParams& p, int KP, int threads, hipStream_t stream) {
    const size_t lds = (size_t)p.Cpad * 8 + (p.Cpad > 256 ? kSelectScratchBytes : 0);
    const dim3 grid(p.rows), block(threads);
    switch (KP) {
#define ATK_CASE(N) case N:                                                                       \
        allow_large_lds((const void*)approx_finish_kernel<DT, N>, lds);                           \
        hipLaunchKernelGGL((approx_finish_kernel<DT, N>), grid, block, lds, stream, p); break;
        ATK_CASE(1) ATK_CASE(2) ATK_CASE(3) ATK_CASE(4) ATK_CASE(6) ATK_CASE(8) ATK_CASE(16) ATK_CASE(32)
#undef ATK_CASE
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_finish(const FinishParams& p, int dtype, int KP, hipStream_t stream) {
    // up to 512 threads: beyond that the 16-wavefront barriers cost more than they buy, unless
    // the rows are so few that most of the chip idles and a row's latency is all that counts
    const int max_threads = p.rows <= 64 ? 1024 : 512;
    int threads = 64;
    while (threads < p.B && threads < max_threads) threads <<= 1;
    if (threads < 256 && p.Cpad >= 1024) threads = 256;     // the sort wants more lanes than buckets
    if (dtype == kFinishScores) return launch_for<score_t>(p, KP, threads, stream);
    switch (dtype) {
        case 0: return launch_for<float>(p, KP, threads, stream);
        case 1: return launch_for<bf16_t>(p, KP, threads, stream);
        case 3: return launch_for<i32_t>(p, KP, threads, stream);
        case 4: return launch_for<u32_t>(p, KP, threads, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace atk
