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

// Stage 2 by ranking, spread over several workgroups per row (few rows: the streaming launch
// left the survivors of every row as sorted runs of equal length).  Keys are distinct, so the
// place of a key in the result is the number of keys above it: its place in its own run plus,
// per other run, the count of greater keys there (a binary search).  Every workgroup ranks the
// keys of its own runs and writes those whose rank is below K to that place of the output;
// nothing is sorted or selected.
// Only the head of every run (its first H keys) is copied to LDS.  With q = ceil(K / runs), the
// least of the runs' q-th keys has at least K keys at or above it, so it bounds the K-th key
// from below; keys under the bound are left out, and when every run's H-th key is under it
// (H is chosen for that: the runs are near-random samples of the survivors) the heads hold all
// that matters.  Otherwise -- the bound is loose because the greatest keys sit in few runs --
// the same searches run on the whole runs in memory: slow, correct, rare.
constexpr int kRankThreads = 256;

template <typename Ptr>
__device__ __forceinline__ int count_greater(Ptr run, int log_len, uint64_t x) {
    int pos = 0;
    for (int s = 1 << (log_len - 1); s >= 1; s >>= 1) pos += run[pos + s - 1] > x ? s : 0;
    return pos + (run[pos] > x ? 1 : 0);
}

template <typename DT>
__global__ void __launch_bounds__(kRankThreads) rank_finish_kernel(RankFinishParams p) {
    extern __shared__ uint64_t rk_lds[];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
    const int row = blockIdx.y;
    const int L = 1 << p.log_run, H = 1 << p.log_head;
    const uint64_t* runs = p.runs + ((size_t)row * p.nruns << p.log_run);
    lds_ptr<uint64_t> heads = (lds_ptr<uint64_t>)rk_lds;                 // [nruns][H]
    lds_ptr<uint32_t> rank = (lds_ptr<uint32_t>)(rk_lds + ((size_t)p.nruns << p.log_head));   // [my runs][L]
    lds_ptr<uint64_t> red = (lds_ptr<uint64_t>)(rk_lds + ((size_t)p.nruns << p.log_head)) +
                            ((p.runs_per_wg << p.log_run) + 1) / 2;
    lds_ptr<uint32_t> open_word = (lds_ptr<uint32_t>)(red + 4);
    {
        // eight 16-byte loads per thread are asked for before the first is stored (positions
        // clamped instead of tested: a load under a test ends in a wait of its own)
        typedef uint64_t u64x2 __attribute__((ext_vector_type(2)));
        const u64x2* src = (const u64x2*)runs;
        lds_ptr<u64x2> dst = (lds_ptr<u64x2>)rk_lds;
        const int nvec = p.nruns << (p.log_head - 1);
        for (int base = tid; base < nvec; base += 8 * kRankThreads) {
            u64x2 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = min(base + u * kRankThreads, nvec - 1);
                v[u] = src[((i >> (p.log_head - 1)) << (p.log_run - 1)) + (i & ((H >> 1) - 1))];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (base + u * kRankThreads < nvec) dst[base + u * kRankThreads] = v[u];
        }
    }
    const int first = (int)blockIdx.x * p.runs_per_wg;
    const int myruns = min(p.runs_per_wg, p.nruns - first);
    for (int i = tid; i < (myruns << p.log_run); i += kRankThreads) rank[i] = 0;
    if (tid == 0) *open_word = 0;
    __syncthreads();
    // lower bound of the K-th key (q <= H by the host's choice of H, or q > L = H)
    uint64_t bound = 0;
    const int q = (p.K + p.nruns - 1) / p.nruns;
    if (q <= H) {
        uint64_t least = ~0ull;
        for (int r = tid; r < p.nruns; r += kRankThreads) least = min(least, heads[(r << p.log_head) + q - 1]);
        for (int o = 32; o >= 1; o >>= 1) {
            const uint64_t other = ((uint64_t)__shfl_xor((unsigned)(least >> 32), o, kWave) << 32) |
                                   __shfl_xor((unsigned)least, o, kWave);
            least = min(least, other);
        }
        if (lane == 0) red[wave] = least;
        __syncthreads();
        bound = min(min(red[0], red[1]), min(red[2], red[3]));
    }
    bool whole_runs = false;               // some run has keys at or above the bound beyond its head
    if (H < L) {
        bool open = false;
        for (int r = tid; r < p.nruns; r += kRankThreads)
            open |= bound == 0 || heads[(r << p.log_head) + H - 1] >= bound;
        if (open) *open_word = 1;
        __syncthreads();
        whole_runs = *open_word != 0;
    }
    const char* rowp = (const char*)p.values + (size_t)row * p.row_stride * elem<DT>::size;

    // Work items: the keys of my runs at or above the bound, cnt[r] at the head of run r (a binary
    // search per run), numbered run after run.  Consecutive threads take consecutive keys of a
    // run: their searches in another run visit mostly the same or neighbouring words.  Few
    // items: several threads share a key, each taking every parts-th run, and add their counts
    // up in LDS.  run_at(r): the keys of run r that are searched, 1 << log_len of them.
    lds_ptr<uint32_t> cnt = open_word + 1;                  // [my runs]
    // len_tag: the logarithm of the searched length as a compile-time constant (the search loops are
    // then unrolled and their offsets are immediates), or 0 for the run-time value log_any.
    auto place_keys = [&](auto run_at, auto len_tag, int log_any) {
        constexpr int CL = decltype(len_tag)::value;
        const int log_len = CL > 0 ? CL : log_any;
        const int Ls = 1 << log_len;
        if (tid < myruns)
            cnt[tid] = bound == 0 ? (uint32_t)Ls : (uint32_t)count_greater(run_at(first + tid), log_len, bound - 1);
        __syncthreads();
        int items = 0;
        for (int r = 0; r < myruns; ++r) items += (int)cnt[r];
        const int parts = items >= kRankThreads ? 1 : kRankThreads / max(items, 1);
        const int part = items >= kRankThreads ? 0 : tid / max(items, 1);
        auto locate = [&](int it, int& r, int& pos) {       // item -> (run of mine, position)
            r = 0; pos = it;
            while (pos >= (int)cnt[r]) { pos -= (int)cnt[r]; ++r; }
        };
        for (int it = tid - part * items; it < items && part < parts; it += kRankThreads) {
            int r, pos;
            locate(it, r, pos);
            const uint64_t x = run_at(first + r)[pos];
            if (x == 0) continue;
            int above = 0;
            int o = part;
            for (; o + 3 * parts < p.nruns; o += 4 * parts) {
                // four searches side by side: their loads overlap
                int p0 = 0, p1 = 0, p2 = 0, p3 = 0;
                const auto r0 = run_at(o), r1 = run_at(o + parts), r2 = run_at(o + 2 * parts), r3 = run_at(o + 3 * parts);
                auto probe = [&](int s) {
                    const uint64_t a0 = r0[p0 + s - 1], a1 = r1[p1 + s - 1], a2 = r2[p2 + s - 1], a3 = r3[p3 + s - 1];
                    p0 += a0 > x ? s : 0; p1 += a1 > x ? s : 0; p2 += a2 > x ? s : 0; p3 += a3 > x ? s : 0;
                };
                if constexpr (CL > 0) {
#pragma unroll
                    for (int s = 1 << (CL - 1); s >= 1; s >>= 1) probe(s);
                } else {
                    for (int s = Ls >> 1; s >= 1; s >>= 1) probe(s);
                }
                const uint64_t a0 = r0[p0], a1 = r1[p1], a2 = r2[p2], a3 = r3[p3];
                above += p0 + p1 + p2 + p3 + (a0 > x ? 1 : 0) + (a1 > x ? 1 : 0) + (a2 > x ? 1 : 0) + (a3 > x ? 1 : 0);
            }
            for (; o < p.nruns; o += parts) above += count_greater(run_at(o), log_len, x);
            if (parts == 1) rank[(r << p.log_run) + pos] = (uint32_t)above;
            else atomicAdd((uint32_t*)&rank[(r << p.log_run) + pos], (uint32_t)above);
        }
        __syncthreads();
        for (int it = tid; it < items; it += kRankThreads) {
            int r, pos;
            locate(it, r, pos);
            const uint64_t key = run_at(first + r)[pos];
            const uint32_t place = rank[(r << p.log_run) + pos];
            if (key != 0 && place < (uint32_t)p.K) {
                const uint32_t n = key_index(key);
                const int64_t o = (int64_t)row * p.K + place;
                elem<DT>::store_bits(p.out_vals, o, key_stored_bits<DT>(key, rowp, n, p.flip));
                p.out_idx[o] = (int32_t)n;
            }
        }
    };
    if (whole_runs) {
        place_keys([&](int r) { return runs + ((size_t)r << p.log_run); }, std::integral_constant<int, 0>{}, p.log_run);
        return;
    }
    auto head_at = [&](int r) { return (lds_ptr<const uint64_t>)(heads + (r << p.log_head)); };
    switch (p.log_head) {
        case 5: place_keys(head_at, std::integral_constant<int, 5>{}, 5); break;
        case 6: place_keys(head_at, std::integral_constant<int, 6>{}, 6); break;
        case 7: place_keys(head_at, std::integral_constant<int, 7>{}, 7); break;
        case 8: place_keys(head_at, std::integral_constant<int, 8>{}, 8); break;
        default: place_keys(head_at, std::integral_constant<int, 0>{}, p.log_head); break;
    }
}

template <typename DT>
hipError_t launch_rank_for(const RankFinishParams& p, hipStream_t stream) {
    const size_t heads = (size_t)p.nruns << p.log_head, mine = (size_t)p.runs_per_wg << p.log_run;
    const size_t lds = heads * 8 + ((mine + 1) / 2) * 8 + 64 + ((size_t)p.runs_per_wg * 4 + 7) / 8 * 8;
    const dim3 grid((p.nruns + p.runs_per_wg - 1) / p.runs_per_wg, p.rows), block(kRankThreads);
    allow_large_lds((const void*)rank_finish_kernel<DT>, lds);
    hipLaunchKernelGGL((rank_finish_kernel<DT>), grid, block, lds, stream, p);
    return hipGetLastError();
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

hipError_t launch_rank_finish(const RankFinishParams& p, int dtype, hipStream_t stream) {
    switch (dtype) {
        case 0: return launch_rank_for<float>(p, stream);
        case 1: return launch_rank_for<bf16_t>(p, stream);
        case 3: return launch_rank_for<i32_t>(p, stream);
        case 4: return launch_rank_for<u32_t>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace atk
