// Exact Top-K of every row by most-significant-digit radix selection on 64-bit keys,
// one workgroup per row.  This is the comparison system on the same hardware (the paper
// compares against an exact Top-K in Section 7) and, with an index payload, the second
// launch of the unfused path (Section 6.1 Step 4 on survivors that do not fit in LDS).
//
// Per row:
//   1. histogram one digit of the keys that still match the known prefix (LDS atomics);
//   2. walk the histogram from the top: digits above the one where the running count
//      reaches the number still needed are certain members, that digit extends the prefix;
//   3. stop as soon as (certain members + keys matching the prefix) fit the LDS buffer --
//      for continuous data that is after the first digit -- otherwise take the next digit
//      (value bits first, then index bits, so ties end up resolved toward the lower index);
//   4. one more pass gathers certain members and prefix matches into LDS, where the same
//      selection-then-wave-sort as in the fused kernel's stage 2 picks and orders the K.
#include "atk_device.h"
#include "select_sort.h"
#include "topk_exact.h"

namespace atk {

namespace {

constexpr int kBins = 2048;
constexpr int kNumDigits = 6;
__device__ __constant__ int kDigitShift[kNumDigits] = {53, 42, 32, 21, 10, 0};
__device__ __constant__ int kDigitBits[kNumDigits] = {11, 11, 10, 11, 11, 10};

template <typename DT, bool PAYLOAD>
__device__ __forceinline__ uint64_t key_at(const void* rowp, const int32_t* payload, int n) {
    const uint32_t b = elem<DT>::load_bits(rowp, n);
    const uint32_t idx = PAYLOAD ? (uint32_t)payload[n] : (uint32_t)n;
    return make_key(b, idx);
}

template <typename DT, bool PAYLOAD>
__global__ void __launch_bounds__(1024) topk_exact_kernel(TopkParams p) {
    extern __shared__ uint64_t lds64[];
    // layout: [0, cap) key buffer (the histogram aliases its start), scratch of the final
    // selection, then 32 control words
    uint32_t* hist = (uint32_t*)lds64;
    void* scratch = lds64 + p.cap;
    uint32_t* ctl = (uint32_t*)((char*)scratch + kSelectScratchBytes);   // 0: digit  1: certain  2: count  3: fill  4..: wave sums
    const int tid = threadIdx.x, T = blockDim.x;
    const int row = blockIdx.x;
    const char* rowp = (const char*)p.values + (size_t)row * p.row_stride * elem<DT>::size;
    const int32_t* payload = PAYLOAD ? p.payload + (size_t)row * p.row_stride : nullptr;
    const int N = p.N;

    uint64_t prefix = 0, mask = 0;
    int need = p.K;          // members still to be taken from the keys matching the prefix
    int certain = 0;         // members already known (keys above the prefix)

    for (int d = 0; d < kNumDigits; ++d) {
        const int shift = kDigitShift[d];
        const uint32_t dmask = (1u << kDigitBits[d]) - 1u;
        for (int i = tid; i < kBins; i += T) hist[i] = 0;
        __syncthreads();
        for (int n = tid; n < N; n += T) {
            const uint64_t key = key_at<DT, PAYLOAD>(rowp, payload, n);
            if ((key & mask) == prefix) atomicAdd(&hist[(uint32_t)(key >> shift) & dmask], 1u);
        }
        __syncthreads();
        // suffix sums over bins: thread t owns bins [t*bpt, (t+1)*bpt)
        const int bpt = kBins / T > 0 ? kBins / T : 1;
        uint32_t mine = 0;
        if (tid * bpt < kBins)
            for (int i = 0; i < bpt; ++i) mine += hist[tid * bpt + i];
        // inclusive suffix scan inside the wave (lane l gets the sum over lanes >= l)
        const int lane = tid & (kWave - 1), wave = tid >> 6;
        uint32_t suf = mine;
        for (int o = 1; o < kWave; o <<= 1) {
            const uint32_t other = __shfl_down(suf, o, kWave);
            if (lane + o < kWave) suf += other;
        }
        if (lane == 0) ctl[4 + wave] = suf;
        __syncthreads();
        uint32_t above = 0;                          // sum over waves after mine
        for (int w = wave + 1; w < (T >> 6); ++w) above += ctl[4 + w];
        const uint32_t incl = suf + above, excl = incl - mine;
        if (tid * bpt < kBins && excl < (uint32_t)need && incl >= (uint32_t)need) {
            uint32_t run = excl;
            for (int i = bpt - 1; i >= 0; --i) {
                const uint32_t c = hist[tid * bpt + i];
                if (run + c >= (uint32_t)need) {
                    ctl[0] = (uint32_t)(tid * bpt + i);
                    ctl[1] = run;                   // keys in higher digits: certain members
                    ctl[2] = c;
                    break;
                }
                run += c;
            }
        }
        __syncthreads();
        const uint32_t digit = ctl[0], more = ctl[1], count = ctl[2];
        __syncthreads();
        certain += (int)more;
        need -= (int)more;
        prefix |= (uint64_t)digit << shift;
        mask |= (uint64_t)dmask << shift;
        if (certain + (int)count <= p.cap) break;
    }

    // gather certain members and prefix matches
    if (tid == 0) ctl[3] = 0;
    __syncthreads();
    for (int n = tid; n < N; n += T) {
        const uint64_t key = key_at<DT, PAYLOAD>(rowp, payload, n);
        if ((key & mask) >= prefix) {
            const uint32_t slot = atomicAdd(&ctl[3], 1u);
            if (slot < (uint32_t)p.cap) lds64[slot] = key;   // always true; keeps a logic slip memory safe
        }
    }
    __syncthreads();
    const int total = min((int)ctl[3], p.cap);
    const int n2 = next_pow2(total);
    for (int i = total + tid; i < n2; i += T) lds64[i] = 0;
    __syncthreads();
    if (!PAYLOAD) {
        wg_topk_from_lds<DT>(lds64, n2, p.K, scratch, rowp, p.out_vals, p.out_idx, (int64_t)row * p.K);
        return;
    }
    // survivor mode: the key's index is the original position, the value sits at the survivor's slot
    lds_bitonic_sort_desc(lds64, n2, n2);
    for (int i = tid; i < p.K; i += T) {
        const uint64_t key = lds64[i];
        const uint32_t idx = key_index(key);
        uint32_t b = key_value_bits(key);
        if (b == 0) {
            // rare: look the survivor up by its index to tell -0.0 from +0.0
            for (int n = 0; n < N; ++n)
                if ((uint32_t)payload[n] == idx) { b = elem<DT>::load_bits(rowp, n); break; }
        }
        elem<DT>::store_bits(p.out_vals, (int64_t)row * p.K + i, b);
        p.out_idx[(int64_t)row * p.K + i] = (int32_t)idx;
    }
}

}  // namespace

hipError_t launch_topk_exact(const TopkParams& p, int dtype, int threads, hipStream_t stream) {
    const size_t lds = (size_t)p.cap * 8 + kSelectScratchBytes + 32 * 4;
    const dim3 grid(p.rows), block(threads);
    const bool payload = p.payload != nullptr;
    if (dtype == 0) {
        if (payload) hipLaunchKernelGGL((topk_exact_kernel<float, true>), grid, block, lds, stream, p);
        else         hipLaunchKernelGGL((topk_exact_kernel<float, false>), grid, block, lds, stream, p);
    } else {
        if (payload) hipLaunchKernelGGL((topk_exact_kernel<bf16_t, true>), grid, block, lds, stream, p);
        else         hipLaunchKernelGGL((topk_exact_kernel<bf16_t, false>), grid, block, lds, stream, p);
    }
    return hipGetLastError();
}

}  // namespace atk
