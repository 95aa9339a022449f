// Exact Top-K of every row by most-significant-digit radix selection on 64-bit keys,
// one workgroup per row.  This is the comparison system on the same hardware (the paper
// compares against an exact Top-K in Section 7) and, with an index payload, the second
// launch of the unfused path (Section 6.1 Step 4 on survivors that do not fit in LDS).
//
// Per row:
//   1. first pass: histogram of the leading 11 value bits (LDS atomics).  The row is taken in
//      chunks; after the first chunk, and then at doubling distances, the histogram so far gives
//      a lower bound (the digit at which K keys have already been seen): keys below it can no
//      longer matter and skip the atomic, which removes nearly all of them and with them the
//      bank conflicts of a peaked distribution;
//   2. walk the histogram from the top: digits above the one where the running count reaches K
//      are certain members, that digit becomes the prefix;
//   3. while (certain members + keys matching the prefix) exceed the LDS buffer -- only with
//      massive ties -- take the next digit (value bits first, then index bits, so ties resolve
//      toward the lower index);
//   4. a last pass gathers certain members and prefix matches into LDS, where the same
//      selection-then-wave-sort as in the fused kernel's stage 2 picks and orders the K.
// Two passes over the row for ordinary data: at most half of the HBM roofline.
//
// Rows of ordinary data are first tried in ONE pass (`onepass` below): the row is streamed once,
// keys above a rising threshold are collected in LDS, and whenever the buffer is half full a
// selection finds a key with at least K keys at or above it, which becomes the new threshold and
// everything below it is dropped.  For data in random order the keys that pass after the first
// few thousand elements are few (about K ln(N / seen)), so the buffer is compacted a handful of
// times per row.  Data that keeps beating the threshold (ascending order) would overflow the
// buffer between two compactions: the attempt is then abandoned and the row done in two passes
// as above, which does not depend on the order of the data.
#include "atk_device.h"
#include "select_sort.h"
#include "topk_exact.h"

namespace atk {

namespace {

constexpr int kNumDigits = 6;
__device__ __constant__ int kDigitShift[kNumDigits] = {53, 42, 32, 21, 10, 0};
__device__ __constant__ int kDigitBits[kNumDigits] = {11, 11, 10, 11, 11, 10};

// Calls fn(bits, n) for every element n of the row: 16-byte vector loads when the row allows
// (no payload, base and stride 16-byte aligned), element loads otherwise.  All threads take part.
template <typename DT, bool VEC, int UN = 4, typename F>
__device__ __forceinline__ void for_each_element(const char* rowp, int begin, int end, F&& fn) {
    const int tid = threadIdx.x, T = blockDim.x;
    constexpr int VE = 16 / elem<DT>::size;
    if constexpr (VEC) {
        // begin is a multiple of VE
        const int nvec = (end - begin) / VE;
        const uint4* vp = (const uint4*)(rowp + (size_t)begin * elem<DT>::size);
        int i = tid;
        for (; i + (UN - 1) * T < nvec; i += UN * T) {
            uint4 v[UN];
#pragma unroll
            for (int u = 0; u < UN; ++u) v[u] = vp[i + u * T];
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const uint32_t* w = (const uint32_t*)&v[u];
#pragma unroll
                for (int e = 0; e < VE; ++e) {
                    uint32_t b;
                    if constexpr (elem<DT>::size == 4) b = w[e];
                    else b = (e & 1) ? (w[e >> 1] & 0xffff0000u) : (w[e >> 1] << 16);
                    fn(b, begin + (i + u * T) * VE + e);
                }
            }
        }
        for (; i < nvec; i += T) {
            const uint4 v = vp[i];
            const uint32_t* w = (const uint32_t*)&v;
#pragma unroll
            for (int e = 0; e < VE; ++e) {
                uint32_t b;
                if constexpr (elem<DT>::size == 4) b = w[e];
                else b = (e & 1) ? (w[e >> 1] & 0xffff0000u) : (w[e >> 1] << 16);
                fn(b, begin + i * VE + e);
            }
        }
        for (int n = begin + nvec * VE + tid; n < end; n += T) fn(elem<DT>::load_bits(rowp, n), n);
    } else {
        for (int n = begin + tid; n < end; n += T) fn(elem<DT>::load_bits(rowp, n), n);
    }
}

// One pass with a rising threshold.  On success the K greatest keys of the row are among the
// `count` keys at the start of `buf` and true is returned; false (all threads alike) when the
// buffer overflowed, with nothing written anywhere but LDS.
//   buf      p.cap keys;  scratch: kSelectScratchBytes;  ctl: control words (3: fill, 5: overflow)
// Until a threshold exists every element is kept, and the row is taken one round of the whole
// workgroup (a 16-byte vector, or one element, per thread) at a time; after that in stretches
// sized by how many keys are expected to pass.
template <typename DT, bool PAYLOAD, bool VEC, bool MINK>
__device__ __forceinline__ bool onepass(const TopkParams& p, const char* rowp, const int32_t* payload,
                                        uint64_t* buf, void* scratch, uint32_t* ctl, int& count) {
    const int tid = threadIdx.x, T = blockDim.x, lane = tid & (kWave - 1);
    const int N = p.N, cap = p.cap;
    const uint32_t flip = MINK ? p.flip : 0u;
    constexpr int VE = VEC ? 16 / elem<DT>::size : 1;
    constexpr int kMaxRounds = 1024;
    constexpr int kInFlight = 4;            // vector loads a lane issues before it looks at the first (8 and 16: no faster)
    auto index_of = [&](int n) -> uint32_t { return PAYLOAD ? (uint32_t)payload[n] : (uint32_t)n; };
    if (tid == 0) { ctl[3] = 0; ctl[5] = 0; }
    __syncthreads();
    uint64_t thr = 0;                       // keys at or below it cannot be among the K greatest
    const int round = T * VE;               // elements one round of the workgroup covers
    int fill = 0;
    int seen_at_thr = 0;                    // elements seen when the threshold was last raised
    for (int done = 0; done < N;) {
        // How far to go before looking at the fill again.  Without a threshold every element is
        // kept: one round.  With one, an element of data in random order passes with probability
        // about K / seen_at_thr: go as far as is expected to fill half of the room that is left.
        int64_t take = round;
        if (seen_at_thr > 0) {
            take = (int64_t)((cap - fill) / 2) * seen_at_thr / p.K / round * round;
            if (take < round) take = round;
            if (take > (int64_t)kMaxRounds * round) take = (int64_t)kMaxRounds * round;
            if (take > 4 * (int64_t)done) take = 4 * (int64_t)done;   // data in ascending order shows early
        }
        const int end = (int)min((int64_t)N, (int64_t)done + take);
        // cheap reject: one compare of the stored value with the threshold's value; only the few
        // elements at or above it have their key built and compared
        const uint32_t thr_bits = elem<DT>::floor_bits((uint32_t)(thr >> 32));
        for_each_element<DT, VEC, kInFlight>(rowp, done, end, [&](uint32_t b, int n) {
            b ^= flip;
            bool pass = elem<DT>::ge(b, thr_bits);
            if (__ballot(pass) == 0) return;
            uint64_t key = 0;
            if (pass) {
                key = make_key<DT>(b, index_of(n));
                pass = key > thr;
            }
            // one LDS atomic per wavefront: the lanes that keep their key take consecutive slots
            const uint64_t m = __ballot(pass);
            if (m != 0) {
                const int leader = __ffsll((unsigned long long)m) - 1;
                uint32_t base = 0;
                if (lane == leader) base = atomicAdd(&ctl[3], (uint32_t)__popcll(m));
                base = (uint32_t)__shfl((int)base, leader, kWave);
                if (pass) {
                    const uint32_t slot = base + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
                    if (slot < (uint32_t)cap) buf[slot] = key;
                    else ctl[5] = 1;                        // no room: the attempt has failed
                }
            }
        });
        done = end;
        __syncthreads();
        const bool overflow = ctl[5] != 0;
        fill = (int)ctl[3];
        __syncthreads();                    // (ctl[3] is rewritten below)
        if (overflow) return false;
        // (the second condition keeps a round of the warm-up, in which every element may pass,
        // from overflowing: a compaction leaves at most kWaveSortMaxKeys keys and the buffer has
        // room for that many plus a round)
        if (done < N && fill > p.K && (fill > cap / 2 || (seen_at_thr == 0 && fill + round > cap))) {
            // new threshold: a key with at least K and at most kWaveSortMaxKeys keys at or above
            // it; the keys below it leave the buffer (through registers: the buffer is compacted
            // in place)
            const uint64_t klo = wg_select_threshold(buf, fill, p.K, scratch);
            if (klo == 0) return false;
            constexpr int kMaxPerThread = 16;               // cap <= 16 * T is checked by the launcher
            uint64_t mine[kMaxPerThread];
#pragma unroll
            for (int j = 0; j < kMaxPerThread; ++j) {
                const int i = tid + j * T;
                mine[j] = (i < fill) ? buf[i] : 0;
            }
            if (tid == 0) ctl[3] = 0;
            __syncthreads();
#pragma unroll
            for (int j = 0; j < kMaxPerThread; ++j)
                if (mine[j] >= klo && mine[j] != 0) buf[atomicAdd(&ctl[3], 1u)] = mine[j];
            __syncthreads();
            fill = (int)ctl[3];
            thr = klo - 1;                  // keys are distinct: "above klo - 1" is "at or above klo"
            seen_at_thr = done;
            __syncthreads();
        }
    }
    count = fill;
    return true;
}

// MINK: the mirrored problem (the K smallest): every loaded pattern passes through the
// order-reversing xor p.flip; the Top-K instantiation carries no trace of it.
// NV > 0: a short row (at most NV 16-byte vectors per thread of a 256-thread workgroup, N a
// multiple of the vector length) is loaded into registers once, all loads in flight together, and
// every pass below runs over the registers: one trip to memory instead of one per chunk and pass,
// which is what a row of a few tens of kilobytes spends its time on.
template <typename DT, bool PAYLOAD, bool VEC, bool MINK, int NV = 0>
__global__ void __launch_bounds__(NV > 0 ? kRegRowThreads : 1024, NV > 0 ? 4 : 1) topk_exact_kernel(TopkParams p) {
    static_assert(NV == 0 || (VEC && !PAYLOAD), "rows in registers: vector loads of the row itself");
    const uint32_t flip = MINK ? p.flip : 0u;
    extern __shared__ uint64_t lds64[];
    // layout: [0, cap) key buffer (the histogram aliases its start), scratch of the final
    // selection, then 32 control words
    uint32_t* hist = (uint32_t*)lds64;
    void* scratch = lds64 + p.cap;
    uint32_t* ctl = (uint32_t*)((char*)scratch + kSelectScratchBytes);   // 3: fill  4..: wave sums
    const int tid = threadIdx.x, T = blockDim.x;
    const int row = blockIdx.x;
    if (p.row_mask && p.row_mask[row] == 0) return;      // (uniform: the whole workgroup leaves)
    const char* rowp = (const char*)p.values + (size_t)row * p.row_stride * elem<DT>::size;
    const int32_t* payload = PAYLOAD ? p.payload + (size_t)row * p.row_stride : nullptr;
    const int N = p.N;
    auto index_of = [&](int n) -> uint32_t { return PAYLOAD ? (uint32_t)payload[n] : (uint32_t)n; };

    constexpr int VE = 16 / elem<DT>::size;
    uint4 regs[NV > 0 ? NV : 1];
    if constexpr (NV > 0) {
        const uint4* vp = (const uint4*)rowp;
        const int nvec = N / VE;
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const int i = u * T + tid;
            regs[u] = i < nvec ? vp[i] : uint4{0u, 0u, 0u, 0u};
        }
    }
    // fn(bits, n) for every element n in [begin, end) (begin a multiple of T * VE when NV > 0)
    auto each = [&](int begin, int end, auto&& fn) {
        if constexpr (NV > 0) {
#pragma unroll
            for (int u = 0; u < NV; ++u) {
                const int first = (u * T + tid) * VE;            // this thread's elements of vector u
                if (first >= begin && first < end) {
                    const uint32_t* w = (const uint32_t*)&regs[u];
#pragma unroll
                    for (int e = 0; e < VE; ++e) {
                        uint32_t b;
                        if constexpr (elem<DT>::size == 4) b = w[e];
                        else b = (e & 1) ? (w[e >> 1] & 0xffff0000u) : (w[e >> 1] << 16);
                        fn(b, first + e);
                    }
                }
            }
        } else {
            for_each_element<DT, VEC>(rowp, begin, end, fn);
        }
    };

    if (NV == 0 && p.onepass) {
        int count = 0;
        if (onepass<DT, PAYLOAD, VEC, MINK>(p, rowp, payload, lds64, scratch, ctl, count)) {
            const int n1 = next_pow2(count);
            for (int i = count + tid; i < n1; i += T) lds64[i] = 0;
            __syncthreads();
            const char* bits_row1 = PAYLOAD ? (const char*)p.orig_values + (size_t)row * p.orig_stride * elem<DT>::size : rowp;
            wg_topk_from_lds<DT>(lds64, n1, p.K, scratch, bits_row1, p.out_vals, p.out_idx, (int64_t)row * p.K, flip);
            return;
        }
        __syncthreads();
    }

    uint64_t prefix = 0, mask = 0;
    int need = p.K;          // members still to be taken from the keys matching the prefix
    int certain = 0;         // members already known (keys above the prefix)

    // ---- digit 0 with a rising lower bound ------------------------------------------------------
    {
        for (int i = tid; i < kSelectBins; i += T) hist[i] = 0;
        __syncthreads();
        // vectors per lane and chunk: more in flight on long rows, early lower bound on short ones
        // (a row in registers is counted in one sweep: finding a lower bound costs more than the
        // atomics it would save)
        const int chunk = NV > 0 ? N : T * VE * (N >= 131072 ? 8 : (N >= 32768 ? 4 : 1));
        uint32_t dmin = 0;
        int next_update = chunk;
        for (int base = 0; base < N; base += chunk) {
            const int end = min(N, base + chunk);
            // (one compare of the stored value rejects what lies below the lower bound)
            const uint32_t dmin_bits = elem<DT>::floor_bits(dmin << 21);
            each(base, end, [&](uint32_t b, int) {
                b ^= flip;
                if (elem<DT>::ge(b, dmin_bits)) atomicAdd(&hist[elem<DT>::ordered(b) >> 21], 1u);
            });
            // (only once at least K keys have been counted: the walk needs K of them)
            if (end >= next_update && end < N && end >= p.K) {
                uint32_t digit, above, count;
                hist_find_digit(hist, ctl, p.K, digit, above, count);
                dmin = digit;                    // K keys at or above this digit exist already
                next_update = next_update <= 0x3fffffff ? next_update * 2 : 0x7fffffff;
            }
        }
        uint32_t digit, above, count;
        hist_find_digit(hist, ctl, need, digit, above, count);
        certain += (int)above;
        need -= (int)above;
        prefix = (uint64_t)digit << 53;
        mask = (uint64_t)0x7ff << 53;
        // ---- further digits, only when ties leave more than the buffer holds ---------------
        for (int d = 1; d < kNumDigits && certain + (int)count > p.cap; ++d) {
            const int shift = kDigitShift[d];
            const uint32_t dmask = (1u << kDigitBits[d]) - 1u;
            for (int i = tid; i < kSelectBins; i += T) hist[i] = 0;
            __syncthreads();
            each(0, N, [&](uint32_t b, int n) {
                const uint64_t key = make_key<DT>(b ^ flip, index_of(n));
                if ((key & mask) == prefix) atomicAdd(&hist[(uint32_t)(key >> shift) & dmask], 1u);
            });
            hist_find_digit(hist, ctl, need, digit, above, count);
            certain += (int)above;
            need -= (int)above;
            prefix |= (uint64_t)digit << shift;
            mask |= (uint64_t)dmask << shift;
        }
    }

    // ---- gather certain members and prefix matches ----------------------------------------------
    if (tid == 0) ctl[3] = 0;
    __syncthreads();
    const uint32_t prefix_bits = elem<DT>::floor_bits((uint32_t)(prefix >> 32));
    if constexpr (NV > 0) {
        // from registers: count first, reserve the slots of a whole wavefront with one atomic, then
        // store -- instead of one atomic round trip per element that qualifies
        // With the leading digit alone as prefix -- the usual case -- one compare of the stored
        // value decides: it holds exactly when the key's leading digit is at or above the prefix's.
        const bool one_digit = mask == ((uint64_t)0x7ff << 53);
        auto general = [&](uint32_t b, int n, uint64_t& key) {
            if (!elem<DT>::ge(b, prefix_bits)) return false;
            key = make_key<DT>(b, (uint32_t)n);
            return (key & mask) >= prefix;
        };
        int mine = 0;
        if (one_digit) {
            each(0, N, [&](uint32_t b, int) { mine += elem<DT>::ge(b ^ flip, prefix_bits) ? 1 : 0; });
        } else {
            each(0, N, [&](uint32_t b, int n) {
                uint64_t key;
                if (general(b ^ flip, n, key)) ++mine;
            });
        }
        const int lane = tid & (kWave - 1);
        int incl = mine;
        for (int o = 1; o < kWave; o <<= 1) {
            const int other = __shfl_up(incl, o, kWave);
            if (lane >= o) incl += other;
        }
        uint32_t base = 0;
        if (lane == kWave - 1 && incl > 0) base = atomicAdd(&ctl[3], (uint32_t)incl);
        base = (uint32_t)__shfl((int)base, kWave - 1, kWave);
        uint32_t slot = base + (uint32_t)(incl - mine);
        // (slot < cap always holds; the test keeps a slip memory safe)
        if (one_digit) {
            each(0, N, [&](uint32_t b, int n) {
                if (elem<DT>::ge(b ^ flip, prefix_bits)) {
                    if (slot < (uint32_t)p.cap) lds64[slot] = make_key<DT>(b ^ flip, (uint32_t)n);
                    ++slot;
                }
            });
        } else {
            each(0, N, [&](uint32_t b, int n) {
                uint64_t key;
                if (general(b ^ flip, n, key)) {
                    if (slot < (uint32_t)p.cap) lds64[slot] = key;
                    ++slot;
                }
            });
        }
    } else
    each(0, N, [&](uint32_t b, int n) {
        // cheap reject on the stored value before the key is built
        b ^= flip;
        if (elem<DT>::ge(b, prefix_bits)) {
            const uint64_t key = make_key<DT>(b, index_of(n));
            if ((key & mask) >= prefix) {
                const uint32_t slot = atomicAdd(&ctl[3], 1u);
                if (slot < (uint32_t)p.cap) lds64[slot] = key;   // always true; keeps a slip memory safe
            }
        }
    });
    __syncthreads();
    const int total = min((int)ctl[3], p.cap);
    const int n2 = next_pow2(total);
    for (int i = total + tid; i < n2; i += T) lds64[i] = 0;
    __syncthreads();
    // survivor mode: a key's index is the original position, so a zero's stored bits are re-read
    // from the original row like everywhere else
    const char* bits_row = PAYLOAD ? (const char*)p.orig_values + (size_t)row * p.orig_stride * elem<DT>::size : rowp;
    wg_topk_from_lds<DT>(lds64, n2, p.K, scratch, bits_row, p.out_vals, p.out_idx, (int64_t)row * p.K, flip);
}

template <typename DT>
hipError_t launch_for(const TopkParams& p, int threads, hipStream_t stream) {
    const size_t lds = (size_t)p.cap * 8 + kSelectScratchBytes + 32 * 4;
    const dim3 grid(p.rows), block(threads);
    const bool vec = p.payload == nullptr && ((uintptr_t)p.values % 16 == 0) &&
                     ((p.row_stride * elem<DT>::size) % 16 == 0);
    auto launch = [&](auto kernel) {
        allow_large_lds((const void*)kernel, lds);
        hipLaunchKernelGGL(kernel, grid, block, lds, stream, p);
    };
    constexpr int VE = 16 / elem<DT>::size;
    const bool in_regs = vec && p.reg_row && threads == kRegRowThreads && p.N % VE == 0 &&
                         p.N <= kRegRowThreads * VE * kRegRowVectors;
    if (p.flip == 0) {
        if (p.payload)    launch(topk_exact_kernel<DT, true, false, false>);
        else if (in_regs) launch(topk_exact_kernel<DT, false, true, false, kRegRowVectors>);
        else if (vec)     launch(topk_exact_kernel<DT, false, true, false>);
        else              launch(topk_exact_kernel<DT, false, false, false>);
    } else {
        if (p.payload)    launch(topk_exact_kernel<DT, true, false, true>);
        else if (in_regs) launch(topk_exact_kernel<DT, false, true, true, kRegRowVectors>);
        else if (vec)     launch(topk_exact_kernel<DT, false, true, true>);
        else              launch(topk_exact_kernel<DT, false, false, true>);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_topk_exact(const TopkParams& p, int dtype, int threads, hipStream_t stream) {
    switch (dtype) {
        case 0: return launch_for<float>(p, threads, stream);
        case 1: return launch_for<bf16_t>(p, threads, stream);
        case 3: return launch_for<i32_t>(p, threads, stream);
        case 4: return launch_for<u32_t>(p, threads, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace atk
