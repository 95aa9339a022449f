// Stage 2 building blocks: exact Top-K of keys that already sit in LDS or registers
// (Section 6.1 Step 4: sort the merged survivors, keep the first K).
//
//   WaveSort<R>      bitonic sort of 64*R keys held R per lane in the registers of one
//                    wavefront: compare-exchanges between registers of a lane are plain
//                    selects, those between lanes fetch the partner's key with a cross-lane
//                    shuffle.  No LDS traffic, no barriers.
//   wg_topk_from_lds workgroup-level Top-K of n keys in LDS.  Small inputs go straight to a
//                    wave sort.  Larger ones are first cut down by selection (an LDS histogram
//                    over equal bins of the interval of keys present finds the bin that holds
//                    the K-th key; keys above it are certain members, keys inside it candidates)
//                    and only the members and candidates are sorted.  A full LDS bitonic sort
//                    remains as the fallback.
#pragma once
#include "atk_device.h"

namespace atk {

constexpr int kWaveSortMaxR = 16;                       // up to 1024 keys per wavefront
constexpr int kWaveSortMaxKeys = kWave * kWaveSortMaxR;
constexpr int kSelectBinBits = 11;
constexpr int kSelectBins = 1 << kSelectBinBits;
// LDS scratch wg_topk_from_lds needs next to the keys when n > 256:
// a compaction buffer of kWaveSortMaxKeys keys (the histogram aliases it) + control words.
constexpr int kSelectScratchBytes = kWaveSortMaxKeys * 8 + 128;

// Value of `x` in lane (lane ^ m).  Distances that a DPP pattern can express (neighbours in a
// quad, mirror images inside 4, 8 or 16 lanes) are plain vector moves; the rest go through the
// cross-lane permute.  m is a constant after unrolling, so only one form survives.
__device__ __forceinline__ uint32_t lane_xor(uint32_t x, int m) {
    if (m == 1) return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0xB1, 0xF, 0xF, true);   // quad_perm [1,0,3,2]
    if (m == 2) return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0x4E, 0xF, 0xF, true);   // quad_perm [2,3,0,1]
    if (m == 3) return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0x1B, 0xF, 0xF, true);   // quad_perm [3,2,1,0]
    if (m == 7) return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0x141, 0xF, 0xF, true);  // row_half_mirror
    if (m == 15) return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0x140, 0xF, 0xF, true); // row_mirror
    return (uint32_t)__shfl_xor((unsigned)x, m, kWave);
}
template <typename KeyT>
__device__ __forceinline__ KeyT lane_xor_key(KeyT x, int m) {
    if constexpr (sizeof(KeyT) == 4) return lane_xor((uint32_t)x, m);
    else return ((uint64_t)lane_xor((uint32_t)(x >> 32), m) << 32) | lane_xor((uint32_t)x, m);
}

// median of three unsigned words.  Written as the instruction itself: the equivalent min/max
// expression sends the optimizer into exponential work on chains of list updates.
__device__ __forceinline__ uint32_t med3_u32(uint32_t a, uint32_t b, uint32_t c) {
    uint32_t d;
    asm("v_med3_u32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
    return d;
}

// Bitonic sorting network in the form whose comparators all point the same way: level kk first
// compares every element e with its mirror image e ^ (kk-1) inside the block, then with
// e ^ (kk/4), ..., e ^ 1; the lower index always keeps the greater key.
template <int R, typename KeyT = uint64_t>
struct WaveSort {
    static constexpr int LOGR = (R == 1 ? 0 : R == 2 ? 1 : R == 4 ? 2 : R == 8 ? 3 : 4);
    static constexpr int LOGN = LOGR + 6;
    static_assert(R == 1 || R == 2 || R == 4 || R == 8 || R == 16, "R must be 1,2,4,8,16");

    __device__ static __forceinline__ void cex(KeyT& hi, KeyT& lo) {     // hi := greater, lo := smaller
        const KeyT a = hi, b = lo;
        if constexpr (sizeof(KeyT) == 4) { hi = max(a, b); lo = min(a, b); }
        else { const bool sw = a < b; hi = sw ? b : a; lo = sw ? a : b; }
    }
    // The greater (want_max) or the smaller of a and b; want_max differs from lane to lane.  The
    // 32-bit form is one median of three: with the greatest word as third operand the median
    // of (a, b, .) is max(a, b), with zero it is min(a, b).
    __device__ static __forceinline__ KeyT pick(KeyT a, KeyT b, bool want_max) {
        if constexpr (sizeof(KeyT) == 4) {
            return med3_u32(a, b, want_max ? 0xffffffffu : 0u);
        } else {
            const bool take_b = (b > a) == want_max;
            return take_b ? b : a;
        }
    }

    // One half-cleaner step at element distance JJ.
    template <int JJ>
    __device__ static __forceinline__ void step(KeyT (&k)[R], int lane) {
        if constexpr (JJ < R) {
#pragma unroll
            for (int j = 0; j < R; ++j)
                if ((j & JJ) == 0) cex(k[j], k[j | JJ]);
        } else {
            constexpr int M = JJ / R;
            const bool lower = (lane & M) == 0;
#pragma unroll
            for (int j = 0; j < R; ++j) k[j] = pick(k[j], lane_xor_key<KeyT>(k[j], M), lower);
        }
    }
    template <int LJ>
    __device__ static __forceinline__ void steps_down(KeyT (&k)[R], int lane) {
        if constexpr (LJ >= 0) {
            step<(1 << LJ)>(k, lane);
            steps_down<LJ - 1>(k, lane);
        }
    }
    // Level KK = 2^LK: the mirror step, then the half-cleaners; then the next level.  Templates
    // rather than loops: every distance must be a compile-time constant (register indices, DPP
    // patterns), whatever the unroller decides.
    template <int LK>
    __device__ static __forceinline__ void levels(KeyT (&k)[R], int lane, int last_level = LOGN) {
        if constexpr (LK <= LOGN) {
            if (LK > last_level) return;       // uniform; folds away when the default is used
            constexpr int KK = 1 << LK;
            if constexpr (KK <= R) {
#pragma unroll
                for (int j = 0; j < R; ++j)
                    if ((j & (KK >> 1)) == 0) cex(k[j], k[j ^ (KK - 1)]);
            } else {
                constexpr int LM = KK / R - 1;                    // lane part of the mirror mask
                const bool lower = (lane & ((KK >> 1) / R)) == 0;
                KeyT recv[R];
#pragma unroll
                for (int j = 0; j < R; ++j) recv[j] = lane_xor_key<KeyT>(k[j ^ (R - 1)], LM);
#pragma unroll
                for (int j = 0; j < R; ++j) k[j] = pick(k[j], recv[j], lower);
            }
            steps_down<LK - 2>(k, lane);
            levels<LK + 1>(k, lane, last_level);
        }
    }

    // Element e = lane*R + j lives in k[j] of `lane`.  After the call e is the rank: k[j] of
    // lane l is the (l*R + j)-th greatest key.
    __device__ static void sort(KeyT (&k)[R]) { levels<1>(k, __lane_id()); }
    // The first log_len levels only: every aligned block of 2^log_len elements ends up sorted.
    __device__ static void sort_blocks(KeyT (&k)[R], int log_len) { levels<1>(k, __lane_id(), log_len); }
};

// A pointer known to point into LDS.  The sorting tails are not inlined and receive generic
// pointers; through this type their accesses are LDS instructions rather than flat ones.
template <typename T> using lds_ptr = __attribute__((address_space(3))) T*;

// Stored bit pattern of the element a key stands for.  Keys are built from values after the
// order-reversing map of the min-K problem (`flip`: 0 for Top-K; xor-ed onto the pattern: the sign
// bit of floating types, all bits of integers), so the pattern comes back through the same xor;
// a zero is re-read from the row, where its sign is (rowp; not read for scores, whose zero is +0.0).
template <typename DT>
__device__ __forceinline__ uint32_t key_stored_bits(uint64_t key, const void* rowp, uint32_t index, uint32_t flip) {
    const uint32_t bits = key_value_bits<DT>(key);
    if (bits == 0 && key != 0) return elem<DT>::load_bits(rowp, index);
    return bits ^ flip;
}

// Position in a staging array of LDS for the key of rank e, chosen so that neither a wavefront
// writing its registers (lane l, register j holds rank l*R + j) nor one reading ranks lane,
// lane + 64, ... meets bank conflicts beyond the width of the access: the position inside each
// aligned group of R is xor-ed with higher rank bits.  WORDS = 32-bit words per key.
template <int R, int WORDS>
__device__ __forceinline__ int staged_rank(int e) {
    return e ^ ((e >> (WORDS == 2 ? 5 : 6)) & (R - 1));
}

// Decode and write the first K of the sorted keys of one wavefront (lane l, register j holds
// rank l*R + j).  The keys pass through `stage` (LDS; only the ranks below K rounded up to a
// multiple of R are touched) so that consecutive lanes write consecutive outputs.
template <typename DT, int R>
__device__ __forceinline__ void wave_write_topk(const uint64_t (&k)[R], int K, const void* rowp,
                                                void* out_vals, int32_t* out_idx, int64_t out_base,
                                                uint64_t* stage_generic, uint32_t flip = 0) {
    lds_ptr<uint64_t> stage = (lds_ptr<uint64_t>)stage_generic;
    const int lane = __lane_id();
    if (lane * R < K) {
#pragma unroll
        for (int j = 0; j < R; ++j) stage[staged_rank<R, 2>(lane * R + j)] = k[j];
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    for (int e = lane; e < K; e += kWave) {
        const uint64_t key = stage[staged_rank<R, 2>(e)];
        const uint32_t n = key_index(key);
        elem<DT>::store_bits(out_vals, out_base + e, key_stored_bits<DT>(key, rowp, n, flip));
        out_idx[out_base + e] = (int32_t)n;
    }
}

// One wavefront sorts `n` (<= 64*R) keys read from LDS and writes the first K; the array (room
// for K rounded up to a multiple of R keys) is reused as staging.
template <typename DT, int R>
__device__ __forceinline__ void wave_sort_from_lds(uint64_t* keys_generic, int n, int K, const void* rowp,
                                                   void* out_vals, int32_t* out_idx, int64_t out_base,
                                                   uint32_t flip) {
    lds_ptr<uint64_t> keys = (lds_ptr<uint64_t>)keys_generic;
    const int lane = __lane_id();
    uint64_t k[R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const int i = j * kWave + lane;                 // any assignment will do: conflict-free
        k[j] = i < n ? keys[i] : 0;
    }
    WaveSort<R>::sort(k);
    wave_write_topk<DT, R>(k, K, rowp, out_vals, out_idx, out_base, keys_generic, flip);
}

// Not inlined on purpose: the sorting networks are long, and every streaming kernel variant
// that finishes in LDS shares this one copy per translation unit.
template <typename DT>
__device__ __noinline__ void wave_sort_dispatch(uint64_t* keys, int n, int K, const void* rowp,
                                                   void* out_vals, int32_t* out_idx, int64_t out_base,
                                                   uint32_t flip = 0) {
    if (n <= 64)       wave_sort_from_lds<DT, 1>(keys, n, K, rowp, out_vals, out_idx, out_base, flip);
    else if (n <= 128) wave_sort_from_lds<DT, 2>(keys, n, K, rowp, out_vals, out_idx, out_base, flip);
    else if (n <= 256) wave_sort_from_lds<DT, 4>(keys, n, K, rowp, out_vals, out_idx, out_base, flip);
    else if (n <= 512) wave_sort_from_lds<DT, 8>(keys, n, K, rowp, out_vals, out_idx, out_base, flip);
    else               wave_sort_from_lds<DT, 16>(keys, n, K, rowp, out_vals, out_idx, out_base, flip);
}

// ---- packed 32-bit keys (bf16 rows of at most 65536 elements) ---------------------------------
// key = ordered 16-bit value << 16 | (0xFFFF - index); 0 = empty.
// cert_flag (optional): where to note whether some bucket (index mod cert_B) contributes cert_Kp or
// more of the K results -- the exactness certificate of the two-stage method, taken here while the
// sorted keys sit in registers: 0 = no bucket does, the K results are the exact Top-K of the row.
template <typename DT, int R, bool CERT>
__device__ __forceinline__ void wave_sort32_from_lds(uint32_t* keys_generic, int n, int K, const void* rowp,
                                                     void* out_vals, int32_t* out_idx, int64_t out_base,
                                                     uint32_t flip, int32_t* cert_flag, int cert_B, int cert_Kp) {
    lds_ptr<uint32_t> keys = (lds_ptr<uint32_t>)keys_generic;
    const int lane = __lane_id();
    uint32_t k[R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const int i = j * kWave + lane;
        k[j] = i < n ? keys[i] : 0;
    }
    WaveSort<R, uint32_t>::sort(k);
    if constexpr (CERT) {
        // counters at the end of the key array, behind what the staging below uses (the keys are
        // in registers by now); no room: the question stays open
        bool doubt = true;
        if ((K + R - 1) / R * R + cert_B <= n) {
            lds_ptr<uint32_t> count = keys + (n - cert_B);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            for (int b = lane; b < cert_B; b += kWave) count[b] = 0;
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            const bool pow2 = (cert_B & (cert_B - 1)) == 0;
#pragma unroll
            for (int j = 0; j < R; ++j)
                if (lane * R + j < K && k[j] != 0) {
                    const uint32_t idx = 0xffffu - (k[j] & 0xffffu);
                    const uint32_t b = pow2 ? (idx & (uint32_t)(cert_B - 1)) : idx % (uint32_t)cert_B;
                    atomicAdd((uint32_t*)&count[b], 1u);         // (result unused: nothing to wait for)
                }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            bool full = false;
            for (int b = lane; b < cert_B; b += kWave) full |= count[b] >= (uint32_t)cert_Kp;
            doubt = __ballot(full) != 0;
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        }
        if (lane == 0) *cert_flag = doubt ? 1 : 0;
    }
    // through LDS (the key array itself) so that consecutive lanes write consecutive outputs
    if (lane * R < K) {
#pragma unroll
        for (int j = 0; j < R; ++j) keys[staged_rank<R, 1>(lane * R + j)] = k[j];
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    for (int e = lane; e < K; e += kWave) {
        const uint32_t key = keys[staged_rank<R, 1>(e)];
        const uint32_t idx = 0xffffu - (key & 0xffffu);
        uint32_t bits = bits_from_ordered(key & 0xffff0000u);
        if (bits == 0 && key != 0) bits = elem<DT>::load_bits(rowp, idx);   // which zero it was
        else bits ^= flip;                                                  // (min-K: back through the sign flip)
        elem<DT>::store_bits(out_vals, out_base + e, bits);
        out_idx[out_base + e] = (int32_t)idx;
    }
}

template <typename DT>
__device__ __noinline__ void wave_sort32_dispatch(uint32_t* keys, int n, int K, const void* rowp,
                                                  void* out_vals, int32_t* out_idx, int64_t out_base,
                                                  uint32_t flip = 0) {
    if (n <= 64)       wave_sort32_from_lds<DT, 1, false>(keys, n, K, rowp, out_vals, out_idx, out_base, flip, nullptr, 0, 0);
    else if (n <= 128) wave_sort32_from_lds<DT, 2, false>(keys, n, K, rowp, out_vals, out_idx, out_base, flip, nullptr, 0, 0);
    else if (n <= 256) wave_sort32_from_lds<DT, 4, false>(keys, n, K, rowp, out_vals, out_idx, out_base, flip, nullptr, 0, 0);
    else if (n <= 512) wave_sort32_from_lds<DT, 8, false>(keys, n, K, rowp, out_vals, out_idx, out_base, flip, nullptr, 0, 0);
    else               wave_sort32_from_lds<DT, 16, false>(keys, n, K, rowp, out_vals, out_idx, out_base, flip, nullptr, 0, 0);
}

// The same, taking the exactness certificate on the way (see wave_sort32_from_lds): a copy of its
// own, so that the plain form carries nothing of it.
template <typename DT>
__device__ __noinline__ void wave_sort32_certify_dispatch(uint32_t* keys, int n, int K, const void* rowp,
                                                          void* out_vals, int32_t* out_idx, int64_t out_base,
                                                          uint32_t flip, int32_t* cert_flag, int cert_B, int cert_Kp) {
    if (n <= 64)       wave_sort32_from_lds<DT, 1, true>(keys, n, K, rowp, out_vals, out_idx, out_base, flip, cert_flag, cert_B, cert_Kp);
    else if (n <= 128) wave_sort32_from_lds<DT, 2, true>(keys, n, K, rowp, out_vals, out_idx, out_base, flip, cert_flag, cert_B, cert_Kp);
    else if (n <= 256) wave_sort32_from_lds<DT, 4, true>(keys, n, K, rowp, out_vals, out_idx, out_base, flip, cert_flag, cert_B, cert_Kp);
    else if (n <= 512) wave_sort32_from_lds<DT, 8, true>(keys, n, K, rowp, out_vals, out_idx, out_base, flip, cert_flag, cert_B, cert_Kp);
    else               wave_sort32_from_lds<DT, 16, true>(keys, n, K, rowp, out_vals, out_idx, out_base, flip, cert_flag, cert_B, cert_Kp);
}

// Slab route of the streaming kernel: the 64*R keys at `keys` (LDS) are the partial lists of
// 64/m buckets, m*R consecutive keys per bucket (m lanes' worth).  One wavefront sorts every
// bucket's keys in registers and the first lane of each bucket writes its K' greatest to
// out[j*B + bucket] (j < K').  No barrier inside: each wavefront works on its own buckets.
template <int R>
__device__ __forceinline__ void wave_merge_bucket_lists(const uint64_t* keys_generic, int log_m,
                                                        int Kprime, uint64_t* out, int B) {
    const lds_ptr<const uint64_t> keys = (lds_ptr<const uint64_t>)keys_generic;
    const int lane = __lane_id();
    uint64_t k[R];
#pragma unroll
    for (int j = 0; j < R; ++j) k[j] = keys[lane * R + j];
    WaveSort<R>::sort_blocks(k, WaveSort<R>::LOGR + log_m);
    if ((lane & ((1 << log_m) - 1)) == 0) {
#pragma unroll
        for (int j = 0; j < R; ++j)
            if (j < Kprime) out[(size_t)j * B + (lane >> log_m)] = k[j];
    }
}
// (not inlined: five sorting networks that every streaming kernel variant would carry)
__device__ __noinline__ bool wave_merge_bucket_lists_dispatch(const uint64_t* keys, int R, int log_m,
                                                              int Kprime, uint64_t* out, int B) {
    switch (R) {
        case 1:  wave_merge_bucket_lists<1>(keys, log_m, Kprime, out, B); return true;
        case 2:  wave_merge_bucket_lists<2>(keys, log_m, Kprime, out, B); return true;
        case 4:  wave_merge_bucket_lists<4>(keys, log_m, Kprime, out, B); return true;
        case 8:  wave_merge_bucket_lists<8>(keys, log_m, Kprime, out, B); return true;
        case 16: wave_merge_bucket_lists<16>(keys, log_m, Kprime, out, B); return true;
        default: return false;
    }
}

// Routes with the ranking finish: one wavefront sorts the n = 64*R keys at `keys` (LDS: final
// list entries, zeros where there are none) and writes them to out[0, n) in rank order, the
// greatest first.  (n = 32: the upper half of the wavefront holds zeros.)
template <int R>
__device__ __forceinline__ void wave_sort_run(const uint64_t* keys_generic, int n, uint64_t* out) {
    const lds_ptr<const uint64_t> keys = (lds_ptr<const uint64_t>)keys_generic;
    const int lane = __lane_id();
    uint64_t k[R];
#pragma unroll
    for (int j = 0; j < R; ++j) k[j] = j * kWave + lane < n ? keys[j * kWave + lane] : 0;   // (any assignment will do)
    WaveSort<R>::sort(k);
#pragma unroll
    for (int j = 0; j < R; ++j)
        if (lane * R + j < n) out[lane * R + j] = k[j];
}
__device__ __noinline__ void wave_sort_run_dispatch(const uint64_t* keys, int n, uint64_t* out) {
    if (n <= 64)       wave_sort_run<1>(keys, n, out);
    else if (n <= 128) wave_sort_run<2>(keys, n, out);
    else if (n <= 256) wave_sort_run<4>(keys, n, out);
    else if (n <= 512) wave_sort_run<8>(keys, n, out);
    else               wave_sort_run<16>(keys, n, out);
}

// Walk a finished histogram from the top bin down.  On return (all threads):
//   digit   the bin in which the running count reaches `need`,
//   above   the total of the bins above it,
//   count   the content of that bin.
// Bins that no key of interest can fall into may hold anything as long as the bins from the
// top down to the answer are exact.  hist: kSelectBins words, ctl: 32 words of LDS scratch.
// Starts and ends with a barrier.
__device__ __forceinline__ void hist_find_digit(const uint32_t* hist, uint32_t* ctl, int need,
                                                uint32_t& digit, uint32_t& above, uint32_t& count) {
    const int tid = threadIdx.x, T = blockDim.x;
    if (tid == 0) { ctl[0] = 0; ctl[1] = 0; ctl[2] = 0; }   // answer if fewer than `need` were counted
    __syncthreads();
    // suffix sums over bins: thread t owns bins [t*bpt, (t+1)*bpt)
    const int bpt = (kSelectBins + T - 1) / T;
    uint32_t mine = 0;
    if ((bpt & 3) == 0) {                     // 16-byte loads (kSelectBins and T are powers of two)
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
        for (int i = 0; i < bpt; i += 4) {
            const u32x4 h = *(const u32x4*)(hist + tid * bpt + i);
            mine += h.x + h.y + h.z + h.w;
        }
    } else {
        for (int i = 0; i < bpt; ++i) {
            const int bin = tid * bpt + i;
            if (bin < kSelectBins) mine += hist[bin];
        }
    }
    const int lane = tid & (kWave - 1), wave = tid >> 6;
    uint32_t suf = mine;                               // inclusive suffix sum inside the wave
    for (int o = 1; o < kWave; o <<= 1) {
        const uint32_t other = __shfl_down(suf, o, kWave);
        if (lane + o < kWave) suf += other;
    }
    if (lane == 0) ctl[4 + wave] = suf;
    __syncthreads();
    // waves after mine: lane l fetches the total of wave l (at most 16 of them), a reduction over
    // the wavefront adds up the later ones -- one LDS round trip instead of one per wave
    const int nwaves = (T + kWave - 1) / kWave;
    uint32_t later = (lane < nwaves && lane > wave) ? ctl[4 + lane] : 0u;
    for (int o = 8; o >= 1; o >>= 1) later += (uint32_t)__shfl_xor((int)later, o, kWave);
    later = (uint32_t)__shfl((int)later, 0, kWave);
    const uint32_t incl = suf + later, excl = incl - mine;
    if (excl < (uint32_t)need && incl >= (uint32_t)need) {
        uint32_t run = excl;
        for (int i = bpt - 1; i >= 0; --i) {
            const int bin = tid * bpt + i;
            if (bin >= kSelectBins) continue;
            const uint32_t c = hist[bin];
            if (run + c >= (uint32_t)need) {
                ctl[0] = (uint32_t)bin; ctl[1] = run; ctl[2] = c;
                break;
            }
            run += c;
        }
    }
    __syncthreads();
    digit = ctl[0]; above = ctl[1]; count = ctl[2];
    __syncthreads();
}

// Visit the n keys of an LDS array, every thread of the workgroup taking keys tid, tid+T, ...;
// four loads are issued before the first key is used so that their latencies overlap.
template <typename F>
__device__ __forceinline__ void for_each_lds_key(const uint64_t* keys, int n, F&& f) {
    const int tid = threadIdx.x, T = blockDim.x;
    for (int base = tid; base < n; base += 4 * T) {
        uint64_t k[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) k[u] = (base + u * T < n) ? keys[base + u * T] : 0;
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (base + u * T < n) f(k[u]);
    }
}

// Histogram pass of the selection over keys in LDS: the keys inside [klo, khi] are counted in
// bins of 2^shift consecutive keys starting at klo (the caller picks shift so that the interval
// spans at most kSelectBins bins), then hist_find_digit answers.
__device__ __forceinline__ void lds_select_bin(const uint64_t* keys, int n, uint64_t klo, uint64_t khi,
                                               int shift, int need, uint32_t* hist, uint32_t* ctl,
                                               uint32_t& digit, uint32_t& above, uint32_t& count) {
    const int tid = threadIdx.x, T = blockDim.x;
    for (int i = tid; i < kSelectBins; i += T) hist[i] = 0;
    __syncthreads();
    for_each_lds_key(keys, n, [&](uint64_t key) {
        if (key >= klo && key <= khi) atomicAdd(&hist[(uint32_t)((key - klo) >> shift)], 1u);
    });
    hist_find_digit(hist, ctl, need, digit, above, count);
}

// Decode and write the first K keys of a sorted LDS array; every thread of the workgroup.
template <typename DT>
__device__ __forceinline__ void wg_write_topk(const uint64_t* keys, int K, const void* rowp,
                                              void* out_vals, int32_t* out_idx, int64_t out_base,
                                              uint32_t flip = 0) {
    for (int i = threadIdx.x; i < K; i += blockDim.x) {
        const uint64_t key = keys[i];
        const uint32_t idx = key_index(key);
        elem<DT>::store_bits(out_vals, out_base + i, key_stored_bits<DT>(key, rowp, idx, flip));
        out_idx[out_base + i] = (int32_t)idx;
    }
}

// One wavefront sorts up to kWaveSortMaxKeys keys in registers; beyond kWgSortMinKeys keys a
// workgroup of at least kWgSortMinThreads threads is faster sorting them in LDS together.
constexpr int kWgSortMinKeys = 256;
constexpr int kWgSortMinThreads = 256;
constexpr int kSideSortKeys = 256;      // a boundary bin of at most this many keys is sorted, not split

// Sort n keys in LDS (n a power of two >= 128 R) far enough that keys[0..K) hold the K greatest
// in order.  Every wavefront sorts runs of 64 R keys in registers; the runs are then merged
// pairwise by the bitonic network in its same-direction form (run a against the mirror image of
// run b, then half-cleaners), and once a merged run would exceed `cap` keys (the power of two
// >= K, at least one run) only its first `cap` positions are kept and cleaned.  A merge level
// costs one barrier-separated LDS stage per distance of a run length and more, plus one pass
// through registers for the shorter distances.  A lone wavefront needs about 5 us for 512 keys
// (the network is one long dependency chain), so short runs on many wavefronts win: R is chosen
// by the caller to give every wavefront a run.  Every thread of the workgroup.
template <int R>
__device__ __forceinline__ void wg_sort_merge_runs(uint64_t* keys_generic, int n, int K) {
    using WS = WaveSort<R, uint64_t>;
    const lds_ptr<uint64_t> keys = (lds_ptr<uint64_t>)keys_generic;
    const int tid = threadIdx.x, T = blockDim.x;
    const int lane = tid & (kWave - 1), wave = tid >> 6, nwaves = T >> 6;
    constexpr int kRun = kWave * R;
    for (int c = wave; c < n / kRun; c += nwaves) {
        uint64_t k[R];
#pragma unroll
        for (int j = 0; j < R; ++j) k[j] = keys[c * kRun + lane * R + j];
        WS::sort(k);
#pragma unroll
        for (int j = 0; j < R; ++j) keys[c * kRun + lane * R + j] = k[j];
    }
    __syncthreads();
    int cap = kRun;
    while (cap < K) cap <<= 1;
    for (int L = kRun; L < n; L <<= 1) {                 // blocks of 2L: runs at +0 and +L
        const int m = L < cap ? L : cap;                 // sorted keys at the start of each run
        const int nblocks = n / (2 * L);
        // mirror step: key i of the first run against key m-1-i of the second; the greater
        // stays in the first run, the smaller goes to the second (unused once runs are cut)
        for (int q = tid; q < nblocks * m; q += T) {
            const int blk = q / m, i = q - blk * m;
            const int a = blk * 2 * L + i, b = blk * 2 * L + L + (m - 1 - i);
            const uint64_t x = keys[a], y = keys[b];
            if (x < y) { keys[a] = y; keys[b] = x; }
        }
        __syncthreads();
        // half-cleaners inside what is kept: both runs while 2m <= cap, else the first run only.
        // Distances of a run length and more go through LDS ...
        const int kept = 2 * m <= cap ? 2 * m : m;       // keys kept per block, from its start
        for (int j = m >> 1; j >= kRun; j >>= 1) {
            for (int q = tid; q < nblocks * (kept >> 1); q += T) {
                const int blk = q / (kept >> 1), i = q - blk * (kept >> 1);
                const int lo = blk * 2 * L + (((i & ~(j - 1)) << 1) | (i & (j - 1)));
                const int hi = lo | j;
                const uint64_t x = keys[lo], y = keys[hi];
                if (x < y) { keys[lo] = y; keys[hi] = x; }
            }
            __syncthreads();
        }
        // ... the shorter ones stay inside aligned pieces of one run length: a wavefront takes a
        // piece into registers and runs all of them there
        const int pieces = kept / kRun;
        for (int c = wave; c < nblocks * pieces; c += nwaves) {
            const int blk = c / pieces;
            const lds_ptr<uint64_t> piece = keys + blk * 2 * L + (c - blk * pieces) * kRun;
            uint64_t k[R];
#pragma unroll
            for (int j = 0; j < R; ++j) k[j] = piece[lane * R + j];
            WS::template steps_down<WS::LOGN - 1>(k, lane);      // distances kRun/2 ... 1
#pragma unroll
            for (int j = 0; j < R; ++j) piece[lane * R + j] = k[j];
        }
        __syncthreads();
    }
}

// The same result by ranking instead of merging, for at most one run per wavefront: after the
// runs are sorted, the final position of a key is its position in its own run plus, for every
// other run, the number of keys there that are greater (a binary search; neighbouring lanes
// hold neighbouring keys and mostly read the same words).  Keys are distinct (the index is part
// of them) except for the empty key 0, whose copies all get the same position behind every real
// key: positions below the number of real keys are written exactly once, and K never exceeds
// that number.  Three barriers in all, whatever the number of runs.
template <int R>
__device__ __forceinline__ void wg_sort_rank_runs(uint64_t* keys_generic, int n, int K) {
    using WS = WaveSort<R, uint64_t>;
    const lds_ptr<uint64_t> keys = (lds_ptr<uint64_t>)keys_generic;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid >> 6;
    constexpr int kRun = kWave * R;
    const int nruns = n / kRun;                          // <= wavefronts of the workgroup
    uint64_t k[R];
    if (wave < nruns) {
#pragma unroll
        for (int j = 0; j < R; ++j) k[j] = keys[wave * kRun + lane * R + j];
        WS::sort(k);
#pragma unroll
        for (int j = 0; j < R; ++j) keys[wave * kRun + lane * R + j] = k[j];
    }
    __syncthreads();
    int rank[R];
    if (wave < nruns) {
#pragma unroll
        for (int j = 0; j < R; ++j) rank[j] = lane * R + j;
        for (int r = 0; r < nruns; ++r) {
            if (r == wave) continue;
            const lds_ptr<uint64_t> run = keys + r * kRun;
#pragma unroll
            for (int j = 0; j < R; ++j) {
                int pos = 0;                             // keys of `run` greater than k[j]
#pragma unroll
                for (int s = kRun / 2; s >= 1; s >>= 1)
                    if (run[pos + s - 1] > k[j]) pos += s;
                if (run[pos] > k[j]) pos += 1;
                rank[j] += pos;
            }
        }
    }
    __syncthreads();
    if (wave < nruns) {
#pragma unroll
        for (int j = 0; j < R; ++j)
            if (rank[j] < K) keys[rank[j]] = k[j];
    }
    __syncthreads();
}

// n >= 256: a multiple of 128 up to 128 keys per wavefront, of 256 up to 256 per wavefront, a
// power of two beyond.  Not inlined: the sorting networks that every kernel variant with a stage 2
// would otherwise carry a copy of.
__device__ __noinline__ void wg_sort_merge_topk(uint64_t* keys, int n, int K) {
    const int per_wave = n / (int)(blockDim.x >> 6);      // keys per wavefront if all take part
    if (per_wave <= 128)      wg_sort_rank_runs<2>(keys, n, K);
    else if (per_wave <= 256) wg_sort_rank_runs<4>(keys, n, K);
    else                      wg_sort_merge_runs<8>(keys, n, K);   // (ranking 8 keys per lane: slower)
}

// A key klo among the n keys in LDS `keys` (key 0 = empty; at least K real keys; K at most
// cap) such that the keys >= klo number at least K and at most cap (by default what one
// wavefront sorts) -- usually at most 2K + 64: the K greatest keys are among them and they fit one sort.  Returns 0
// if no such key was found (cannot happen; callers fall back to sorting everything).  Called by
// every thread of the workgroup, ends with a barrier; `scratch` as for wg_topk_from_lds (the
// histogram and a buffer of kSideSortKeys keys alias its start).
__device__ __noinline__ uint64_t wg_select_threshold(const uint64_t* keys, int n, int K, void* scratch,
                                                     int cap = kWaveSortMaxKeys) {
    const int tid = threadIdx.x;
    uint64_t* buf = (uint64_t*)scratch;
    uint32_t* hist = (uint32_t*)scratch;                          // aliases buf
    uint32_t* ctl = (uint32_t*)((char*)scratch + kWaveSortMaxKeys * 8);
    // The keys are the survivors of a first selection and sit in a narrow band of values:
    // digits taken from fixed bit positions would put most of them into one bin, pass after
    // pass (and a band that straddles a power of two shares no leading bits at all).  So the
    // band is measured first (greatest and least value present) and every pass cuts the
    // interval of keys that can still hold the K-th one into equal bins, 2048 at most: keys
    // are compared as 64-bit integers, value word first, so the bins are intervals of values
    // and, inside one value, of indices (ties resolve toward the lowest index).
    const int lane = tid & (kWave - 1);
    if (tid == 0) { ctl[20] = 0u; ctl[21] = 0xffffffffu; }
    __syncthreads();
    uint32_t vhi = 0u, vlo = 0xffffffffu;
    for_each_lds_key(keys, n, [&](uint64_t key) {
        if (key != 0) {
            const uint32_t v = (uint32_t)(key >> 32);
            vhi = max(vhi, v);
            vlo = min(vlo, v);
        }
    });
    for (int o = kWave / 2; o >= 1; o >>= 1) {
        vhi = max(vhi, (uint32_t)__shfl_xor((int)vhi, o, kWave));
        vlo = min(vlo, (uint32_t)__shfl_xor((int)vlo, o, kWave));
    }
    if (lane == 0) { atomicMax(&ctl[20], vhi); atomicMin(&ctl[21], vlo); }
    __syncthreads();
    vhi = ctl[20]; vlo = ctl[21];
    // every real key lies in [klo, khi] (a real key is never 0: its low word is ~index)
    uint64_t klo = ((uint64_t)vlo << 32) | 1ull, khi = ((uint64_t)vhi << 32) | 0xffffffffull;
    int need = K, certain = 0;
    bool fits = false;
    for (int pass = 0; !fits; ++pass) {
        const uint64_t span = khi - klo;
        const int span_bits = span ? 64 - __clzll((long long)span) : 0;
        const int shift = span_bits > kSelectBinBits ? span_bits - kSelectBinBits : 0;
        uint32_t digit, above, count;
        lds_select_bin(keys, n, klo, khi, shift, need, hist, ctl, digit, above, count);
        certain += (int)above;
        need -= (int)above;
        klo += (uint64_t)digit << shift;
        const uint64_t bin_span = (1ull << shift) - 1ull;          // (klo + bin_span may wrap)
        if (khi - klo > bin_span) khi = klo + bin_span;
        // stop when members + candidates fit one sort; prefer a sort of at most 2K keys.
        // With shift == 0 a bin is one key, so the loop ends there at the latest.
        fits = certain + (int)count <= cap &&
               (certain + (int)count <= 2 * K + 64 || pass >= 2 || shift == 0);
        if (!fits && (int)count <= kSideSortKeys) {
            // The bin that holds the K-th key is small: rather than cut it again, sort its
            // keys in one wavefront and read the K-th key off; what remains is "every key
            // at or above it", exactly K of them.
            if (tid == 0) ctl[3] = 0;
            __syncthreads();
            for_each_lds_key(keys, n, [&](uint64_t key) {
                if (key >= klo && key <= khi) {
                    const uint32_t slot = atomicAdd(&ctl[3], 1u);
                    if (slot < (uint32_t)kSideSortKeys) buf[slot] = key;
                }
            });
            __syncthreads();
            if (tid < kWave) {
                constexpr int RS = kSideSortKeys / kWave;
                uint64_t k[RS];
#pragma unroll
                for (int j = 0; j < RS; ++j) {
                    const int i = j * kWave + lane;
                    k[j] = i < (int)count ? buf[i] : 0;
                }
                if (count <= (uint32_t)kWave) {      // usually: a handful of keys
                    uint64_t one[1] = {k[0]};
                    WaveSort<1>::sort(one);
                    buf[lane] = one[0];
                } else {
                    WaveSort<RS>::sort(k);
#pragma unroll
                    for (int j = 0; j < RS; ++j) buf[lane * RS + j] = k[j];
                }
            }
            __syncthreads();
            klo = buf[need - 1];
            fits = true;
            __syncthreads();          // buf is filled again by the caller
        }
        if (shift == 0 && !fits) return 0;           // cannot happen (see above); ends the loop
    }
    return klo;
}

// Top-K (descending) of the n keys in LDS `keys` (n a power of two, key 0 = empty, at least K
// real keys), written decoded to out_*[out_base + 0..K).  Called by every thread of the
// workgroup; `scratch` is kSelectScratchBytes of LDS (unused when n <= 256): a buffer of
// kWaveSortMaxKeys keys, which the histogram aliases, then 32 control words.
// The keys array is used as working storage.
template <typename DT>
__device__ __forceinline__ void wg_topk_from_lds(uint64_t* keys, int n, int K, void* scratch,
                                                 const void* rowp, void* out_vals,
                                                 int32_t* out_idx, int64_t out_base, uint32_t flip = 0) {
    const int tid = threadIdx.x, T = blockDim.x;
    // few keys, or most of them wanted: sort them all
    if (n <= 256 || (n <= kWaveSortMaxKeys && 4 * K > n)) {
        if (n > kWgSortMinKeys && T >= kWgSortMinThreads) {
            wg_sort_merge_topk(keys, n, K);
            wg_write_topk<DT>(keys, K, rowp, out_vals, out_idx, out_base, flip);
            return;
        }
        if (tid < kWave) wave_sort_dispatch<DT>(keys, n, K, rowp, out_vals, out_idx, out_base, flip);
        return;
    }
    // twice that many keys with an eighth or more of them wanted: sorting them all (four runs,
    // two merge levels) is still cheaper than the selection passes (measured; from 4096 keys on,
    // or for a smaller share, the selection wins)
    if (T >= kWgSortMinThreads && n == 2 * kWaveSortMaxKeys && 8 * K >= n) {
        wg_sort_merge_topk(keys, n, K);
        wg_write_topk<DT>(keys, K, rowp, out_vals, out_idx, out_base, flip);
        return;
    }
    if (K <= kWaveSortMaxKeys) {
        uint64_t* buf = (uint64_t*)scratch;
        uint32_t* ctl = (uint32_t*)((char*)scratch + kWaveSortMaxKeys * 8);
        const uint64_t klo = wg_select_threshold(keys, n, K, scratch);
        if (klo != 0) {
            if (tid == 0) ctl[3] = 0;
            __syncthreads();
            // certain members and candidates -> buf (the histogram is dead by now)
            for_each_lds_key(keys, n, [&](uint64_t key) {
                if (key >= klo) {
                    const uint32_t slot = atomicAdd(&ctl[3], 1u);
                    if (slot < (uint32_t)kWaveSortMaxKeys) buf[slot] = key;
                }
            });
            __syncthreads();
            const int total = min((int)ctl[3], kWaveSortMaxKeys);
            if (total > kWgSortMinKeys && T >= kWgSortMinThreads) {
                // many keys and many idle wavefronts: sort in LDS with all of them
                // whole runs of the ranking sort (128 or 256 keys, one per wavefront); a power of two
                // only where the merging sort takes over
                const int nwaves = T >> 6;
                int padded = (total + 127) & ~127;
                if (padded > 128 * nwaves) padded = (total + 255) & ~255;
                if (padded > 256 * nwaves) padded = next_pow2(total);
                for (int i = total + tid; i < padded; i += T) buf[i] = 0;
                __syncthreads();
                wg_sort_merge_topk(buf, padded, K);
                wg_write_topk<DT>(buf, K, rowp, out_vals, out_idx, out_base, flip);
                return;
            }
            if (tid < kWave) wave_sort_dispatch<DT>(buf, total, K, rowp, out_vals, out_idx, out_base, flip);
            return;
        }
    }
    // More wanted than a wavefront sorts, yet less than half of the keys: the keys at or above
    // a threshold (K to 2K + 64 of them, as many as all wavefronts order together at most) are
    // moved to the front of the array and ordered there by all wavefronts, instead of ordering
    // everything (16384 keys, K = 2048: 204 -> 80 us a row).
    const int order_cap = min(n / 2, 512 * (T >> 6));
    if (K > kWaveSortMaxKeys && K <= order_cap && T >= kWgSortMinThreads) {
        uint32_t* ctl = (uint32_t*)((char*)scratch + kWaveSortMaxKeys * 8);
        const uint64_t klo = wg_select_threshold(keys, n, K, scratch, order_cap);
        if (klo != 0) {
            if (tid == 0) ctl[3] = 0;
            __syncthreads();
            // in place, four keys per thread and round: a round's keys are all in registers
            // before the first is written, and a key never moves behind where it was read
            lds_ptr<uint64_t> kl = (lds_ptr<uint64_t>)keys;
            for (int base = 0; base < n; base += 4 * T) {
                uint64_t k[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) k[u] = base + u * T + tid < n ? kl[base + u * T + tid] : 0;
                __syncthreads();
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (k[u] >= klo && k[u] != 0) kl[atomicAdd(&ctl[3], 1u)] = k[u];
                __syncthreads();
            }
            const int total = (int)ctl[3];
            const int nwaves = T >> 6;
            int padded = (total + 127) & ~127;
            if (padded > 128 * nwaves) padded = (total + 255) & ~255;
            if (padded > 256 * nwaves) padded = next_pow2(total);
            for (int i = total + tid; i < padded; i += T) kl[i] = 0;
            __syncthreads();
            wg_sort_merge_topk(keys, padded, K);
            wg_write_topk<DT>(keys, K, rowp, out_vals, out_idx, out_base, flip);
            return;
        }
    }
    // fallback: order everything
    lds_bitonic_sort_desc(keys, n, n);
    wg_write_topk<DT>(keys, K, rowp, out_vals, out_idx, out_base, flip);
}

}  // namespace atk
