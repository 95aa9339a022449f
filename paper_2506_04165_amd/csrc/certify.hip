// Exact Top-K out of the two-stage approximate result, with a certificate.
//
// The two-stage method (Section 6.1) loses an element of the true Top-K only in a bucket that
// holds more than K' of them (Section 6.2 counts exactly these collisions).  That event leaves a
// trace in the result: let t be the K-th key of the approximate result, a lower bound of the
// true K-th key because the survivors are a subset of the row.  An element x of the true Top-K
// that stage 1 dropped has K' kept elements of its bucket above it, all above t, so all K' of
// them are in the result.  Hence:
//   * a row in whose result no bucket appears K' times is exact as it stands (the certificate);
//   * otherwise the true Top-K lies in (result elements of the other buckets) + (elements of the
//     buckets that appear K' times whose key is >= t): those buckets are read again from the row
//     (N/B elements each), and the K greatest keys of that union are the exact result.
// For data in random order the expected number of such buckets per row is
// B * P[Binomial(K, 1/B) >= K'], a few hundredths at the settings the host picks, so nearly every
// row costs K counter updates in LDS and nothing else.  A row with more flagged buckets or more
// qualifying elements than the workgroup's buffer takes (adversarial placement, massive ties) is
// marked in hard_rows and left to the radix-selection kernel.
#include "atk_device.h"
#include "select_sort.h"
#include "certify.h"

namespace atk {

namespace {

constexpr int kCertifyThreads = 256;
constexpr int kCertifyWaves = kCertifyThreads / kWave;

struct CertifyLds {
    uint64_t* buf;        // [cap] the result's keys (sorted), then what a repair adds
    uint64_t* bmin;       // [kCertifyMaxFlagged + 1] least result key of every bucket in doubt; last: the K-th key
    uint32_t* hist;       // [B] result elements per bucket (of the row the workgroup works on)
    int* flagged;         // [kCertifyMaxFlagged] buckets with K' of them
    uint32_t* ctl;        // 0: keys added by the repair  4: buckets in doubt  8: rows to redo
};

// The workgroup checks, and if need be repairs, one row: hist/flagged/nf are the row's counters,
// the buckets in doubt and their number.  Every thread; ends with the row's exact result in place,
// or the row marked hard.  Nearly always nothing was dropped that matters, so the check comes
// first and is kept short: the elements of the buckets in doubt are asked for at once, beside the
// result's indices; only the result's elements of those buckets have their values read (the least
// of them bounds what the bucket can still contribute), and the result's keys are rebuilt in LDS
// only when something has to be merged into them.
template <typename DT>
__device__ void certify_repair(const CertifyParams& p, const CertifyLds& L, int row, uint32_t* hist,
                               const int* flagged, int nf) {
    const int tid = threadIdx.x, T = blockDim.x;
    const int K = p.K, B = p.B, per_bucket = p.N / B;
    const int64_t out_base = (int64_t)row * K;
    if (nf > kCertifyMaxFlagged || (int64_t)nf * per_bucket > p.max_scan) {
        if (tid == 0) p.hard_rows[row] = 1;
        return;
    }
    const char* rowp = (const char*)p.values + (size_t)row * p.row_stride * elem<DT>::size;
    const int total = nf * per_bucket;
    constexpr int kRegs = 4;                     // elements (and result indices: K <= 1024) per thread in registers
    auto element_of = [&](int e) -> uint32_t {   // position in the row of element e of the buckets in doubt
        const int f = e / per_bucket, j = e - f * per_bucket;
        return (uint32_t)j * (uint32_t)B + (uint32_t)flagged[f];
    };
    uint32_t ebits[kRegs], myidx[kRegs], myval[kRegs];
#pragma unroll
    for (int u = 0; u < kRegs; ++u) {
        const int e = tid + u * T;
        ebits[u] = elem<DT>::load_bits(rowp, element_of(min(e, total - 1)));      // (clamped, not branched: see below)
    }
#pragma unroll
    for (int u = 0; u < kRegs; ++u) {
        const int i = tid + u * T;
        // Loads at a clamped position with the result masked afterwards, never a load under a
        // test: the compiler ends every such test with a wait, one memory latency per load.
        const int ic = min(i, K - 1);
        myidx[u] = (uint32_t)p.out_idx[out_base + ic];
        myval[u] = elem<DT>::load_bits(p.out_vals, out_base + ic);   // (needed or not: no second wait)
        if (i >= K) myidx[u] = 0xffffffffu;
    }
    // the counters of the buckets in doubt now name their slot
    for (int f = tid; f < nf; f += T) {
        hist[flagged[f]] = 0x80000000u | (uint32_t)f;
        L.bmin[f] = ~0ull;
    }
    if (tid == 0) L.ctl[0] = 0;
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kRegs; ++u) {
        if (myidx[u] == 0xffffffffu) continue;
        const int i = tid + u * T;
        const uint32_t h = hist[myidx[u] % (uint32_t)B];
        if ((h & 0x80000000u) || i == K - 1) {
            const uint64_t key = make_key<DT>(myval[u] ^ p.flip, myidx[u]);
            if (h & 0x80000000u) atomicMin((unsigned long long*)&L.bmin[h & 0x7fffffffu], (unsigned long long)key);
            if (i == K - 1) L.bmin[kCertifyMaxFlagged] = key;   // the K-th key of the result
        }
    }
    __syncthreads();
    const uint64_t t_key = L.bmin[kCertifyMaxFlagged];
    // elements of the buckets in doubt that stage 1 dropped (below the bucket's K' kept ones) and
    // that beat the K-th key of the result: with them the union holds the true Top-K
    const int room = p.cap - K;                  // extras the buffer takes behind the result's keys
    uint64_t* ext = L.buf + K;
    {
        auto consider = [&](int e, uint32_t b) {
            const uint64_t key = make_key<DT>(b ^ p.flip, element_of(e));
            if (key > t_key && key < L.bmin[e / per_bucket]) {
                const uint32_t slot = atomicAdd(&L.ctl[0], 1u);
                if (slot < (uint32_t)room) ext[slot] = key;
            }
        };
#pragma unroll
        for (int u = 0; u < kRegs; ++u) {
            const int e = tid + u * T;
            if (e < total) consider(e, ebits[u]);
        }
        for (int e = tid + kRegs * T; e < total; e += T) consider(e, elem<DT>::load_bits(rowp, element_of(e)));
    }
    __syncthreads();
    const int extras = (int)L.ctl[0];
    if (extras == 0) return;                     // nothing was missing after all
    if (extras > room) {
        if (tid == 0) p.hard_rows[row] = 1;
        return;
    }
    // The result's keys to LDS: they are sorted, so nothing has to be sorted again.  Every key's
    // new rank is its old one plus the extras above it; an extra's rank is the number of result
    // keys above it (binary search) plus the extras above it.  Ranks below K are written; all
    // reads of the old result are done by then.
#pragma unroll
    for (int u = 0; u < kRegs; ++u)
        if (myidx[u] != 0xffffffffu) L.buf[tid + u * T] = make_key<DT>(myval[u] ^ p.flip, myidx[u]);
    __syncthreads();
    auto write = [&](int pos, uint64_t key) {
        const uint32_t idx = key_index(key);
        elem<DT>::store_bits(p.out_vals, out_base + pos, key_stored_bits<DT>(key, rowp, idx, p.flip));
        p.out_idx[out_base + pos] = (int32_t)idx;
    };
    for (int i = tid; i < K; i += T) {
        const uint64_t key = L.buf[i];
        int pos = i;
        for (int j = 0; j < extras; ++j) pos += ext[j] > key ? 1 : 0;
        if (pos < K && pos != i) write(pos, key);
    }
    for (int j = tid; j < extras; j += T) {
        const uint64_t key = ext[j];
        int lo = 0, hi = K;                      // number of result keys above key
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (L.buf[mid] > key) lo = mid + 1; else hi = mid;
        }
        int pos = lo;
        for (int q = 0; q < extras; ++q) pos += ext[q] > key ? 1 : 0;
        if (pos < K) write(pos, key);
    }
}

// One row by the whole workgroup: count, then check and repair.  Every thread.
template <typename DT>
__device__ void certify_row_wg(const CertifyParams& p, const CertifyLds& L, int row) {
    const int tid = threadIdx.x, T = blockDim.x;
    const int K = p.K, B = p.B;
    const int64_t out_base = (int64_t)row * K;
    // the result's indices are asked for first (K <= 1024: at most four per thread), the counters
    // are cleared while they travel
    constexpr int kPerThread = kWaveSortMaxKeys / kCertifyThreads;
    uint32_t mine[kPerThread];
#pragma unroll
    for (int u = 0; u < kPerThread; ++u) {
        const int i = tid + u * T;
        mine[u] = (uint32_t)p.out_idx[out_base + min(i, K - 1)];     // (clamped, masked below: no load under a test)
        if (i >= K) mine[u] = 0xffffffffu;
    }
    for (int b = tid; b < B; b += T) L.hist[b] = 0;
    if (tid == 0) L.ctl[4] = 0;
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kPerThread; ++u)
        if (mine[u] != 0xffffffffu) atomicAdd(&L.hist[mine[u] % (uint32_t)B], 1u);
    __syncthreads();
    for (int b = tid; b < B; b += T)
        if (L.hist[b] >= (uint32_t)p.Kprime) {
            const uint32_t slot = atomicAdd(&L.ctl[4], 1u);
            if (slot < (uint32_t)kCertifyMaxFlagged) L.flagged[slot] = b;
        }
    __syncthreads();
    const int nf = (int)L.ctl[4];                // (the same for every thread)
    if (nf > 0) certify_repair<DT>(p, L, row, L.hist, L.flagged, nf);
}

constexpr int kWaveCheckBuckets = 4;             // buckets in doubt a lone wavefront checks itself ...
constexpr int kWaveCheckRegs = 4;                // ... if they hold at most this many elements per lane

// One row by one wavefront, no barrier: count; if buckets are in doubt and few, check them (the
// result's least key per such bucket, the K-th key, the buckets' elements against both).
// Returns true when the row is certified, false when the workgroup has to look at it.
//   hist: B counters of this wavefront;  small: 2 * kWaveCheckBuckets + 2 words of 64 bits
template <typename DT>
__device__ bool certify_row_wave(const CertifyParams& p, int row, uint32_t* hist, uint64_t* small) {
    const int lane = threadIdx.x & (kWave - 1);
    const int K = p.K, B = p.B, per_bucket = p.N / B;
    const int64_t out_base = (int64_t)row * K;
    uint32_t* count = (uint32_t*)&small[kWaveCheckBuckets + 1];          // buckets in doubt
    int* flagged = (int*)&small[kWaveCheckBuckets + 2];                  // [2 * kWaveCheckBuckets]
    for (int b = lane; b < B; b += kWave) hist[b] = 0;
    if (lane == 0) *count = 0;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    // (the indices eight loads at a time: one memory latency per 512 of them, not per 64)
    for (int i0 = 0; i0 < K; i0 += 8 * kWave) {
        uint32_t idx[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = i0 + u * kWave + lane;
            idx[u] = (uint32_t)p.out_idx[out_base + min(i, K - 1)];  // (clamped, masked: no load under a test)
            if (i >= K) idx[u] = 0xffffffffu;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (idx[u] != 0xffffffffu) atomicAdd(&hist[idx[u] % (uint32_t)B], 1u);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    for (int b = lane; b < B; b += kWave)
        if (hist[b] >= (uint32_t)p.Kprime) {
            const uint32_t slot = atomicAdd(count, 1u);
            if (slot < (uint32_t)kWaveCheckBuckets) flagged[slot] = b;
        }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    const int nf = (int)*count;
    if (nf == 0) return true;
    const int total = nf * per_bucket;
    if (nf > kWaveCheckBuckets || total > kWaveCheckRegs * kWave) return false;
    // the elements of the buckets in doubt, all loads at once
    const char* rowp = (const char*)p.values + (size_t)row * p.row_stride * elem<DT>::size;
    uint32_t ebits[kWaveCheckRegs];
#pragma unroll
    for (int u = 0; u < kWaveCheckRegs; ++u) {
        const int e = min(lane + u * kWave, total - 1);       // (clamped: no load under a test)
        const int f = e / per_bucket, j = e - f * per_bucket;
        ebits[u] = elem<DT>::load_bits(rowp, (uint32_t)j * (uint32_t)B + (uint32_t)flagged[f]);
    }
    // ... and with them the result's indices and values (needed or not: a load behind a test, or
    // behind the fence below, would wait for memory a second time)
    auto fetch = [&](int i0, uint32_t (&idx)[8], uint32_t (&val)[8]) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = i0 + u * kWave + lane;
            const int ic = min(i, K - 1);                    // (clamped, masked: no load under a test)
            idx[u] = (uint32_t)p.out_idx[out_base + ic];
            val[u] = elem<DT>::load_bits(p.out_vals, out_base + ic);
            if (i >= K) idx[u] = 0xffffffffu;
        }
    };
    // least result key of every bucket in doubt, and the K-th key
    auto note = [&](int i0, const uint32_t (&idx)[8], const uint32_t (&val)[8]) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (idx[u] == 0xffffffffu) continue;
            const int i = i0 + u * kWave + lane;
            const uint32_t h = hist[idx[u] % (uint32_t)B];
            if ((h & 0x80000000u) || i == K - 1) {
                const uint64_t key = make_key<DT>(val[u] ^ p.flip, idx[u]);
                if (h & 0x80000000u) atomicMin((unsigned long long*)&small[h & 0x7fffffffu], (unsigned long long)key);
                if (i == K - 1) small[kWaveCheckBuckets] = key;
            }
        }
    };
    uint32_t idx0[8], val0[8];
    fetch(0, idx0, val0);
    if (lane < nf) {
        hist[flagged[lane]] = 0x80000000u | (uint32_t)lane;
        small[lane] = ~0ull;
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    note(0, idx0, val0);
    for (int i0 = 8 * kWave; i0 < K; i0 += 8 * kWave) {
        uint32_t idx[8], val[8];
        fetch(i0, idx, val);
        note(i0, idx, val);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    const uint64_t t_key = small[kWaveCheckBuckets];
    bool missing = false;
#pragma unroll
    for (int u = 0; u < kWaveCheckRegs; ++u) {
        const int e = lane + u * kWave;
        if (e < total) {
            const int f = e / per_bucket, j = e - f * per_bucket;
            const uint32_t n = (uint32_t)j * (uint32_t)B + (uint32_t)flagged[f];
            const uint64_t key = make_key<DT>(ebits[u] ^ p.flip, n);
            missing |= key > t_key && key < small[f];
        }
    }
    return __ballot(missing) == 0;
}

constexpr int kRowsPerWave = 1;                  // rows a wavefront takes in the many-rows form
static_assert(kCertifyWaves * kRowsPerWave == kCertifyRowsPerWg, "rows of a workgroup in the many-rows form");

template <typename DT>
__global__ void __launch_bounds__(kCertifyThreads, 8) certify_kernel(CertifyParams p) {
    extern __shared__ uint64_t lds64[];
    CertifyLds L;
    L.buf = lds64;
    L.bmin = L.buf + p.cap;
    L.hist = (uint32_t*)(L.bmin + kCertifyMaxFlagged + 1);
    L.flagged = (int*)(L.hist + p.B);
    L.ctl = (uint32_t*)(L.flagged + kCertifyMaxFlagged);               // 16 words, then 32 rows to redo
    const int tid = threadIdx.x;
    const int per_bucket = p.N / p.B;
    const int first_row = blockIdx.x * p.rows_per_wg;

    if (tid == 0)                                // (the thread that may set them again below)
        for (int r = 0; r < p.rows_per_wg; ++r)
            if (first_row + r < p.rows) p.hard_rows[first_row + r] = 0;
    if (per_bucket <= p.Kprime) return;          // every bucket was kept whole: nothing can be missing

    if (p.rows_per_wg == 1) {
        if (p.open_rows && p.open_rows[first_row] == 0) return;
        certify_row_wg<DT>(p, L, first_row);
        return;
    }
    // many short rows: every wavefront certifies kRowsPerWave rows by itself; what it cannot
    // settle (many buckets in doubt, or a dropped element that belongs into the result) the
    // workgroup takes afterwards
    uint32_t* todo = L.ctl + 16;
    uint64_t* wave_small = (uint64_t*)(((uintptr_t)(todo + kCertifyWaves * kRowsPerWave) + 7) & ~(uintptr_t)7);
    uint32_t* wave_hist = (uint32_t*)(wave_small + kCertifyWaves * (2 * kWaveCheckBuckets + 2));
    const int w = tid >> 6;
    if (tid == 0) L.ctl[8] = 0;
    __syncthreads();
    for (int q = 0; q < kRowsPerWave; ++q) {
        const int row = first_row + q * kCertifyWaves + w;
        if (row >= p.rows) break;
        if (p.open_rows && p.open_rows[row] == 0) continue;
        const bool ok = certify_row_wave<DT>(p, row, wave_hist + (size_t)w * p.B,
                                             wave_small + w * (2 * kWaveCheckBuckets + 2));
        if (!ok && (tid & (kWave - 1)) == 0) todo[atomicAdd(&L.ctl[8], 1u)] = (uint32_t)row;
    }
    __syncthreads();
    const int ntodo = (int)L.ctl[8];
    for (int t = 0; t < ntodo; ++t) {
        certify_row_wg<DT>(p, L, (int)todo[t]);
        __syncthreads();
    }
}

template <typename DT>
hipError_t launch_for(const CertifyParams& p, hipStream_t stream) {
    const size_t lds = certify_lds_bytes(p);
    allow_large_lds((const void*)certify_kernel<DT>, lds);
    const int grid = (p.rows + p.rows_per_wg - 1) / p.rows_per_wg;
    hipLaunchKernelGGL(certify_kernel<DT>, dim3(grid), dim3(kCertifyThreads), lds, stream, p);
    return hipGetLastError();
}

}  // namespace

size_t certify_lds_bytes(const CertifyParams& p) {
    size_t bytes = (size_t)p.cap * 8 + (kCertifyMaxFlagged + 1) * 8 +
                   (size_t)p.B * 4 + kCertifyMaxFlagged * 4 + 16 * 4;
    if (p.rows_per_wg > 1)      // rows to redo, the wavefronts' small arrays and counters
        bytes += kCertifyWaves * kRowsPerWave * 4 + 8 + kCertifyWaves * (2 * kWaveCheckBuckets + 2) * 8 +
                 (size_t)kCertifyWaves * p.B * 4;
    return bytes;
}

hipError_t launch_certify(const CertifyParams& p, int dtype, hipStream_t stream) {
    if (p.B > kCertifyMaxB || p.K > kWaveSortMaxKeys || p.cap < 2 * p.K || (p.cap & (p.cap - 1)) || p.N % p.B ||
        (p.rows_per_wg != 1 && p.rows_per_wg != kCertifyRowsPerWg))
        return hipErrorInvalidValue;
    switch (dtype) {
        case 0: return launch_for<float>(p, stream);
        case 1: return launch_for<bf16_t>(p, stream);
        case 3: return launch_for<i32_t>(p, stream);
        case 4: return launch_for<u32_t>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace atk
