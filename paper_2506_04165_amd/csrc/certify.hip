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

template <typename DT>
__global__ void __launch_bounds__(kCertifyThreads) certify_kernel(CertifyParams p) {
    extern __shared__ uint64_t lds64[];
    // layout: key buffer [cap], selection scratch, counters [B], flagged buckets, control words
    uint64_t* buf = lds64;
    void* scratch = lds64 + p.cap;
    uint32_t* hist = (uint32_t*)((char*)scratch + kSelectScratchBytes);
    int* flagged = (int*)(hist + p.B);
    uint32_t* ctl = (uint32_t*)(flagged + kCertifyMaxFlagged);      // 0: flagged buckets  1: keys in buf
    const int tid = threadIdx.x, T = blockDim.x;
    const int row = blockIdx.x;
    const int K = p.K, B = p.B;
    const int64_t out_base = (int64_t)row * K;
    const int per_bucket = p.N / B;

    if (tid == 0) p.hard_rows[row] = 0;
    if (per_bucket <= p.Kprime) return;          // every bucket was kept whole: nothing can be missing
    // the result's indices are asked for first (K <= 1024: at most four per thread), the counters
    // are cleared while they travel
    constexpr int kPerThread = kWaveSortMaxKeys / kCertifyThreads;
    uint32_t mine[kPerThread];
#pragma unroll
    for (int u = 0; u < kPerThread; ++u) {
        const int i = tid + u * T;
        mine[u] = i < K ? (uint32_t)p.out_idx[out_base + i] : 0xffffffffu;
    }
    for (int b = tid; b < B; b += T) hist[b] = 0;
    if (tid == 0) { ctl[0] = 0; ctl[1] = 0; }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kPerThread; ++u)
        if (mine[u] != 0xffffffffu) atomicAdd(&hist[mine[u] % (uint32_t)B], 1u);
    __syncthreads();
    for (int b = tid; b < B; b += T)
        if (hist[b] >= (uint32_t)p.Kprime) {
            const uint32_t slot = atomicAdd(&ctl[0], 1u);
            if (slot < (uint32_t)kCertifyMaxFlagged) flagged[slot] = b;
        }
    __syncthreads();
    const int nf = (int)ctl[0];
    if (nf == 0) return;                         // certified

    // ---- repair ---------------------------------------------------------------------------------
    if (nf > kCertifyMaxFlagged || (int64_t)nf * per_bucket > p.max_scan) {
        if (tid == 0) p.hard_rows[row] = 1;
        return;
    }
    const char* rowp = (const char*)p.values + (size_t)row * p.row_stride * elem<DT>::size;
    const uint64_t t_key = make_key<DT>(elem<DT>::load_bits(p.out_vals, out_base + K - 1) ^ p.flip,
                                        (uint32_t)p.out_idx[out_base + K - 1]);
    // the result's elements of unflagged buckets ...
    for (int i = tid; i < K; i += T) {
        const uint32_t idx = (uint32_t)p.out_idx[out_base + i];
        if (hist[idx % (uint32_t)B] < (uint32_t)p.Kprime) {
            const uint32_t slot = atomicAdd(&ctl[1], 1u);       // (fewer than K <= cap / 2 of them)
            buf[slot] = make_key<DT>(elem<DT>::load_bits(p.out_vals, out_base + i) ^ p.flip, idx);
        }
    }
    // ... and every element of a flagged bucket at or above t (the result's own among them)
    const int total = nf * per_bucket;
    for (int e = tid; e < total; e += T) {
        const int f = e / per_bucket, j = e - f * per_bucket;
        const uint32_t n = (uint32_t)j * (uint32_t)B + (uint32_t)flagged[f];
        const uint64_t key = make_key<DT>(elem<DT>::load_bits(rowp, n) ^ p.flip, n);
        if (key >= t_key) {
            const uint32_t slot = atomicAdd(&ctl[1], 1u);
            if (slot < (uint32_t)p.cap) buf[slot] = key;
        }
    }
    __syncthreads();
    const int fill = (int)ctl[1];
    if (fill > p.cap) {                          // more than the buffer takes: the output is untouched
        if (tid == 0) p.hard_rows[row] = 1;
        return;
    }
    const int n2 = next_pow2(fill);              // fill >= K: the result's K elements are all in the union
    for (int i = fill + tid; i < n2; i += T) buf[i] = 0;
    __syncthreads();
    wg_topk_from_lds<DT>(buf, n2, K, scratch, rowp, p.out_vals, p.out_idx, out_base, p.flip);
}

template <typename DT>
hipError_t launch_for(const CertifyParams& p, hipStream_t stream) {
    const size_t lds = certify_lds_bytes(p);
    allow_large_lds((const void*)certify_kernel<DT>, lds);
    hipLaunchKernelGGL(certify_kernel<DT>, dim3(p.rows), dim3(kCertifyThreads), lds, stream, p);
    return hipGetLastError();
}

}  // namespace

size_t certify_lds_bytes(const CertifyParams& p) {
    return (size_t)p.cap * 8 + kSelectScratchBytes + (size_t)p.B * 4 + kCertifyMaxFlagged * 4 + 16 * 4;
}

hipError_t launch_certify(const CertifyParams& p, int dtype, hipStream_t stream) {
    if (p.B > kCertifyMaxB || p.K > kWaveSortMaxKeys || p.cap < 2 * p.K || (p.cap & (p.cap - 1)) || p.N % p.B)
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
