// Device-side building blocks shared by the libatk kernels (gfx950, wave64).
//
// The total order used everywhere (value descending, equal values -> lower index first)
// is realised as an unsigned 64-bit key:  high word = order-preserving image of the
// binary32 value, low word = ~index.  Keys of distinct elements are distinct, a larger
// key means "comes first", and key 0 is reserved for "no element".
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace atk {

constexpr int kWave = 64;

struct bf16_t { uint16_t bits; };   // storage only; compared after widening to binary32

// ---- value <-> ordered word -------------------------------------------------------------
// Negative floats map to (0 - bits), non-negative ones to (bits | 2^31).  Both zeros land on
// 2^31, so -0.0 and +0.0 compare equal; -inf maps to 0x00800000, so 0 stays free as "empty".
__device__ __forceinline__ uint32_t ordered_from_bits(uint32_t b) {
    return (b >> 31) ? (0u - b) : (b | 0x80000000u);
}
__device__ __forceinline__ uint32_t bits_from_ordered(uint32_t o) {
    return (o >= 0x80000000u) ? (o - 0x80000000u) : (0u - o);   // a zero decodes as +0.0
}
__device__ __forceinline__ uint64_t make_key(uint32_t value_bits, uint32_t index) {
    return ((uint64_t)ordered_from_bits(value_bits) << 32) | (uint32_t)(~index);
}
__device__ __forceinline__ uint32_t key_index(uint64_t key) { return ~(uint32_t)key; }
__device__ __forceinline__ uint32_t key_value_bits(uint64_t key) {
    return bits_from_ordered((uint32_t)(key >> 32));
}

// ---- element access ---------------------------------------------------------------------
template <typename DT> struct elem;
template <> struct elem<float> {
    static constexpr int size = 4;
    __device__ static uint32_t load_bits(const void* base, int64_t i) {
        return ((const uint32_t*)base)[i];
    }
    __device__ static void store_bits(void* base, int64_t i, uint32_t b) {
        ((uint32_t*)base)[i] = b;
    }
};
template <> struct elem<bf16_t> {
    static constexpr int size = 2;
    __device__ static uint32_t load_bits(const void* base, int64_t i) {
        return (uint32_t)((const uint16_t*)base)[i] << 16;
    }
    __device__ static void store_bits(void* base, int64_t i, uint32_t b) {
        ((uint16_t*)base)[i] = (uint16_t)(b >> 16);
    }
};

// A load of V consecutive elements as one memory instruction (2, 4, 8 or 16 bytes).
template <int BYTES> struct vec_bytes;
template <> struct vec_bytes<2>  { using type = uint16_t; };
template <> struct vec_bytes<4>  { using type = uint32_t; };
template <> struct vec_bytes<8>  { using type = uint2; };
template <> struct vec_bytes<16> { using type = uint4; };

template <typename DT, int V> struct vec_load {
    using vec_t = typename vec_bytes<V * elem<DT>::size>::type;
    __device__ static vec_t load(const void* p) { return *(const vec_t*)p; }
    // binary32 bit pattern of element v of the vector
    __device__ static uint32_t bits(const vec_t& x, int v) {
        if constexpr (sizeof(vec_t) == 2) {
            return (uint32_t)x << 16;
        } else {
            const uint32_t* w = (const uint32_t*)&x;
            if constexpr (elem<DT>::size == 4) return w[v];
            else return (v & 1) ? (w[v >> 1] & 0xffff0000u) : (w[v >> 1] << 16);
        }
    }
};

// ---- LDS bitonic sort, descending, of `total` keys in segments of `seg` (powers of two,
// seg | total).  Called by every thread of the workgroup; ends with a barrier.
__device__ __forceinline__ void lds_bitonic_sort_desc(uint64_t* a, int total, int seg) {
    const int nthreads = blockDim.x;
    const int half = total >> 1;
    for (int k = 2; k <= seg; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = threadIdx.x; i < half; i += nthreads) {
                const int lo = ((i & ~(j - 1)) << 1) | (i & (j - 1));
                const int hi = lo | j;
                const bool desc = ((lo & (seg - 1)) & k) == 0;
                const uint64_t x = a[lo], y = a[hi];
                if ((x < y) == desc) { a[lo] = y; a[hi] = x; }
            }
            __syncthreads();
        }
    }
}

__device__ __forceinline__ int next_pow2(int x) {
    int p = 1;
    while (p < x) p <<= 1;
    return p;
}

}  // namespace atk
