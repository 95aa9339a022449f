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
__device__ __forceinline__ uint32_t key_index(uint64_t key) { return ~(uint32_t)key; }

// ---- element access ---------------------------------------------------------------------
template <typename DT> struct elem;
template <> struct elem<float> {
    static constexpr int size = 4;
    // a >= b as values (stored patterns; -0.0 equals +0.0), and the pattern of the least value
    // whose ordered image is at least `o` (images below that of -inf belong to no value)
    __device__ static bool ge(uint32_t a, uint32_t b) { return __uint_as_float(a) >= __uint_as_float(b); }
    __device__ static uint32_t floor_bits(uint32_t o) { return o < 0x00800000u ? 0xff800000u : bits_from_ordered(o); }
    // order-preserving image of the element's binary32 pattern, and back
    __device__ static uint32_t ordered(uint32_t bits) { return ordered_from_bits(bits); }
    __device__ static uint32_t from_ordered(uint32_t o) { return bits_from_ordered(o); }
    __device__ static uint32_t load_bits(const void* base, int64_t i) {
        return ((const uint32_t*)base)[i];
    }
    __device__ static void store_bits(void* base, int64_t i, uint32_t b) {
        ((uint32_t*)base)[i] = b;
    }
};
template <> struct elem<bf16_t> {
    static constexpr int size = 2;
    // a >= b as values (stored patterns; -0.0 equals +0.0), and the pattern of the least value
    // whose ordered image is at least `o` (images below that of -inf belong to no value)
    __device__ static bool ge(uint32_t a, uint32_t b) { return __uint_as_float(a) >= __uint_as_float(b); }
    __device__ static uint32_t floor_bits(uint32_t o) { return o < 0x00800000u ? 0xff800000u : bits_from_ordered(o); }
    // order-preserving image of the element's binary32 pattern, and back
    __device__ static uint32_t ordered(uint32_t bits) { return ordered_from_bits(bits); }
    __device__ static uint32_t from_ordered(uint32_t o) { return bits_from_ordered(o); }
    __device__ static uint32_t load_bits(const void* base, int64_t i) {
        return (uint32_t)((const uint16_t*)base)[i] << 16;
    }
    __device__ static void store_bits(void* base, int64_t i, uint32_t b) {
        ((uint16_t*)base)[i] = (uint16_t)(b >> 16);
    }
};

// binary32 scores that exist only inside keys (matmul-fused path): there is no stored array to
// re-read, and a score that compares equal to zero is +0.0.
struct score_t {};
template <> struct elem<score_t> {
    static constexpr int size = 4;
    // a >= b as values (stored patterns; -0.0 equals +0.0), and the pattern of the least value
    // whose ordered image is at least `o` (images below that of -inf belong to no value)
    __device__ static bool ge(uint32_t a, uint32_t b) { return __uint_as_float(a) >= __uint_as_float(b); }
    __device__ static uint32_t floor_bits(uint32_t o) { return o < 0x00800000u ? 0xff800000u : bits_from_ordered(o); }
    // order-preserving image of the element's binary32 pattern, and back
    __device__ static uint32_t ordered(uint32_t bits) { return ordered_from_bits(bits); }
    __device__ static uint32_t from_ordered(uint32_t o) { return bits_from_ordered(o); }
    __device__ static uint32_t load_bits(const void*, int64_t) { return 0; }
    __device__ static void store_bits(void* base, int64_t i, uint32_t b) {
        ((uint32_t*)base)[i] = b;
    }
};

// 32-bit integers (the compute types signed and unsigned inputs are promoted to in Section 6.3's
// listing).  "bits" is the stored word; the ordered image flips the sign bit of signed values.
// Every word is a legitimate value, so nothing in the value half marks "empty": keys stay
// distinct from 0 through their index half.
struct i32_t {};
struct u32_t {};
template <> struct elem<i32_t> {
    static constexpr int size = 4;
    __device__ static bool ge(uint32_t a, uint32_t b) { return (int32_t)a >= (int32_t)b; }
    __device__ static uint32_t floor_bits(uint32_t o) { return o ^ 0x80000000u; }
    __device__ static uint32_t ordered(uint32_t bits) { return bits ^ 0x80000000u; }
    __device__ static uint32_t from_ordered(uint32_t o) { return o ^ 0x80000000u; }
    __device__ static uint32_t load_bits(const void* base, int64_t i) { return ((const uint32_t*)base)[i]; }
    __device__ static void store_bits(void* base, int64_t i, uint32_t b) { ((uint32_t*)base)[i] = b; }
};
template <> struct elem<u32_t> {
    static constexpr int size = 4;
    __device__ static bool ge(uint32_t a, uint32_t b) { return a >= b; }
    __device__ static uint32_t floor_bits(uint32_t o) { return o; }
    __device__ static uint32_t ordered(uint32_t bits) { return bits; }
    __device__ static uint32_t from_ordered(uint32_t o) { return o; }
    __device__ static uint32_t load_bits(const void* base, int64_t i) { return ((const uint32_t*)base)[i]; }
    __device__ static void store_bits(void* base, int64_t i, uint32_t b) { ((uint32_t*)base)[i] = b; }
};

// key of an element: ordered image of its value in the high word, ~index in the low word
template <typename DT>
__device__ __forceinline__ uint64_t make_key(uint32_t value_bits, uint32_t index) {
    return ((uint64_t)elem<DT>::ordered(value_bits) << 32) | (uint32_t)(~index);
}
template <typename DT>
__device__ __forceinline__ uint32_t key_value_bits(uint64_t key) {
    return elem<DT>::from_ordered((uint32_t)(key >> 32));
}

// A load of V consecutive elements as one memory instruction (2, 4, 8 or 16 bytes).
template <int BYTES> struct vec_bytes;
template <> struct vec_bytes<2>  { using type = uint16_t; };
template <> struct vec_bytes<4>  { using type = uint32_t; };
template <> struct vec_bytes<8>  { using type = uint2; };
template <> struct vec_bytes<16> { using type = uint4; };

// Buffer addressing: a 128-bit resource descriptor in SGPRs names a uniform base address; a
// load adds a per-lane 32-bit byte offset (VGPR) and a uniform 32-bit byte offset (SGPR), so
// streaming a row costs no vector address arithmetic at all.
using buffer_rsrc = __amdgpu_buffer_rsrc_t;
__device__ __forceinline__ buffer_rsrc make_rsrc(const void* uniform_base) {
    // raw buffer (stride 0), 2^32-1 addressable bytes, 32-bit data format
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(uniform_base), 0, 0xffffffff, 0x00020000);
}
// Cache policy of the streaming loads: every input byte is read exactly once, so the loads
// are marked non-temporal (aux bit 1) and do not displace useful lines from the caches.
#ifndef ATK_LOAD_AUX
#define ATK_LOAD_AUX 2
#endif
template <int BYTES> struct buffer_load;
template <> struct buffer_load<2> {
    __device__ static uint16_t run(buffer_rsrc r, uint32_t voff, uint32_t soff) {
        return __builtin_amdgcn_raw_buffer_load_b16(r, voff, soff, ATK_LOAD_AUX);
    }
};
template <> struct buffer_load<4> {
    __device__ static uint32_t run(buffer_rsrc r, uint32_t voff, uint32_t soff) {
        return __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, ATK_LOAD_AUX);
    }
};
template <> struct buffer_load<8> {
    __device__ static uint2 run(buffer_rsrc r, uint32_t voff, uint32_t soff) {
        return __builtin_bit_cast(uint2, __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, ATK_LOAD_AUX));
    }
};
template <> struct buffer_load<16> {
    __device__ static uint4 run(buffer_rsrc r, uint32_t voff, uint32_t soff) {
        return __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, ATK_LOAD_AUX));
    }
};

template <typename DT, int V> struct vec_load {
    static constexpr int bytes = V * elem<DT>::size;
    using vec_t = typename vec_bytes<bytes>::type;
    __device__ static vec_t load(buffer_rsrc r, uint32_t lane_bytes, uint32_t uniform_bytes) {
        return buffer_load<bytes>::run(r, lane_bytes, uniform_bytes);
    }
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

// Host: kernels that ask for more than 64 KB of dynamic LDS have to say so first.  The grant
// holds per kernel and device, so it is asked for once and remembered (per calling thread).
inline void allow_large_lds(const void* kernel, size_t lds_bytes) {
    if (lds_bytes <= 64 * 1024) return;
    struct Granted { const void* kernel; int device; size_t bytes; };
    constexpr int kSlots = 64;
    static thread_local Granted table[kSlots];
    static thread_local int used = 0, victim = 0;
    int dev = 0;
    (void)hipGetDevice(&dev);
    int slot = -1;
    for (int i = 0; i < used; ++i)
        if (table[i].kernel == kernel && table[i].device == dev) {
            if (table[i].bytes >= lds_bytes) return;
            slot = i;
            break;
        }
    (void)hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (slot < 0) slot = used < kSlots ? used++ : (victim = (victim + 1) % kSlots);
    table[slot] = {kernel, dev, lds_bytes};
}

__device__ __forceinline__ int next_pow2(int x) {
    int p = 1;
    while (p < x) p <<= 1;
    return p;
}

}  // namespace atk
