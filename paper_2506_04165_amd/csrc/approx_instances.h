// The list of compiled (dtype, KP, V, R) variants of the fused kernel.
//   KP  list length held in registers (>= the requested K'; shorter requests use a prefix)
//   V   consecutive elements per load, R loads per step; V*R lists per lane
// Register budget: V*R*KP <= 32 list entries per lane.
#pragma once

// X(DTYPE_TAG, C++ type, KP, V, R, REP)   REP: 0 value+step lists, 1 packed 32-bit keys,
//                                          2 sorted batches of 64-bit keys, 3 insertion lists of
//                                          64-bit keys (integer inputs), 4 value+step lists
//                                          with deferred insertion, 5 packed keys in the lists and
//                                          64-bit keys from there on (16-bit rows of any length)
// DTYPE_TAG: 0 fp32, 1 bf16 (fp16 runs on the bf16 kernels), 3 int32, 4 uint32
#define ATK_INSTANCES_NL1(X, TAG, T, V, R, P) \
    X(TAG, T, 1, V, R, P) X(TAG, T, 2, V, R, P) X(TAG, T, 3, V, R, P) X(TAG, T, 4, V, R, P) \
    X(TAG, T, 6, V, R, P) X(TAG, T, 8, V, R, P) X(TAG, T, 16, V, R, P) X(TAG, T, 32, V, R, P)
#define ATK_INSTANCES_NL2(X, TAG, T, V, R, P) \
    X(TAG, T, 1, V, R, P) X(TAG, T, 2, V, R, P) X(TAG, T, 3, V, R, P) X(TAG, T, 4, V, R, P) \
    X(TAG, T, 6, V, R, P) X(TAG, T, 8, V, R, P) X(TAG, T, 16, V, R, P)
#define ATK_INSTANCES_NL4(X, TAG, T, V, R, P) \
    X(TAG, T, 1, V, R, P) X(TAG, T, 2, V, R, P) X(TAG, T, 3, V, R, P) X(TAG, T, 4, V, R, P) \
    X(TAG, T, 6, V, R, P) X(TAG, T, 8, V, R, P)
#define ATK_INSTANCES_NL8(X, TAG, T, V, R, P) \
    X(TAG, T, 1, V, R, P) X(TAG, T, 2, V, R, P) X(TAG, T, 3, V, R, P) X(TAG, T, 4, V, R, P)
#define ATK_INSTANCES_NL16(X, TAG, T, V, R, P) \
    X(TAG, T, 1, V, R, P) X(TAG, T, 2, V, R, P)

#define ATK_INSTANCES_F32_SMALL(X) \
    ATK_INSTANCES_NL1(X, 0, float, 1, 1, 0) ATK_INSTANCES_NL2(X, 0, float, 2, 1, 0)
#define ATK_INSTANCES_F32_WIDE(X) \
    ATK_INSTANCES_NL4(X, 0, float, 4, 1, 0) ATK_INSTANCES_NL8(X, 0, float, 4, 2, 0) \
    ATK_INSTANCES_NL16(X, 0, float, 4, 4, 0)
#define ATK_INSTANCES_BF16_SMALL(X) \
    ATK_INSTANCES_NL1(X, 1, bf16_t, 1, 1, 0) ATK_INSTANCES_NL2(X, 1, bf16_t, 2, 1, 0)
#define ATK_INSTANCES_BF16_WIDE(X) \
    ATK_INSTANCES_NL4(X, 1, bf16_t, 4, 1, 0) ATK_INSTANCES_NL8(X, 1, bf16_t, 8, 1, 0) \
    ATK_INSTANCES_NL16(X, 1, bf16_t, 8, 2, 0)

#define ATK_INSTANCES_I32_SMALL(X) \
    ATK_INSTANCES_NL1(X, 3, i32_t, 1, 1, 3) ATK_INSTANCES_NL2(X, 3, i32_t, 2, 1, 3)
#define ATK_INSTANCES_I32_WIDE(X) \
    ATK_INSTANCES_NL4(X, 3, i32_t, 4, 1, 3) ATK_INSTANCES_NL8(X, 3, i32_t, 4, 2, 3) \
    ATK_INSTANCES_NL16(X, 3, i32_t, 4, 4, 3)
#define ATK_INSTANCES_U32_SMALL(X) \
    ATK_INSTANCES_NL1(X, 4, u32_t, 1, 1, 3) ATK_INSTANCES_NL2(X, 4, u32_t, 2, 1, 3)
#define ATK_INSTANCES_U32_WIDE(X) \
    ATK_INSTANCES_NL4(X, 4, u32_t, 4, 1, 3) ATK_INSTANCES_NL8(X, 4, u32_t, 4, 2, 3) \
    ATK_INSTANCES_NL16(X, 4, u32_t, 4, 4, 3)

// single-element loads with several loads per step: for rows whose base address, stride or
// bucket count rule out vector loads
#define ATK_INSTANCES_F32_UNALIGNED(X) \
    ATK_INSTANCES_NL2(X, 0, float, 1, 2, 0) ATK_INSTANCES_NL4(X, 0, float, 1, 4, 0) \
    ATK_INSTANCES_NL8(X, 0, float, 1, 8, 0) ATK_INSTANCES_NL16(X, 0, float, 1, 16, 0)
#define ATK_INSTANCES_BF16_UNALIGNED(X) \
    ATK_INSTANCES_NL2(X, 1, bf16_t, 1, 2, 0) ATK_INSTANCES_NL4(X, 1, bf16_t, 1, 4, 0) \
    ATK_INSTANCES_NL8(X, 1, bf16_t, 1, 8, 0) ATK_INSTANCES_NL16(X, 1, bf16_t, 1, 16, 0)

#define ATK_INSTANCES_I32_UNALIGNED(X) \
    ATK_INSTANCES_NL2(X, 3, i32_t, 1, 2, 3) ATK_INSTANCES_NL4(X, 3, i32_t, 1, 4, 3) \
    ATK_INSTANCES_NL8(X, 3, i32_t, 1, 8, 3) ATK_INSTANCES_NL16(X, 3, i32_t, 1, 16, 3)
#define ATK_INSTANCES_U32_UNALIGNED(X) \
    ATK_INSTANCES_NL2(X, 4, u32_t, 1, 2, 3) ATK_INSTANCES_NL4(X, 4, u32_t, 1, 4, 3) \
    ATK_INSTANCES_NL8(X, 4, u32_t, 1, 8, 3) ATK_INSTANCES_NL16(X, 4, u32_t, 1, 16, 3)

// bf16 rows of at most 65536 elements: lists of packed 32-bit keys
#define ATK_PACKED_NL1(X, V, R) \
    X(1, bf16_t, 1, V, R, 1) X(1, bf16_t, 2, V, R, 1) X(1, bf16_t, 3, V, R, 1) X(1, bf16_t, 4, V, R, 1) \
    X(1, bf16_t, 6, V, R, 1) X(1, bf16_t, 8, V, R, 1) X(1, bf16_t, 16, V, R, 1) \
    X(1, bf16_t, 32, V, R, 1)
#define ATK_PACKED_NL2(X, V, R) \
    X(1, bf16_t, 1, V, R, 1) X(1, bf16_t, 2, V, R, 1) X(1, bf16_t, 3, V, R, 1) X(1, bf16_t, 4, V, R, 1) \
    X(1, bf16_t, 6, V, R, 1) X(1, bf16_t, 8, V, R, 1) X(1, bf16_t, 16, V, R, 1)
#define ATK_PACKED_NL4(X, V, R) \
    X(1, bf16_t, 1, V, R, 1) X(1, bf16_t, 2, V, R, 1) X(1, bf16_t, 3, V, R, 1) X(1, bf16_t, 4, V, R, 1) \
    X(1, bf16_t, 6, V, R, 1) X(1, bf16_t, 8, V, R, 1)
#define ATK_PACKED_NL8(X, V, R) \
    X(1, bf16_t, 1, V, R, 1) X(1, bf16_t, 2, V, R, 1) X(1, bf16_t, 3, V, R, 1) X(1, bf16_t, 4, V, R, 1)
#define ATK_PACKED_NL16(X, V, R) X(1, bf16_t, 1, V, R, 1) X(1, bf16_t, 2, V, R, 1)
#define ATK_INSTANCES_BF16_PACKED(X) \
    ATK_PACKED_NL1(X, 1, 1) ATK_PACKED_NL2(X, 2, 1) ATK_PACKED_NL4(X, 4, 1) \
    ATK_PACKED_NL8(X, 8, 1) ATK_PACKED_NL16(X, 8, 2)

// value+step lists with deferred insertion (REP 4), for long buckets: lists of 2 to 8 entries,
// aligned vector loads; lists of 16 entries with one or two lists per lane (with 32 entries the
// variant spills: 380 -> 1100 us)
#define ATK_DEFER_NL1(X, TAG, T, V, R) \
    X(TAG, T, 2, V, R, 4) X(TAG, T, 3, V, R, 4) X(TAG, T, 4, V, R, 4) X(TAG, T, 6, V, R, 4) X(TAG, T, 8, V, R, 4)
#define ATK_DEFER_NL8(X, TAG, T, V, R) X(TAG, T, 2, V, R, 4) X(TAG, T, 3, V, R, 4) X(TAG, T, 4, V, R, 4)
#define ATK_INSTANCES_F32_DEFER(X) \
    ATK_DEFER_NL1(X, 0, float, 1, 1) ATK_DEFER_NL1(X, 0, float, 2, 1) ATK_DEFER_NL1(X, 0, float, 4, 1) \
    ATK_DEFER_NL8(X, 0, float, 4, 2) X(0, float, 2, 4, 4, 4) \
    X(0, float, 16, 1, 1, 4) X(0, float, 16, 2, 1, 4)
#define ATK_INSTANCES_BF16_DEFER(X) \
    ATK_DEFER_NL1(X, 1, bf16_t, 1, 1) ATK_DEFER_NL1(X, 1, bf16_t, 2, 1) ATK_DEFER_NL1(X, 1, bf16_t, 4, 1) \
    ATK_DEFER_NL8(X, 1, bf16_t, 8, 1) X(1, bf16_t, 2, 8, 2, 4) \
    X(1, bf16_t, 16, 1, 1, 4) X(1, bf16_t, 16, 2, 1, 4)

// 16-bit rows of any length (at most 65535 steps): lists of packed 32-bit keys, 64-bit keys from
// the lists on (REP 5); lists of up to 8 entries, of 16 and 32 with one or two lists per lane
#define ATK_LONG16_NL(X, V, R) \
    X(1, bf16_t, 1, V, R, 5) X(1, bf16_t, 2, V, R, 5) X(1, bf16_t, 3, V, R, 5) X(1, bf16_t, 4, V, R, 5)
#define ATK_INSTANCES_BF16_LONG(X) \
    ATK_LONG16_NL(X, 1, 1) X(1, bf16_t, 6, 1, 1, 5) X(1, bf16_t, 8, 1, 1, 5) \
    ATK_LONG16_NL(X, 2, 1) X(1, bf16_t, 6, 2, 1, 5) X(1, bf16_t, 8, 2, 1, 5) \
    ATK_LONG16_NL(X, 4, 1) X(1, bf16_t, 6, 4, 1, 5) X(1, bf16_t, 8, 4, 1, 5) \
    ATK_LONG16_NL(X, 8, 1) X(1, bf16_t, 1, 8, 2, 5) X(1, bf16_t, 2, 8, 2, 5) \
    X(1, bf16_t, 16, 1, 1, 5) X(1, bf16_t, 32, 1, 1, 5) X(1, bf16_t, 16, 2, 1, 5)

// large K', at most 256 buckets: sorted batches of 64-bit keys, one list per lane
#define ATK_INSTANCES_BATCHED(X) \
    X(0, float, 8, 1, 1, 2) X(0, float, 16, 1, 1, 2) X(0, float, 32, 1, 1, 2) \
    X(1, bf16_t, 8, 1, 1, 2) X(1, bf16_t, 16, 1, 1, 2) X(1, bf16_t, 32, 1, 1, 2) \
    X(3, i32_t, 8, 1, 1, 2) X(3, i32_t, 16, 1, 1, 2) X(3, i32_t, 32, 1, 1, 2) \
    X(4, u32_t, 8, 1, 1, 2) X(4, u32_t, 16, 1, 1, 2) X(4, u32_t, 32, 1, 1, 2)

#define ATK_ALL_INSTANCES(X) \
    ATK_INSTANCES_F32_SMALL(X) ATK_INSTANCES_F32_WIDE(X) ATK_INSTANCES_F32_UNALIGNED(X) \
    ATK_INSTANCES_BF16_SMALL(X) ATK_INSTANCES_BF16_WIDE(X) ATK_INSTANCES_BF16_UNALIGNED(X) \
    ATK_INSTANCES_BF16_PACKED(X) ATK_INSTANCES_BATCHED(X) \
    ATK_INSTANCES_F32_DEFER(X) ATK_INSTANCES_BF16_DEFER(X) ATK_INSTANCES_BF16_LONG(X) \
    ATK_INSTANCES_I32_SMALL(X) ATK_INSTANCES_I32_WIDE(X) ATK_INSTANCES_I32_UNALIGNED(X) \
    ATK_INSTANCES_U32_SMALL(X) ATK_INSTANCES_U32_WIDE(X) ATK_INSTANCES_U32_UNALIGNED(X)
