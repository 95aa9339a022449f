// Fused two-stage approximate Top-K kernel (Section 6.1 Steps 1-4 in one launch).
//
// Work decomposition (ours; the paper's TPU kernel vectorises across buckets and walks the
// grid sequentially, neither of which carries over):
//   * a "group" of G lanes owns one row; a workgroup holds rows_per_wg groups;
//   * per step the group reads `S` consecutive elements of its row, lane t taking R loads of
//     V consecutive elements at offsets (r*G + t)*V; S is a multiple of B, so the bucket a
//     given register slot sees never changes and the K'-lists live in VGPRs with static
//     indexing (Section 6.3's "lists stay in registers" remark, without the state loads);
//   * S == B ("one owner"): every bucket belongs to exactly one slot of one lane, the lists
//     are final as they stand.  S == G*V == m*B ("m owners", small B): m lanes hold partial
//     lists of the same bucket; they are merged per bucket through LDS before stage 2;
//   * the update of one list with one element is Algorithm 1 restated for the fixed order:
//     compare the element with every entry (element on the left, so no dependency chain),
//     then each entry takes its upper neighbour, the element, or itself.  Elements arrive in
//     increasing index per slot, so a strict compare keeps the lower index on ties; empty
//     entries are NaN and the compare is written as !(x <= entry) so that anything, a real
//     -inf included, displaces them;
//   * survivors become 64-bit keys in LDS, a workgroup-wide bitonic sort orders each row's
//     B*K' candidates, and the first K are decoded and written out (stage 2).
//   * mode 1 writes the survivors in the [rows, K', B] layout of Section 6.3 instead.
#pragma once
#include "atk_device.h"
#include "select_sort.h"

namespace atk {

struct ApproxParams {
    const void* values;
    int64_t row_stride;   // elements
    int rows, N, K, Kprime, B;
    int G;                // lanes per row (power of two)
    int log2G;
    int rows_per_wg;
    int S;                // elements consumed per step by one group: max(B, G*V)
    int nsteps;           // N / S
    int owners;           // lanes*slots sharing a bucket: S / B
    int seg;              // owners > 1: power of two >= owners*KP, LDS keys per bucket
    int Cpad;             // power of two >= B*K', LDS keys per row for stage 2
    int aux_offset;       // LDS keys before the auxiliary region (partial lists / select scratch)
    int mode;             // 0: stage 2 fused, write out_*; 1: write survivors to surv_*;
                          // 2: this workgroup covers one segment of its row, write partial keys;
                          // 3: this workgroup covers slab_w buckets of its row over all steps
                          //    (owners lanes per bucket), write their final K' keys
                          // 4: like 1 (one owner per bucket, G >= 64), but the survivors of every
                          //    wavefront leave as one sorted run of run_len keys, part_keys being
                          //    [rows, gridDim.y * G / 64, run_len]
    int tail;             // mode 0, how stage 2 runs: 0 generic LDS sort of every row of the
                          // workgroup; 1 at most 1024 candidates per row, sorted in registers by
                          // the first wavefront of the row's group; 2 one row per workgroup,
                          // radix selection + wave sort
    int nseg;             // mode 2: segments per row (gridDim.y)
    int seg_steps;        // mode 2: steps per segment (the last one may be shorter)
    int slab_w;           // mode 3: buckets per workgroup, a power of two (gridDim.y = B / slab_w)
    int run_len;          // mode 3: > 0 (slab_w times a power of two >= K', at most 256; one row per
                          // workgroup): the workgroup's slab_w*K' final keys leave as one sorted,
                          // zero-padded run, part_keys being [rows, B / slab_w, run_len]
    int chunk;            // modes 0 and 1, one owner per bucket: > 0 cuts the row along the bucket
                          // axis, a workgroup taking buckets [blockIdx.y*chunk, +chunk) over all steps
                          // (gridDim.y = ceil(B / chunk)); 0: the whole row.  In mode 0 (chunk must
                          // divide B, one row per workgroup) stage 2 runs on the chunk's own
                          // survivors and the K greatest of them go to out_*[(row*gridDim.y +
                          // blockIdx.y)*K ...]: a row's result is among its chunks' results
    uint64_t* part_keys;  // mode 2: [rows, nseg, K', B] keys, 0 = empty entry; mode 3: [rows, K', B]
    void* out_vals;
    int32_t* out_idx;
    void* surv_vals;
    int32_t* surv_idx;
    int32_t* cert_flags;  // optional [rows] (packed-key variants only): 0 where no bucket contributes K' of the
                          // row's K results (the results are then the exact Top-K), 1 where one does or
                          // the question stays open; see certify.hip
    uint32_t flip;        // 0: the K greatest.  The K smallest (min-K): the mask that reverses the order
                          // of the element type, xor-ed onto every loaded pattern -- the sign bit of
                          // a floating type (0x80000000 on the widened pattern), all bits of an
                          // integer -- and again onto every pattern that is written out
    int surv_aligned;     // mode 1: both survivor arrays start at multiples of 16 bytes (vector stores allowed)
    int defer_from;       // value+step lists: the step from which elements may be set aside instead of
                          // inserted at once (variants with deferred insertion, see Lists<4>)
};

// Plain two-way select on values; written as a function of values so that it is emitted as a
// select (v_cndmask) and never as a divergent branch.
template <typename T>
__device__ __forceinline__ T sel(bool c, T a, T b) { return c ? a : b; }

// ---- per-lane K'-lists --------------------------------------------------------------------
// Two representations of the same thing (the K' greatest elements a register slot has seen,
// greatest first):
//
//  * value + step (any input): the list update is Algorithm 1 restated for the fixed order:
//    compare the element with every entry (element on the left, so no dependency chain), then
//    each entry takes its upper neighbour, the element, or itself; 5K'-2 lane operations.
//    Empty entries are NaN and the test is !(x <= entry), so anything displaces them.
//
//  * packed 32-bit key (bf16 rows of at most 65536 elements): ordered 16-bit value in the high
//    half, 0xFFFF - step in the low half.  Within one list keys are distinct and "greater key"
//    is exactly the total order, so the update is one max and K'-1 medians-of-three on integers
//    -- K' lane operations -- and no index needs tracking.  Key 0 is the empty entry.
template <int REP, int KP, int NL> struct Lists;

template <int KP, int NL>
struct Lists<0, KP, NL> {
    static constexpr bool exact_bits = false;    // a zero entry may carry the other zero's sign
    static constexpr bool holds_ordered = false; // bits() is the stored pattern itself
    float val[NL][KP];
    int32_t stp[NL][KP];
    __device__ __forceinline__ void init() {
        const float empty = __builtin_nanf("");
#pragma unroll
        for (int l = 0; l < NL; ++l)
#pragma unroll
            for (int k = 0; k < KP; ++k) { val[l][k] = empty; stp[l][k] = 0; }
    }
    __device__ __forceinline__ void insert(int l, float x, int32_t step) {
        bool c[KP];
#pragma unroll
        for (int k = 0; k < KP; ++k) c[k] = !(x <= val[l][k]);
#pragma unroll
        for (int k = KP - 1; k >= 1; --k) {
            const float v0 = sel(c[k], x, val[l][k]);
            const int32_t s0 = sel(c[k], step, stp[l][k]);
            val[l][k] = sel(c[k - 1], val[l][k - 1], v0);
            stp[l][k] = sel(c[k - 1], stp[l][k - 1], s0);
        }
        val[l][0] = sel(c[0], x, val[l][0]);
        stp[l][0] = sel(c[0], step, stp[l][0]);
    }
    // The same update once no entry is empty any more (K' elements have gone through the list):
    // the values need no compare-and-select, entry k becomes the median of (entry k-1, entry k,
    // element) -- the shift of Algorithm 1 as a clamp; only the steps follow the compares.
    // 4K'-1 lane operations.  The median may return either zero when +0.0 meets -0.0, which is
    // why a zero is re-read from the row when it is reported (exact_bits is false).
    __device__ __forceinline__ void insert_full(int l, float x, int32_t step) {
        bool c[KP];
#pragma unroll
        for (int k = 0; k < KP; ++k) c[k] = x > val[l][k];
#pragma unroll
        for (int k = KP - 1; k >= 1; --k) {
            stp[l][k] = sel(c[k - 1], stp[l][k - 1], sel(c[k], step, stp[l][k]));
            val[l][k] = __builtin_amdgcn_fmed3f(val[l][k - 1], val[l][k], x);
        }
        stp[l][0] = sel(c[0], step, stp[l][0]);
        val[l][0] = sel(c[0], x, val[l][0]);
    }
    __device__ __forceinline__ bool valid(int l, int k) const { return val[l][k] == val[l][k]; }
    __device__ __forceinline__ uint32_t bits(int l, int k) const { return __float_as_uint(val[l][k]); }
    // e: offset of the slot inside a step, S: elements per step
    __device__ __forceinline__ uint32_t index(int l, int k, uint32_t S, uint32_t e) const {
        return (uint32_t)stp[l][k] * S + e;
    }
};

//  * value + step with deferred insertion: the same lists, see below.
template <int KP, int NL>
struct Lists<4, KP, NL> : Lists<0, KP, NL> {
    using Lists<0, KP, NL>::val;
    using Lists<0, KP, NL>::insert_full;
    // Deferred insertion (full lists only).  Once a list has seen many elements, few of the
    // following ones beat its least entry.  Such an element is only set aside (one compare, two
    // selects); it enters the list when another element of the same list, in any lane of the
    // wavefront, wants the place where it waits -- a wavefront-uniform branch that is rarely
    // taken -- or at the end.  Elements wait at most one per list, and nothing overtakes a
    // waiting element inside its list, so the list ends up exactly as with immediate insertion.
    float pend_v[NL];
    int32_t pend_s[NL];          // < 0: nothing waits
    __device__ __forceinline__ void pend_init() {
#pragma unroll
        for (int l = 0; l < NL; ++l) { pend_v[l] = 0.0f; pend_s[l] = -1; }
    }
    __device__ __forceinline__ bool beats_least(int l, float x) const { return x > val[l][KP - 1]; }
    __device__ __forceinline__ void set_aside(int l, bool hit, float x, int32_t step) {
        pend_v[l] = sel(hit, x, pend_v[l]);
        pend_s[l] = sel(hit, step, pend_s[l]);
    }
    __device__ __forceinline__ void flush(int l) {
        // lanes where nothing waits insert -inf, which changes nothing
        insert_full(l, sel(pend_s[l] >= 0, pend_v[l], -__builtin_inff()), pend_s[l]);
        pend_s[l] = -1;
    }
};

template <int KP, int NL>
struct Lists<1, KP, NL> {
    static constexpr bool exact_bits = false;    // -0.0 is stored as +0.0
    static constexpr bool holds_ordered = false;
    uint32_t key[NL][KP];
    __device__ __forceinline__ void init() {
#pragma unroll
        for (int l = 0; l < NL; ++l)
#pragma unroll
            for (int k = 0; k < KP; ++k) key[l][k] = 0;
    }
    __device__ __forceinline__ void insert(int l, uint32_t x) {
#pragma unroll
        for (int k = KP - 1; k >= 1; --k)
            key[l][k] = med3_u32(key[l][k - 1], key[l][k], x);
        key[l][0] = max(key[l][0], x);
    }
    __device__ __forceinline__ bool valid(int l, int k) const { return key[l][k] != 0; }
    __device__ __forceinline__ uint32_t bits(int l, int k) const {
        return bits_from_ordered(key[l][k] & 0xffff0000u);
    }
    // the low half of a key is 0xFFFF - step; e: offset of the slot inside a step
    __device__ __forceinline__ uint32_t index(int l, int k, uint32_t S, uint32_t e) const {
        return (0xffffu - (key[l][k] & 0xffffu)) * S + e;
    }
};

//  * packed 32-bit keys in the lists, 64-bit keys from there on (16-bit rows of any length
//    with at most 65535 steps): stage 1 as above -- the step fits the low half whatever the
//    row's length -- and what leaves the lists is turned into the general (value, position)
//    keys, so every route and stage 2 of the value+step lists apply unchanged.
template <int KP, int NL>
struct Lists<5, KP, NL> : Lists<1, KP, NL> {};

//  * sorted batches of 64-bit keys (large K', one list per lane): K' consecutive elements of the
//    slot are turned into keys (ordered value << 32 | ~step), sorted in registers by a bitonic
//    network, and merged with the running list (element-wise max against the reversed batch
//    gives a bitonic sequence holding the K' greatest of both; log2 K' more stages order it).
//    About 11 compare-exchanges per element at K' = 32 instead of 32 list positions.
template <int KP>
__device__ __forceinline__ void reg_cex_desc(uint64_t& a, uint64_t& b) {   // a := greater
    const bool sw = a < b;
    const uint64_t hi = sw ? b : a, lo = sw ? a : b;
    a = hi; b = lo;
}
template <int KP>
__device__ __forceinline__ void reg_bitonic_merge_desc(uint64_t (&a)[KP]) {   // a bitonic -> descending
#pragma unroll
    for (int j = KP / 2; j >= 1; j >>= 1)
#pragma unroll
        for (int i = 0; i < KP; ++i)
            if ((i & j) == 0) reg_cex_desc<KP>(a[i], a[i | j]);
}
template <int KP>
__device__ __forceinline__ void reg_bitonic_sort_desc(uint64_t (&a)[KP]) {
#pragma unroll
    for (int k = 2; k <= KP; k <<= 1)
#pragma unroll
        for (int j = k / 2; j >= 1; j >>= 1)
#pragma unroll
            for (int i = 0; i < KP; ++i)
                if ((i & j) == 0) {
                    if ((i & k) == 0 || k == KP) reg_cex_desc<KP>(a[i], a[i | j]);
                    else reg_cex_desc<KP>(a[i | j], a[i]);
                }
}

template <int KP, int NL>
struct Lists<2, KP, NL> {
    static_assert(NL == 1, "sorted batches keep one list per lane");
    static constexpr bool exact_bits = false;    // -0.0 is stored as +0.0
    static constexpr bool holds_ordered = true;
    uint64_t key[KP];                            // descending, 0 = empty
    __device__ __forceinline__ void init() {
#pragma unroll
        for (int k = 0; k < KP; ++k) key[k] = 0;
    }
    // batch: KP keys in any order (0 = none); afterwards key[] holds the KP greatest of both
    __device__ __forceinline__ void merge(uint64_t (&batch)[KP]) {
        reg_bitonic_sort_desc<KP>(batch);
#pragma unroll
        for (int k = 0; k < KP; ++k) key[k] = max(key[k], batch[KP - 1 - k]);
        reg_bitonic_merge_desc<KP>(key);
    }
    __device__ __forceinline__ bool valid(int, int k) const { return key[k] != 0; }
    // ordered image of the value (holds_ordered): the kernel maps it back for its element type
    __device__ __forceinline__ uint32_t bits(int, int k) const { return (uint32_t)(key[k] >> 32); }
    // the low word of a key is ~step; e: offset of the slot inside a step
    __device__ __forceinline__ uint32_t index(int, int k, uint32_t S, uint32_t e) const {
        return (~(uint32_t)key[k]) * S + e;
    }
};

//  * 64-bit keys with insertion (integer inputs): an entry is (ordered value << 32 | ~step), so
//    "greater key" is the total order inside a list and an entry is never 0; the update is
//    Algorithm 1 on keys: K' 64-bit compares, then every entry takes its upper neighbour, the
//    new key or itself.  Float inputs do not use it: their value+step lists compare in one
//    32-bit instruction.
template <int KP, int NL>
struct Lists<3, KP, NL> {
    static constexpr bool exact_bits = true;
    static constexpr bool holds_ordered = true;
    uint64_t key[NL][KP];                        // descending, 0 = empty
    __device__ __forceinline__ void init() {
#pragma unroll
        for (int l = 0; l < NL; ++l)
#pragma unroll
            for (int k = 0; k < KP; ++k) key[l][k] = 0;
    }
    __device__ __forceinline__ void insert(int l, uint32_t ordered, int32_t step) {
        const uint64_t x = ((uint64_t)ordered << 32) | (uint32_t)(~(uint32_t)step);
        bool c[KP];
#pragma unroll
        for (int k = 0; k < KP; ++k) c[k] = x > key[l][k];
#pragma unroll
        for (int k = KP - 1; k >= 1; --k)
            key[l][k] = sel(c[k - 1], key[l][k - 1], sel(c[k], x, key[l][k]));
        key[l][0] = sel(c[0], x, key[l][0]);
    }
    __device__ __forceinline__ bool valid(int l, int k) const { return key[l][k] != 0; }
    __device__ __forceinline__ uint32_t bits(int l, int k) const { return (uint32_t)(key[l][k] >> 32); }
    __device__ __forceinline__ uint32_t index(int l, int k, uint32_t S, uint32_t e) const {
        return (~(uint32_t)key[l][k]) * S + e;
    }
};

template <typename DT, int KP, int V, int R, int REP = 0>
struct ApproxKernel {
    static constexpr bool PACKED = REP == 1;             // packed lists and the 32-bit stage 2
    static constexpr bool PACKED_LISTS = REP == 1 || REP == 5;
    static constexpr bool BATCHED = REP == 2;
    static constexpr int NL = V * R;
    static constexpr int DW = (V * elem<DT>::size + 3) / 4;           // dwords per load
    static constexpr int U_ = 32 / (R * DW);                          // 32 dwords of loads in flight,
    static constexpr int U = U_ < 1 ? 1 : (U_ > 16 ? 16 : U_);        // at most 16 steps
    using VL = vec_load<DT, V>;
    using vec_t = typename VL::vec_t;
    static_assert(!PACKED_LISTS || elem<DT>::size == 2, "packed keys are for 16-bit inputs");

    // Stored bit pattern of a list entry (lists of keys hold the ordered image instead).
    __device__ static __forceinline__ uint32_t stored_bits(const Lists<REP, KP, NL>& L, int l, int k) {
        if constexpr (Lists<REP, KP, NL>::holds_ordered) return elem<DT>::from_ordered(L.bits(l, k));
        else return L.bits(l, k);
    }

    // Feed the V elements of one load into their lists.
    // FULL: every list has already taken K' elements (value+step lists then use the shorter
    // update).
    template <bool FULL = false>
    __device__ static __forceinline__ void consume(Lists<REP, KP, NL>& L, const vec_t& x, int r,
                                                   int step, uint32_t flip) {
        if constexpr (BATCHED) {
            (void)L; (void)x; (void)r; (void)step;       // batches are fed by the streaming loop
        } else if constexpr (REP == 3) {
#pragma unroll
            for (int v = 0; v < V; ++v)
                L.insert(r * V + v, elem<DT>::ordered(VL::bits(x, v) ^ flip), step);
        } else if constexpr (!PACKED_LISTS) {
#pragma unroll
            for (int v = 0; v < V; ++v) {
                if constexpr (FULL && KP > 1) L.insert_full(r * V + v, __uint_as_float(VL::bits(x, v) ^ flip), step);
                else L.insert(r * V + v, __uint_as_float(VL::bits(x, v) ^ flip), step);
            }
        } else {
            // Low half of every key of this step: 0xFFFF - step.  All elements of one list share
            // the slot, so the step alone orders them; the position is rebuilt from it later.
            uint32_t low;
            asm("v_mov_b32 %0, %1" : "=v"(low) : "s"(0xffffu - (uint32_t)step));
            if constexpr (sizeof(vec_t) == 2) {
                L.insert(r * V, ordered_from_bits(((uint32_t)x << 16) ^ flip) | low);
            } else {
                typedef short short2_t __attribute__((ext_vector_type(2)));
                typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));
#pragma unroll
                for (int d = 0; d < V / 2; ++d) {
                    // two bf16 per dword: ordered 16-bit images of both with packed 16-bit ops
                    // (sign fill, flip, and +1 on negatives so that -0.0 lands on +0.0's image)
                    const uint32_t w = ((const uint32_t*)&x)[d] ^ (flip | (flip >> 16));   // both halves
                    const uint32_t sg = __builtin_bit_cast(uint32_t, __builtin_bit_cast(short2_t, w) >> (short)15);
                    const uint32_t fl = w ^ (sg | 0x80008000u);
                    const uint32_t o = __builtin_bit_cast(
                        uint32_t, __builtin_bit_cast(ushort2_t, fl) - __builtin_bit_cast(ushort2_t, sg));
                    L.insert(r * V + 2 * d, (o << 16) | low);
                    L.insert(r * V + 2 * d + 1, (o & 0xffff0000u) | low);
                }
            }
        }
    }

    // MINK: the mirrored problem; every loaded pattern passes through the order-reversing xor
    // (the Top-K instantiation carries no trace of it).
    template <bool MINK>
    __device__ static void run(const ApproxParams& p, uint64_t* lds) {
        const uint32_t flip = MINK ? p.flip : 0u;
        const int tid = threadIdx.x;
        const int g = tid >> p.log2G;
        const int t = tid & (p.G - 1);
        const int row = blockIdx.x * p.rows_per_wg + g;
        const bool row_ok = row < p.rows;
        const char* rowp = (const char*)p.values +
                           (size_t)(row_ok ? row : 0) * p.row_stride * elem<DT>::size;

        Lists<REP, KP, NL> L;
        L.init();

        int off[R];
        bool slot_ok[R];
        const int chunk_first = p.chunk > 0 ? (int)blockIdx.y * p.chunk : 0;
        const int chunk_len = p.chunk > 0 ? min(p.chunk, p.S - chunk_first) : p.S;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int o = (r * p.G + t) * V;
            slot_ok[r] = o < chunk_len;
            off[r] = slot_ok[r] ? chunk_first + o : 0;    // idle slots re-read offset 0; their lists are dropped
        }
        if (p.mode == 3) {
            // a slab of buckets: lane t is owner t / slab_w of bucket first + t % slab_w, and a
            // step spans `owners` consecutive bucket rounds of the row
            off[0] = (t / p.slab_w) * p.B + (int)blockIdx.y * p.slab_w + (t & (p.slab_w - 1));
        }

        // ---- stage 1: stream the row (or this workgroup's segment of it) once ------------------
        // A load address is (uniform base of the step, in a buffer descriptor) + (per-lane
        // 32-bit byte offset), so streaming needs no vector address arithmetic.  U steps are
        // loaded back to back and then consumed in order; other waves cover the wait.
        constexpr int ES = elem<DT>::size;
        const char* wg_base = (const char*)p.values +
                              (size_t)blockIdx.x * p.rows_per_wg * p.row_stride * ES;
        const uint32_t step_bytes = (uint32_t)p.S * ES;
        uint32_t lane_off[R];
#pragma unroll
        for (int r = 0; r < R; ++r)
            lane_off[r] = (uint32_t)(((size_t)(row_ok ? g : 0) * p.row_stride + off[r]) * ES);

        // Wavefronts that stream outrank those that sort: a streaming wavefront needs few issue
        // slots to turn its loads around, and every slot it waits for behind another wavefront's
        // sorting network is memory bandwidth not asked for (measured on many short rows: 4-8 %).
        // The sorted-batch lists sort while they stream and gain nothing from it.
        if constexpr (!BATCHED) __builtin_amdgcn_s_setprio(1);
        int s = 0, s_end = p.nsteps;
        if (p.mode == 2) {
            s = blockIdx.y * p.seg_steps;
            s_end = min(p.nsteps, s + p.seg_steps);
        }
        if constexpr (BATCHED) {
            // K' steps at a time: load them, turn them into keys, sort-merge into the list
            static_assert(V == 1 && R == 1, "sorted batches: one list per lane");
            for (; s < s_end; s += KP) {
                const buffer_rsrc rs = make_rsrc(wg_base + (size_t)s * step_bytes);
                const int nb = min(KP, s_end - s);          // uniform: the last batch may be short
                vec_t buf[KP];
#pragma unroll
                for (int u = 0; u < KP; ++u)
                    buf[u] = VL::load(rs, lane_off[0], (uint32_t)(u < nb ? u : 0) * step_bytes);
                uint64_t batch[KP];
#pragma unroll
                for (int u = 0; u < KP; ++u) {
                    const uint64_t key = ((uint64_t)elem<DT>::ordered(VL::bits(buf[u], 0) ^ flip) << 32) |
                                         (uint32_t)(~(uint32_t)(s + u));
                    batch[u] = u < nb ? key : 0;
                }
                L.merge(batch);
            }
        } else {
        // every slot takes one element per step: after KP steps no list entry is empty
        constexpr bool TWO_PHASE = (REP == 0 || REP == 4) && KP > 1;
        if constexpr (TWO_PHASE) {
            // the first KP steps (fewer on a short walk), loaded together like any other batch
            const int nfill = min(KP, s_end - s);                  // uniform
            if (nfill > 0) {
                const buffer_rsrc rs = make_rsrc(wg_base + (size_t)s * step_bytes);
                vec_t buf[KP][R] = {};
#pragma unroll
                for (int u = 0; u < KP; ++u)
                    if (u < nfill) {
#pragma unroll
                        for (int r = 0; r < R; ++r)
                            buf[u][r] = VL::load(rs, lane_off[r], (uint32_t)u * step_bytes);
                    }
#pragma unroll
                for (int u = 0; u < KP; ++u)
                    if (u < nfill) {
#pragma unroll
                        for (int r = 0; r < R; ++r) consume<false>(L, buf[u][r], r, s + u, flip);
                    }
                s += nfill;
            }
        }
        // The variants with deferred insertion set elements aside instead of inserting them
        // (see Lists<4>) while that pays: a batch of U steps runs in that form, and when more
        // than a quarter of its list updates had to insert after all (ascending data: every
        // element beats its list) the following batches insert at once, 1, 2, 4, ... of them
        // before the next attempt.
        constexpr bool DEFER = REP == 4;
        static_assert(!DEFER || KP > 1, "deferred insertion is for lists of two entries or more");
        uint64_t waiting[NL] = {};          // per list: the lanes where an element waits (uniform)
        int direct_batches = 0, backoff = 1;
        if constexpr (DEFER) L.pend_init();
        auto flush_all = [&]() {
            if constexpr (DEFER) {
#pragma unroll
                for (int l = 0; l < NL; ++l)
                    if (waiting[l] != 0) { L.flush(l); waiting[l] = 0; }
            }
        };
        for (; s + U <= s_end; s += U) {
            const buffer_rsrc rs = make_rsrc(wg_base + (size_t)s * step_bytes);
            vec_t buf[U][R];
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int r = 0; r < R; ++r)
                    buf[u][r] = VL::load(rs, lane_off[r], (uint32_t)u * step_bytes);
            if constexpr (DEFER) {
                if (direct_batches == 0 && s >= p.defer_from) {
                    int inserted = 0;
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        // one branch per step: when an element of any list wants a place where
                        // another one waits, everything that waits enters its list first
                        float x[NL];
                        bool hit[NL];
                        uint64_t hits[NL], clash = 0;
#pragma unroll
                        for (int r = 0; r < R; ++r)
#pragma unroll
                            for (int v = 0; v < V; ++v) {
                                const int l = r * V + v;
                                x[l] = __uint_as_float(VL::bits(buf[u][r], v) ^ flip);
                                hit[l] = L.beats_least(l, x[l]);
                                hits[l] = __ballot(hit[l]);
                                clash |= hits[l] & waiting[l];
                            }
                        if (clash != 0) { flush_all(); ++inserted; }
#pragma unroll
                        for (int l = 0; l < NL; ++l) {
                            L.set_aside(l, hit[l], x[l], s + u);
                            waiting[l] |= hits[l];
                        }
                    }
                    if (inserted * 4 > U) {
                        flush_all();
                        direct_batches = backoff;
                        backoff = min(backoff * 2, 64);
                    } else {
                        backoff = 1;
                    }
                    continue;
                }
                if (direct_batches > 0) --direct_batches;
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int r = 0; r < R; ++r)
                    consume<TWO_PHASE>(L, buf[u][r], r, s + u, flip);
        }
        flush_all();
        if (s < s_end) {
            // the last, short batch: its loads are issued together as well (a step-by-step tail
            // would pay a memory latency per step); the count is uniform, so the tests are scalar
            const int nlast = s_end - s;                           // 1 .. U-1
            const buffer_rsrc rs = make_rsrc(wg_base + (size_t)s * step_bytes);
            vec_t buf[U][R] = {};
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (u < nlast) {
#pragma unroll
                    for (int r = 0; r < R; ++r)
                        buf[u][r] = VL::load(rs, lane_off[r], (uint32_t)u * step_bytes);
                }
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (u < nlast) {
#pragma unroll
                    for (int r = 0; r < R; ++r) consume<TWO_PHASE>(L, buf[u][r], r, s + u, flip);
                }
            s = s_end;
        }
        }

        if constexpr (!BATCHED) __builtin_amdgcn_s_setprio(0);
        const int C = (p.chunk > 0 ? chunk_len : p.B) * p.Kprime;   // candidates of this workgroup's row (part)
        // where this workgroup's K results go (a chunk of a row has a result of its own)
        const int64_t out_base = (p.chunk > 0 ? (int64_t)row * gridDim.y + blockIdx.y : (int64_t)row) * p.K;
        if constexpr (PACKED) {
            // packed variants only run fused, one owner per bucket, at most 1024 candidates per
            // row: the keys go to LDS as they are and the first wavefront of the row's group
            // sorts them in registers
            uint32_t* cand32 = (uint32_t*)lds + (size_t)g * p.Cpad;
            for (int i = C + t; i < p.Cpad; i += p.G) cand32[i] = 0;
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int v = 0; v < V; ++v)
#pragma unroll
                    for (int k = 0; k < KP; ++k)
                        if (slot_ok[r] && k < p.Kprime) {
                            // same value half, low half now 0xFFFF - position in the row
                            const uint32_t n = L.index(r * V + v, k, (uint32_t)p.S, (uint32_t)(off[r] + v));
                            const uint32_t key = (L.key[r * V + v][k] & 0xffff0000u) | (0xffffu - n);
                            cand32[(off[r] + v) * p.Kprime + k] = row_ok ? key : 0;
                        }
            // a row's keys are written and sorted by the same wavefront unless several share it
            if (p.G > kWave) __syncthreads();
            else __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            if (p.G >= kWave) {
                if (t < kWave && row_ok)
                {
                    if (p.cert_flags)
                        wave_sort32_certify_dispatch<DT>(cand32, p.Cpad, p.K, rowp, p.out_vals, p.out_idx,
                                                         (int64_t)row * p.K, flip, p.cert_flags + row, p.B, p.Kprime);
                    else
                        wave_sort32_dispatch<DT>(cand32, p.Cpad, p.K, rowp, p.out_vals, p.out_idx,
                                                 (int64_t)row * p.K, flip);
                }
            } else {
                // several rows per wavefront: it sorts them one after the other
                const int per_wave = kWave / p.G;
                for (int j = 0; j < per_wave; ++j) {
                    const int gl = (tid >> 6) * per_wave + j;
                    const int rw = blockIdx.x * p.rows_per_wg + gl;
                    if (rw < p.rows)
                    {
                        uint32_t* keys32 = (uint32_t*)lds + (size_t)gl * p.Cpad;
                        const char* rowp_w = (const char*)p.values + (size_t)rw * p.row_stride * ES;
                        if (p.cert_flags)
                            wave_sort32_certify_dispatch<DT>(keys32, p.Cpad, p.K, rowp_w, p.out_vals, p.out_idx,
                                                             (int64_t)rw * p.K, flip, p.cert_flags + rw, p.B, p.Kprime);
                        else
                            wave_sort32_dispatch<DT>(keys32, p.Cpad, p.K, rowp_w, p.out_vals, p.out_idx,
                                                     (int64_t)rw * p.K, flip);
                    }
                }
            }
            return;
        }

        // ---- survivors -> LDS keys (or straight to memory for one-owner mode 1) ---------------
        uint64_t* cand = lds + (size_t)g * p.Cpad;                    // per-row stage-2 segment
        if (p.mode == 4) {
            // survivors through memory, ranking finish: the survivors of every wavefront leave as
            // one sorted run (its lanes' final list entries, a power of two per lane, zeros where
            // there are none), staged in the wavefront's own piece of LDS
            const int lane = tid & (kWave - 1), per_lane = p.run_len / kWave;
            uint64_t* stage = lds + (size_t)(tid >> 6) * p.run_len;
            for (int sl = NL * p.Kprime; sl < per_lane; ++sl) stage[sl * kWave + lane] = 0;
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int v = 0; v < V; ++v)
#pragma unroll
                    for (int k = 0; k < KP; ++k) {
                        if (k >= p.Kprime) continue;
                        const int l = r * V + v;
                        const uint32_t n = L.index(l, k, (uint32_t)p.S, (uint32_t)(off[r] + v));
                        stage[(l * p.Kprime + k) * kWave + lane] =
                            slot_ok[r] && row_ok ? make_key<DT>(stored_bits(L, l, k), n) : 0;
                    }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            if (row_ok)
                wave_sort_run_dispatch(stage, p.run_len, p.part_keys +
                    (((int64_t)row * gridDim.y + blockIdx.y) * (p.G >> 6) + (t >> 6)) * p.run_len);
            return;
        }
        if (p.owners == 1) {
            if (p.mode == 0) {
                for (int i = C + t; i < p.Cpad; i += p.G) cand[i] = 0;
            }
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const bool live = slot_ok[r] && row_ok;
                uint32_t sv_vec[KP][4], si_vec[KP][4];      // mode 1 with 16-byte stores (folded away otherwise)
                (void)sv_vec; (void)si_vec;
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    const int bucket = off[r] + v;
#pragma unroll
                    for (int k = 0; k < KP; ++k) {
                        if (!live || k >= p.Kprime) continue;
                        const int l = r * V + v;
                        const uint32_t n = L.index(l, k, (uint32_t)p.S, (uint32_t)bucket);
                        uint32_t b = stored_bits(L, l, k);
                        if (p.mode == 0) {
                            cand[(bucket - chunk_first) * p.Kprime + k] = make_key<DT>(b, n);
                        } else if (p.mode == 2) {
                            // a segment shorter than K' steps leaves empty entries
                            const int64_t o = (((int64_t)row * p.nseg + blockIdx.y) * p.Kprime + k) * p.B + bucket;
                            p.part_keys[o] = L.valid(l, k) ? make_key<DT>(b, n) : 0;
                        } else {
                            if (!Lists<REP, KP, NL>::exact_bits && (b << 1) == 0)   // either zero
                                b = elem<DT>::load_bits(rowp, n);       // which zero it was
                            else
                                b ^= flip;                            // the stored pattern
                            const int64_t o = ((int64_t)row * p.Kprime + k) * p.B + bucket;
                            if ((V == 4 || V == 2) && elem<DT>::size == 4 && p.surv_aligned) {
                                // the V buckets of a load are neighbours in plane k: one 16- or 8-byte
                                // store each for values and indices (a lane's 4-byte stores, V elements
                                // apart from its neighbours', were measured to write 1.6x the bytes)
                                sv_vec[k][v] = b; si_vec[k][v] = n;
                                if (v == V - 1) {
                                    uint32_t* dv = (uint32_t*)p.surv_vals + (o - (V - 1));
                                    int32_t* di = p.surv_idx + (o - (V - 1));
                                    if constexpr (V == 4) {
                                        *(uint4*)dv = make_uint4(sv_vec[k][0], sv_vec[k][1], sv_vec[k][2], sv_vec[k][3]);
                                        *(uint4*)di = make_uint4(si_vec[k][0], si_vec[k][1], si_vec[k][2], si_vec[k][3]);
                                    } else {
                                        *(uint2*)dv = make_uint2(sv_vec[k][0], sv_vec[k][1]);
                                        *(uint2*)di = make_uint2(si_vec[k][0], si_vec[k][1]);
                                    }
                                }
                            } else {
                                elem<DT>::store_bits(p.surv_vals, o, b);
                                p.surv_idx[o] = (int32_t)n;
                            }
                        }
                    }
                }
            }
            if (p.mode != 0) return;
            if (!row_ok) { for (int i = t; i < C; i += p.G) cand[i] = 0; }
            __syncthreads();
        } else {
            // m owners per bucket: partial lists -> [bucket][owner*KP + k], sort each bucket's
            // segment, keep its first K'.  Partial lists may be short: NaN entries become key 0.
            const int nb = p.mode == 3 ? p.slab_w : p.B;             // buckets of this workgroup
            const int b_first = p.mode == 3 ? (int)blockIdx.y * p.slab_w : 0;
            uint64_t* part = lds + p.aux_offset + (size_t)g * nb * p.seg;
            for (int i = t; i < nb * p.seg + (p.mode == 3 ? p.run_len : 0); i += p.G) part[i] = 0;   // (and the run behind)
            if (p.mode != 3) { for (int i = C + t; i < p.Cpad; i += p.G) cand[i] = 0; }
            __syncthreads();
            if (row_ok) {
#pragma unroll
                for (int v = 0; v < V; ++v) {           // R == 1 in this mode
                    const int e = off[0] + v;
                    const int bucket = e % p.B - b_first, owner = e / p.B;
#pragma unroll
                    for (int k = 0; k < KP; ++k) {
                        const uint32_t n = L.index(v, k, (uint32_t)p.S, (uint32_t)e);
                        if (L.valid(v, k))
                            part[(size_t)bucket * p.seg + owner * KP + k] = make_key<DT>(stored_bits(L, v, k), n);
                    }
                }
            }
            __syncthreads();
            if (p.mode == 3 && p.seg <= 16 * p.owners) {
                // each wavefront holds the lists of 64 / owners buckets, seg / owners keys per
                // lane: sorted in registers, the final K' keys go straight to memory
                const int wave = tid >> 6, per_lane = p.seg / p.owners, per_wave = kWave / p.owners;
                if (p.run_len > 0) {
                    // ranking finish: the workgroup's final keys leave as one sorted run.  They
                    // are gathered behind the partial lists ([j][bucket], entries K' <= j <
                    // run_len / slab_w stay zero as cleared above) and the first wavefront sorts them.
                    uint64_t* run = lds + p.aux_offset + (size_t)nb * p.seg;
                    wave_merge_bucket_lists_dispatch(part + (size_t)wave * kWave * per_lane, per_lane,
                                                     31 - __clz(p.owners), p.Kprime, run + wave * per_wave, nb);
                    __syncthreads();
                    if (wave == 0)
                        wave_sort_run_dispatch(run, p.run_len, p.part_keys +
                            ((int64_t)row * (p.B / p.slab_w) + blockIdx.y) * p.run_len);
                    return;
                }
                if (row_ok)
                    wave_merge_bucket_lists_dispatch(
                        part + (size_t)wave * kWave * per_lane, per_lane, 31 - __clz(p.owners), p.Kprime,
                        p.part_keys + (int64_t)row * p.Kprime * p.B + b_first + wave * per_wave, p.B);
                return;
            }
            lds_bitonic_sort_desc(lds + p.aux_offset, p.rows_per_wg * nb * p.seg, p.seg);
            if (p.mode == 3) {
                // the slab's final lists, laid out like one segment's partial keys
                if (row_ok)
                    for (int i = t; i < nb * p.Kprime; i += p.G) {
                        const int k = i / nb, lb = i - k * nb;
                        p.part_keys[((int64_t)row * p.Kprime + k) * p.B + b_first + lb] =
                            part[(size_t)lb * p.seg + k];
                    }
                return;
            }
            for (int i = t; i < C; i += p.G) {
                const int bucket = i / p.Kprime, k = i - bucket * p.Kprime;
                const uint64_t key = part[(size_t)bucket * p.seg + k];
                if (p.mode == 0) {
                    cand[i] = key;
                } else if (row_ok) {
                    const uint32_t n = key_index(key);
                    const uint32_t b = key_stored_bits<DT>(key, rowp, n, flip);
                    const int64_t o = ((int64_t)row * p.Kprime + k) * p.B + bucket;
                    elem<DT>::store_bits(p.surv_vals, o, b);
                    p.surv_idx[o] = (int32_t)n;
                }
            }
            if (p.mode != 0) return;
            __syncthreads();
        }

        // ---- stage 2: exact Top-K of each row's candidates --------------------------------------
        if (p.tail == 1) {
            // few candidates: the first wavefront of every row's group sorts them in registers
            if (t < kWave && row_ok)
                wave_sort_dispatch<DT>(cand, p.Cpad, p.K, rowp, p.out_vals, p.out_idx, out_base, flip);
            return;
        }
        if (p.tail == 2) {
            // one row per workgroup: thin the candidates out by radix selection, wave-sort the rest
            wg_topk_from_lds<DT>(lds, p.Cpad, p.K, lds + p.aux_offset, rowp, p.out_vals, p.out_idx,
                                 out_base, flip);
            return;
        }
        lds_bitonic_sort_desc(lds, p.rows_per_wg * p.Cpad, p.Cpad);
        if (row_ok) {
            for (int i = t; i < p.K; i += p.G) {
                const uint64_t key = cand[i];
                const uint32_t n = key_index(key);
                elem<DT>::store_bits(p.out_vals, out_base + i, key_stored_bits<DT>(key, rowp, n, flip));
                p.out_idx[out_base + i] = (int32_t)n;
            }
        }
    }
};

// The sorted-batch representation holds two K'-lists of 64-bit keys per lane and is only
// launched with at most 256 lanes per workgroup, which lets it use the larger register budget.
#ifndef ATK_PACKED_WAVES
#define ATK_PACKED_WAVES 6      // wavefronts per SIMD the packed variants are compiled for
#endif
template <typename DT, int KP, int V, int R, int REP, bool MINK>
__global__ void __launch_bounds__(REP == 2 ? 256 : 1024, REP == 1 ? ATK_PACKED_WAVES : 1) approx_topk_kernel(ApproxParams p) {
    extern __shared__ uint64_t atk_lds[];
    ApproxKernel<DT, KP, V, R, REP>::template run<MINK>(p, atk_lds);
}

// Host-side launcher, one explicit instantiation per supported (dtype, KP, V, R, REP).
template <typename DT, int KP, int V, int R, int REP>
hipError_t launch_approx(const ApproxParams& p, int grid, int block, size_t lds_bytes,
                         hipStream_t stream);

#define ATK_DEFINE_LAUNCH(DT, KP, V, R, REP)                                                    \
    template <>                                                                                 \
    hipError_t launch_approx<DT, KP, V, R, REP>(const ApproxParams& p, int grid, int block,     \
                                                   size_t lds_bytes, hipStream_t stream) {      \
        const dim3 g(grid, p.mode == 2 ? p.nseg : (p.mode == 3 ? p.B / p.slab_w :               \
                           (p.chunk > 0 ? (p.B + p.chunk - 1) / p.chunk : 1)));                 \
        if (p.flip == 0) {                                                                      \
            allow_large_lds((const void*)approx_topk_kernel<DT, KP, V, R, REP, false>, lds_bytes); \
            hipLaunchKernelGGL((approx_topk_kernel<DT, KP, V, R, REP, false>), g, dim3(block),  \
                               lds_bytes, stream, p);                                           \
        } else {                                                                                \
            allow_large_lds((const void*)approx_topk_kernel<DT, KP, V, R, REP, true>, lds_bytes); \
            hipLaunchKernelGGL((approx_topk_kernel<DT, KP, V, R, REP, true>), g, dim3(block),   \
                               lds_bytes, stream, p);                                           \
        }                                                                                       \
        return hipGetLastError();                                                               \
    }

}  // namespace atk
