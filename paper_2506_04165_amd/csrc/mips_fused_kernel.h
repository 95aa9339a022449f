// Kernel template of the matmul-fused stage 1 of the approximate Top-K (Section 7.3; appendix "Matmul-fused
// implementation"; Section 6.1 Steps 1-2 on scores that exist only in registers).
//
// Decomposition (ours; the paper's kernel walks a 3-D grid sequentially and keeps the lists in
// on-chip memory, which does not carry over):
//   * a workgroup of 4 wavefronts owns a slab of 32 buckets and a tile of 128 queries, and
//     walks the elements of those buckets: step j covers the database vectors j*B + b0 + [0,32),
//     32 contiguous vectors, so a given accumulator register sees the same (query, bucket)
//     pair at every step and its K'-list lives in registers with static indexing, exactly as
//     in the streaming kernel;
//   * the 32 x D database tile goes through LDS (double buffered, one barrier per step) and is
//     the row operand of v_mfma_f32_32x32x16_bf16; the query fragments are the column operand
//     and stay in registers for the whole walk.  Each wavefront computes a 32 (buckets) x 32
//     (queries) tile of binary32 scores per step: D/16 matrix instructions;
//   * every score then updates its list (Algorithm 1 restated, branch-free; see ScoreLists).
//     Skipping the update when no lane of the wavefront beats its list's tail was measured and
//     is slower: one lane in 64 nearly always does, and the branches serialise the updates;
//   * when there are too few (slab, tile) pairs to fill the chip the walk is cut into
//     segments run by different workgroups; the per-bucket merge of the partial lists and
//     Steps 3-4 are the finishing launch shared with the split streaming path;
//   * the block index is decoded so that the workgroups sharing a database tile (same slab and
//     segment, different queries) run on the same XCD and find the tile in its L2.
//
// Scores are binary32 sums formed by the matrix instruction; accumulation order inside the
// instruction is the hardware's.  A zero score is +0.0 (the accumulator starts at +0.0).
#pragma once
#include "mips_fused.h"
#include "approx_kernel.h"

namespace atk {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

// operand fragment type and matrix instruction for the two 16-bit vector types
template <bool F16> struct MipsFrag {
    using type = bf16x8;
    __device__ static __forceinline__ floatx16 mfma(type a, type b, floatx16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
};
template <> struct MipsFrag<true> {
    using type = f16x8;
    __device__ static __forceinline__ floatx16 mfma(type a, type b, floatx16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
};
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // one 16-byte move

// The K' greatest scores each accumulator register has seen, greatest first, with the step at
// which each arrived.  Scores are finite, so the empty entry is -inf and the values need no
// compare-and-select: entry k becomes the median of (entry k-1, entry k, score), the head the
// maximum (Algorithm 1's shift, as a clamp).  Only the steps follow the compare results.  A
// strict compare keeps the earlier (lower-index) element ahead on ties.  Written without
// branches on purpose: the 16 updates of a step are independent and interleave.
template <int KP>
struct ScoreLists {
    float val[16][KP];
    int32_t stp[16][KP];
    __device__ __forceinline__ void init() {
#pragma unroll
        for (int i = 0; i < 16; ++i)
#pragma unroll
            for (int k = 0; k < KP; ++k) { val[i][k] = -__builtin_inff(); stp[i][k] = 0; }
    }
    __device__ __forceinline__ void insert(int i, float x, int32_t step) {
        if constexpr (KP == 1) {       // measured: two selects on one compare beat max + select
            const bool c0 = x > val[i][0];
            val[i][0] = sel(c0, x, val[i][0]);
            stp[i][0] = sel(c0, step, stp[i][0]);
            return;
        }
        bool c[KP];
#pragma unroll
        for (int k = 0; k < KP; ++k) c[k] = x > val[i][k];
#pragma unroll
        for (int k = KP - 1; k >= 1; --k) {
            stp[i][k] = sel(c[k - 1], stp[i][k - 1], sel(c[k], step, stp[i][k]));
            val[i][k] = __builtin_amdgcn_fmed3f(val[i][k - 1], val[i][k], x);
        }
        stp[i][0] = sel(c[0], step, stp[i][0]);
        val[i][0] = sel(c[0], x, val[i][0]);      // (a float max would be canonicalised: three instructions)
    }
    __device__ __forceinline__ bool valid(int i, int k) const { return val[i][k] != -__builtin_inff(); }
    __device__ __forceinline__ uint32_t bits(int i, int k) const { return __float_as_uint(val[i][k]); }
};

// KS = D / 16: matrix instructions per score tile; MQ: 32-query sub-tiles per wavefront.  With
// MQ = 2 every database fragment read from LDS feeds two matrix instructions (half the LDS
// traffic per score) at the price of twice the lists: only short lists leave room for that.
// F16: the vectors are IEEE binary16 instead of bfloat16 (same layout, the other matrix instruction).
template <int KP, int KS, int MQ, bool F16>
__global__ void __launch_bounds__(256) mips_stage1_kernel(MipsParams p) {
    constexpr int D = KS * 16;
    constexpr int kRowBytes = D * 2 + 16;             // padded: rows 16 apart share no LDS bank
    constexpr int kTileBytes = kMipsSlab * kRowBytes;
    constexpr int NLD = KS / 4;                       // 16-byte loads per thread and step
    // after the walk the same memory stages the keys for coalesced stores: 32 x (256+16) bytes
    // per wavefront
    constexpr int kStageRowBytes = kMipsSlab * 8 + 16;
    constexpr int kStageBytes = 4 * 32 * kStageRowBytes;
    constexpr int kLdsBytes = 2 * kTileBytes > kStageBytes ? 2 * kTileBytes : kStageBytes;
    __shared__ __attribute__((aligned(16))) char lds_raw[kLdsBytes];
    char (*tile)[kTileBytes] = reinterpret_cast<char (*)[kTileBytes]>(lds_raw);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, col = lane & 31;

    // ---- block -> (slab, segment, query tile) ---------------------------------------------------
    const int ngroups = p.nslab * p.nseg;             // (slab, segment) pairs: one database walk each
    int group, qt;
    if ((ngroups & 7) == 0) {
        // consecutive block ids go round the 8 XCDs: keep the nqt workgroups of a walk on one
        const int xcd = blockIdx.x & 7, y = blockIdx.x >> 3;
        group = (y / p.nqt) * 8 + xcd;
        qt = y % p.nqt;
    } else {
        group = blockIdx.x / p.nqt;
        qt = blockIdx.x % p.nqt;
    }
    const int slab = group % p.nslab, seg = group / p.nslab;
    const int b0 = slab * kMipsSlab;
    const int j0 = seg * p.seg_steps;
    const int j1 = min(p.nsteps, j0 + p.seg_steps);

    // ---- query fragments: lane (col, half) holds query col, dims (2s + half)*8 .. +8 of step s ---
    const int q_first = (qt * 4 + wave) * (32 * MQ);          // first query of this wavefront
    using frag_t = typename MipsFrag<F16>::type;
    frag_t qf[MQ][KS];
#pragma unroll
    for (int m = 0; m < MQ; ++m) {
        const int q = q_first + m * 32 + col;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            u32x4 w = {0, 0, 0, 0};
            if (q < p.Q) w = *(const u32x4*)(p.queries + (size_t)q * D + (2 * s + half) * 8);
            qf[m][s] = __builtin_bit_cast(frag_t, w);
        }
    }

    ScoreLists<KP> L[MQ];
#pragma unroll
    for (int m = 0; m < MQ; ++m) L[m].init();

    // ---- walk ------------------------------------------------------------------------------------
    // the tile of step j is 32*D*2 contiguous bytes; thread t moves the 16-byte pieces t + 256u
    // Software pipeline: the matrix instructions of step j+1 are issued before the list updates
    // of step j, so the matrix core and the LDS work under the vector ALU's shadow.
    u32x4 pre[NLD];
    const char* src = (const char*)p.database + ((size_t)j0 * p.B + b0) * (size_t)(D * 2) + tid * 16;
    const size_t step_bytes = (size_t)p.B * (D * 2);
    auto fetch = [&]() {
#pragma unroll
        for (int u = 0; u < NLD; ++u) pre[u] = *(const u32x4*)(src + u * 4096);
        src += step_bytes;
    };
    auto stage = [&](int b) {
#pragma unroll
        for (int u = 0; u < NLD; ++u) {
            const int c = tid + 256 * u;
            *(u32x4*)(tile[b] + (c / (2 * KS)) * kRowBytes + (c % (2 * KS)) * 16) = pre[u];
        }
    };
    floatx16 acc[MQ];
    auto scores_of = [&](int b) {
#pragma unroll
        for (int m = 0; m < MQ; ++m)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[m][i] = 0.0f;
        const char* rowp = tile[b] + col * kRowBytes + half * 16;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const frag_t a = __builtin_bit_cast(frag_t, *(const u32x4*)(rowp + s * 32));
#pragma unroll
            for (int m = 0; m < MQ; ++m) acc[m] = MipsFrag<F16>::mfma(a, qf[m][s], acc[m]);
        }
    };
    if (j0 < j1) {
        fetch();
        stage(0);
        __syncthreads();
        if (j0 + 1 < j1) fetch();
        scores_of(0);
    }
    int buf = 0;
    for (int j = j0; j + 1 < j1; ++j) {
        float x[MQ][16];
#pragma unroll
        for (int m = 0; m < MQ; ++m)
#pragma unroll
            for (int i = 0; i < 16; ++i) x[m][i] = acc[m][i];
        stage(buf ^ 1);          // last read two steps ago, before every wave's previous barrier
        __syncthreads();
        if (j + 2 < j1) fetch();
        scores_of(buf ^ 1);
#pragma unroll
        for (int m = 0; m < MQ; ++m)
#pragma unroll
            for (int i = 0; i < 16; ++i) L[m].insert(i, x[m][i], j);
        // Issue order for the region after the barrier: LDS reads, then each matrix instruction
        // followed by its share of the list updates, so that the matrix core works under the
        // vector ALU (left to itself the scheduler puts all matrix instructions first and the
        // wavefront waits for the chain).
        if constexpr (KP >= 3) {
            __builtin_amdgcn_sched_group_barrier(0x100, KS, 0);           // LDS reads
#pragma unroll
            for (int s = 0; s < KS * MQ; ++s) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);        // one matrix instruction
                __builtin_amdgcn_sched_group_barrier(0x002, (16 * (4 * KP)) / KS, 0);   // vector ALU
            }
        }
        buf ^= 1;
    }
    if (j0 < j1) {
#pragma unroll
        for (int m = 0; m < MQ; ++m)
#pragma unroll
            for (int i = 0; i < 16; ++i) L[m].insert(i, acc[m][i], j1 - 1);
    }

    // ---- partial lists out, as keys --------------------------------------------------------------
    // accumulator i of lane (col, half) is the score of bucket row 8*(i/4) + 4*half + i%4.  A
    // lane's keys of one list position are 32 bytes here, 32 bytes there; they are transposed
    // through LDS so that every query's 32 buckets leave as one 256-byte run.
    __syncthreads();                                   // every wavefront is done with the tiles
    char* stage_w = lds_raw + wave * (32 * kStageRowBytes);
#pragma unroll
    for (int m = 0; m < MQ; ++m) {
#pragma unroll
        for (int k = 0; k < KP; ++k) {
            if (k < p.Kprime) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int bl = 8 * (i >> 2) + 4 * half + (i & 3);
                    const uint32_t n = (uint32_t)L[m].stp[i][k] * (uint32_t)p.B + (uint32_t)(b0 + bl);
                    *(uint64_t*)(stage_w + col * kStageRowBytes + bl * 8) =
                        L[m].valid(i, k) ? make_key<score_t>(L[m].bits(i, k), n) : 0;
                }
                __syncthreads();
                // 16 lanes x 16 bytes cover one query's row; a wavefront stores 4 rows at a time
#pragma unroll
                for (int r = 0; r < 8; ++r) {
                    const int ql = r * 4 + (lane >> 4), chunk = lane & 15;
                    const u32x4 v = *(const u32x4*)(stage_w + ql * kStageRowBytes + chunk * 16);
                    const int qq = q_first + m * 32 + ql;
                    if (qq < p.Q) {
                        uint64_t* dst = p.part_keys + (((size_t)qq * p.nseg + seg) * p.Kprime + k) * p.B + b0;
                        *(u32x4*)((char*)dst + chunk * 16) = v;
                    }
                }
                __syncthreads();
            }
        }
    }
}

template <int KP, bool F16>
hipError_t launch_for_type(const MipsParams& p, hipStream_t stream) {
    const dim3 grid((unsigned)(p.nslab * p.nseg * p.nqt)), block(256);
    switch (p.D) {
        case 64:  hipLaunchKernelGGL((mips_stage1_kernel<KP, 4, mips_subtiles(KP, 64), F16>), grid, block, 0, stream, p); break;
        case 128: hipLaunchKernelGGL((mips_stage1_kernel<KP, 8, mips_subtiles(KP, 128), F16>), grid, block, 0, stream, p); break;
        case 256: hipLaunchKernelGGL((mips_stage1_kernel<KP, 16, mips_subtiles(KP, 256), F16>), grid, block, 0, stream, p); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}
template <int KP>
hipError_t launch_for(const MipsParams& p, hipStream_t stream) {
    return p.f16 ? launch_for_type<KP, true>(p, stream) : launch_for_type<KP, false>(p, stream);
}

}  // namespace

}  // namespace atk
