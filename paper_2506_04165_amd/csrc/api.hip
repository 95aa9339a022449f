// C ABI of libatk: argument validation, launch planning and dispatch (host code only).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <string>

#include "../../include/atk.h"
#include "approx_instances.h"
#include "approx_finish.h"
#include "mips_fused.h"
#include "approx_kernel.h"
#include "topk_exact.h"
#include "certify.h"
#include "select_params.h"

namespace atk {

// ---- compiled kernel variants -------------------------------------------------------------
using LaunchFn = hipError_t (*)(const ApproxParams&, int, int, size_t, hipStream_t);
struct Variant { int dtype, KP, V, R, rep; LaunchFn fn; bool packed() const { return rep == 1; } };

#define ATK_X(TAG, T, KP, V, R, P) extern template hipError_t launch_approx<T, KP, V, R, P>(const ApproxParams&, int, int, size_t, hipStream_t);
ATK_ALL_INSTANCES(ATK_X)
#undef ATK_X

static const Variant kVariants[] = {
#define ATK_X(TAG, T, KP, V, R, P) {TAG, KP, V, R, P, &launch_approx<T, KP, V, R, P>},
    ATK_ALL_INSTANCES(ATK_X)
#undef ATK_X
};

// The variant with the given list length and lists per lane; `vector_ok(V)` says whether
// V-element loads are legal for this problem.  The widest legal load wins.
// `packed_ok`: the problem allows lists of packed 32-bit keys (preferred when compiled).
template <typename Pred>
static const Variant* find_variant(int dtype, int KP, int NL, bool packed_ok, Pred vector_ok) {
    const Variant* best = nullptr;
    for (const Variant& v : kVariants) {
        if (v.dtype != dtype || v.KP != KP || v.V * v.R != NL || !vector_ok(v.V) || v.rep == 2 || v.rep == 4 || v.rep == 5) continue;
        if (v.packed() && !packed_ok) continue;
        if (!best || (v.packed() && !best->packed()) || (v.packed() == best->packed() && v.V > best->V))
            best = &v;
    }
    return best;
}

// ---- limits -------------------------------------------------------------------------------
constexpr int kMaxListLen = 32;          // longest K'-list kept in registers
constexpr int kMaxEntriesPerLane = 32;   // V*R*KP
constexpr int kMaxLanes = 1024;
// Most buckets: a lane reaches the elements of up to 32 steps from one base address through
// 32-bit byte offsets, a step being B elements.
constexpr int kMaxBuckets = 1 << 24;
// Longest row.  Kernel loops step 32-bit element counters by up to a chunk (32768) past the end
// before they test them, so the last 65536 values of the int range stay out.
constexpr int64_t kMaxN = 0x7fffffffLL - 0xffff;
constexpr size_t kLdsBudget = 144 * 1024; // dynamic LDS per workgroup (the CU has 160 KB)
constexpr int kMaxFusedCandidates = 16384;  // keys of one row that stage 2 can hold in LDS
constexpr int kExactCap = 16384;         // exact kernel: largest LDS key buffer
constexpr int kExactMaxK = 8192;
constexpr int64_t kOnepassMinN = 524288; // exact kernel: shortest row that is tried in one pass
constexpr int64_t kTargetWaves = 2048;   // 256 CUs x 4 SIMDs x 2 waves: below this the chip idles
constexpr int64_t kTargetWorkgroups = 256; // ... and with fewer workgroups than CUs some CUs have none
constexpr int kMinSegmentSteps = 8;      // do not cut a row into pieces shorter than this
constexpr int kMaxSegments = 128;
constexpr size_t kMinSplitBytes = 4u << 20;
constexpr int kSlabBuckets = 32;         // buckets per workgroup on the slab route
constexpr size_t kSlabMinRowBytes = 128u << 10;
constexpr size_t kSlabMaxBytes = 256u << 20;

static thread_local std::string g_last_hip_error;

// ---- library-owned scratch for the entry point that may not allocate ------------------------------
// Device memory that exists from the moment the code object is loaded, one copy per GPU, held
// until the process ends.  Host code never uses the array's name as an address: the address on
// the current device is asked for once per device and kept.
constexpr size_t kScratchBytes = ATK_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];          // per device; filled under g_scratch_mutex
static std::mutex g_scratch_mutex;

// Address of `scratch` on the current device (NULL and *err set when HIP refuses).
static void* scratch_on_current_device(hipError_t* err) {
    *err = hipSuccess;
    int dev = 0;
    if ((*err = hipGetDevice(&dev)) != hipSuccess) return nullptr;
    if (dev < 0 || dev >= kMaxDevices) { *err = hipErrorInvalidDevice; return nullptr; }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        *err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (*err != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

static int pow2_ceil(int64_t x) { int p = 1; while (p < x) p <<= 1; return p; }
static int pow2_floor(int64_t x) { int p = 1; while ((int64_t)p * 2 <= x) p <<= 1; return p; }
static int log2_of(int64_t pow2) { int l = 0; while (((int64_t)1 << l) < pow2) ++l; return l; }
static int ilog2(int x) { int l = 0; while ((1 << l) < x) ++l; return l; }
static bool is_pow2(int64_t x) { return x > 0 && (x & (x - 1)) == 0; }
static int elem_size(int dtype) { return (dtype == ATK_BF16 || dtype == ATK_F16) ? 2 : 4; }

// The element type the kernels are compiled for, or -1.  fp16 runs on the bf16 kernels: both are
// sign-magnitude formats, so ordering the 16-bit patterns (or those patterns widened by 16 zero
// bits and compared as binary32) orders the values, -0.0 and +0.0 coincide in both, and results
// are reported as the stored 16-bit patterns; with NaN excluded no reinterpreted fp16 is a NaN.
static int kernel_dtype(int dtype) {
    switch (dtype) {
        case ATK_F32: case ATK_BF16: case ATK_I32: case ATK_U32: return dtype;
        case ATK_F16: return ATK_BF16;
        default: return -1;
    }
}

// ---- developer options ---------------------------------------------------------------------
// Launch-geometry switches for experiments and tests; results never depend on them.  Initial
// values come from the environment, read once when the first call needs them; afterwards only
// atk_set_option changes them, so a product call reads no environment variable.
struct Options {
    int lanes_per_row = 0;    // 0: planner's choice, else a power of two <= 1024
    int segments = 0;         // > 0: force this many row segments on the split route
    int slab = 1;             // 0 never / 1 planner's choice / 2 whenever possible: slab route
    int rank_finish = 1;      // 0: stage 2 of the slab route is never spread over several workgroups per row
    int defer = 1;            // 0: list updates always insert at once; 2: elements are set aside whenever the lists allow it
    int rank_wgs = 2048;      // most workgroups of the ranking finish when survivors go through memory
    int slab_owners = 0;      // 0: planner's choice (8), else a power of two: most lanes that share a bucket on the slab route
    int slab_width = 0;       // 0: planner's choice, else buckets per workgroup on the slab route with the
                              // ranking finish (a power of two >= 32)
    int packed = 1;           // 0: no packed 32-bit keys for 16-bit rows
    int subwave = 1;          // 0: no several-rows-per-wavefront variants
    int batch_min_kp = 16;    // list length from which sorted batches are used
    int mips_segments = 0;    // > 0: segments of the database walk of the fused inner-product entry
    int unfused = 0;          // 1: survivors always go through the workspace (two launches)
    int chunked = 0;          // 1: survivors beyond LDS: every bucket chunk's workgroup runs stage 2 on its
                              // own survivors and passes on its K greatest (smaller workspace; measured
                              // no faster than passing all survivors on, slower when rows are few)
    int onepass = 1;          // 0: the exact kernel always takes two passes over a row; 2: one pass
                              // is tried on short rows too
    int certified = 1;        // 0: the exact entry points never go through the two-stage kernels + certificate
    int reg_rows = 1;         // 0: the exact kernel never keeps a short row in registers
    int exact_threads = 0;    // 0: planner's choice, else lanes of an exact-kernel workgroup (a power of two, 64..1024)
};
static Options g_opt;
static unsigned g_opt_generation = 1;      // bumped by every change: cached plans are keyed on it

static void options_from_env_once() {
    static const bool done = [] {
        auto env = [](const char* name, int fallback) {
            const char* s = std::getenv(name);
            return (s && *s) ? std::atoi(s) : fallback;
        };
        Options o;
        o.lanes_per_row = env("ATK_LANES_PER_ROW", o.lanes_per_row);
        o.segments = env("ATK_SEGMENTS", o.segments);
        o.slab = env("ATK_SLAB", o.slab);
        o.rank_finish = env("ATK_RANK_FINISH", o.rank_finish);
        o.slab_width = env("ATK_SLAB_WIDTH", o.slab_width);
        o.rank_wgs = env("ATK_RANK_WGS", o.rank_wgs);
        o.defer = env("ATK_DEFER", o.defer);
        o.slab_owners = env("ATK_SLAB_OWNERS", o.slab_owners);
        if (o.slab_owners < 0 || o.slab_owners > 32 || (o.slab_owners & (o.slab_owners - 1))) o.slab_owners = 0;
        o.packed = env("ATK_NO_PACKED", 0) ? 0 : 1;
        o.subwave = env("ATK_NO_SUBWAVE", 0) ? 0 : 1;
        o.batch_min_kp = env("ATK_BATCH_MIN_KP", o.batch_min_kp);
        o.mips_segments = env("ATK_MIPS_SEGMENTS", o.mips_segments);
        o.unfused = env("ATK_UNFUSED", o.unfused);
        o.onepass = env("ATK_ONEPASS", o.onepass);
        o.chunked = env("ATK_CHUNKED", o.chunked);
        // an unusable value is ignored, it never turns a legal call into an error
        if (o.lanes_per_row < 0 || o.lanes_per_row > kMaxLanes || (o.lanes_per_row & (o.lanes_per_row - 1)))
            o.lanes_per_row = 0;
        g_opt = o;
        return true;
    }();
    (void)done;
}

// ---- validation (host only; every error can be provoked without a GPU) ----------------------
static int validate_common(const void* values, int dtype, int64_t rows, int64_t N,
                           int64_t row_stride) {
    if (kernel_dtype(dtype) < 0) return ATK_UNSUPPORTED;
    if (rows < 0 || rows > 0x7fffffff || N <= 0 || N > kMaxN || row_stride < N)
        return ATK_INVALID_ARG;
    if (rows > 0 && !values) return ATK_INVALID_ARG;
    if ((uintptr_t)values % elem_size(dtype)) return ATK_INVALID_ARG;
    return ATK_OK;
}

static int validate_method(int64_t N, int K, int Kp, int B) {
    if (B < 1 || N % B != 0) return ATK_INVALID_ARG;             // equal buckets (Section 6.3)
    if (Kp < 1 || Kp > K || (int64_t)Kp > N / B) return ATK_INVALID_ARG;   // 1 <= K' <= K
    if (K < 1 || (int64_t)K > (int64_t)B * Kp || (int64_t)K > N) return ATK_INVALID_ARG;
    return ATK_OK;
}

// ---- launch plan --------------------------------------------------------------------------
struct Plan {
    int status = ATK_OK;
    bool route_exact = false;   // K' == K: the method is the exact Top-K (Section 1)
    bool fused = true;
    const Variant* var = nullptr;
    int G = 0, rows_per_wg = 1, S = 0, nsteps = 0, owners = 1, seg = 0, Cpad = 0;
    int block = 0, grid = 0;
    int tail = 0;               // see ApproxParams::tail
    size_t aux_offset = 0;      // LDS keys before the auxiliary region
    size_t lds = 0;
    size_t workspace = 0;       // bytes the plan needs (0: none)
    int nseg = 1, seg_steps = 0;  // > 1: rows are cut into segments, finished by a second launch
    int chunk = 0, nchunk = 1;    // > 0: a workgroup takes `chunk` buckets of a row over all steps
    int chunk_k = 0;              // > 0: ... and runs stage 2 on them itself, leaving its chunk_k greatest
                                  // (of which the exact kernel picks the row's K); 0: all survivors leave
    int slab_w = 0;             // > 0: workgroups take slabs of this many buckets (see below)
    int defer_from = 0x7fffffff; // variants with deferred insertion: the step from which elements may be set aside
    int run_len = 0;            // slab route, > 0: a slab's final keys leave as one sorted run of this length and
    int rank_runs_per_wg = 0;   // stage 2 is the ranking finish, a workgroup placing the keys of this many runs
};

// Ranking finish: how much of every sorted run is held in LDS, as a power of two.  With q =
// ceil(K / runs) the bound on the K-th key is the least of the runs' q-th keys; a run (a
// near-random sample of the survivors) then has about q + 3 sqrt(q) + 3 keys above the bound,
// and four standard deviations more cover the run that has the most.
static int rank_log_head(int K, int64_t nruns, int log_run) {
    const int64_t q = (K + nruns - 1) / nruns;
    if (q > ((int64_t)1 << log_run)) return log_run;
    const double mu = (double)q + 3.0 * std::sqrt((double)q) + 3.0, need = mu + 4.0 * std::sqrt(mu);
    int lh = 5;
    while (lh < log_run && (((int64_t)1 << lh) < need || ((int64_t)1 << lh) < q)) ++lh;
    return lh;
}

static int list_len_for(int Kp) {
    static const int lens[] = {1, 2, 3, 4, 6, 8, 16, 32};
    for (int l : lens) if (l >= Kp) return l;
    return 0;
}

// Choose how lanes map to buckets.  `stage1_only` plans the survivor-writing launch.
// `ws_avail` is the workspace the caller offers (SIZE_MAX when only asking what would be used):
// splitting rows is an optimisation and is dropped when the workspace is too small for it.
static Plan compute_plan(const void* values, int dtype, int64_t rows, int64_t N, int64_t row_stride,
                         int K, int Kp, int B, bool stage1_only, size_t ws_avail) {
    Plan pl;
    const int es = elem_size(dtype);
    const int KP = list_len_for(Kp);
    if (KP == 0 || KP > kMaxListLen) {
        if (Kp == K && !stage1_only) { pl.route_exact = true; return pl; }
        pl.status = ATK_UNSUPPORTED;
        return pl;
    }
    if (B > kMaxBuckets) { pl.status = ATK_UNSUPPORTED; return pl; }
    int maxNL = kMaxEntriesPerLane / KP;
    if (maxNL > 16) maxNL = 16;
    maxNL = pow2_floor(maxNL);

    // lanes we would like on one row: about 224 elements per lane, within [64, 1024]
    int Gd = pow2_floor(N / 224 > 0 ? N / 224 : 1);
    if (Gd < 64) Gd = 64;
    if (Gd > kMaxLanes) Gd = kMaxLanes;
    // short rows with many survivors: stage 2 (a selection among B*K' keys by the row's lanes) then
    // weighs more than the stream, and wants a lane per eight keys (16384 x 4096, 1024 buckets,
    // K' = 4, bf16: 590 us with 128 lanes a row, 430 us with 512; 2048 x 32768 fp32: 140 -> 93 us)
    if (pow2_ceil((int64_t)B * Kp) > kWaveSortMaxKeys && pow2_ceil((int64_t)B * Kp) <= kMaxFusedCandidates) {
        const int for_stage2 = pow2_ceil((int64_t)B * Kp) / 8 > kMaxLanes ? kMaxLanes : pow2_ceil((int64_t)B * Kp) / 8;
        if (Gd < for_stage2) Gd = for_stage2;
    }
    if (g_opt.lanes_per_row > 0) Gd = g_opt.lanes_per_row;

    auto aligned_for = [&](int V) {
        return B % V == 0 && row_stride % V == 0 && ((uintptr_t)values % (size_t)(V * es)) == 0;
    };

    int G = 0, NL = 1, owners = 1;
    const bool want_shared = B < Gd && B < 64 && is_pow2(B);
    if (want_shared) {
        // several lanes per bucket; partial lists merged through LDS
        G = Gd;
        while (G > B && (N % G != 0)) G >>= 1;
        // keep partial lists + candidates inside the LDS budget
        while (G > B && (size_t)(pow2_ceil((int64_t)(G / B) * KP) * B + pow2_ceil((int64_t)B * Kp)) * 8 > kLdsBudget)
            G >>= 1;
        if (G > B) { owners = G / B; NL = 1; }
        else G = 0;
    }
    // Survivors that do not fit the fused kernel's LDS leave through memory (unfused route), and
    // so does everything when only stage 1 was asked for.
    const bool through_memory = !stage1_only && (pow2_ceil((int64_t)B * Kp) > kMaxFusedCandidates ||
                                                 g_opt.unfused != 0);
    bool chunked = false;
    if (G == 0) {
        owners = 1;
        G = B >= Gd ? Gd : pow2_ceil(B);
        if (G > kMaxLanes) G = kMaxLanes;
        for (;;) {
            NL = pow2_ceil((B + G - 1) / G);
            if (NL <= maxNL) break;
            if (G >= kMaxLanes) {
                // more buckets than one workgroup has list entries for: the row is cut along the
                // bucket axis, every workgroup taking G*NL buckets of it over all steps
                NL = maxNL;
                chunked = true;
                break;
            }
            G <<= 1;
        }
        if ((through_memory || stage1_only) && G >= 64) {
            // nothing is merged inside the workgroup on this route, so cutting a row along the
            // bucket axis costs nothing: smaller workgroups until the chip is full
            auto waves = [&] { return rows * (int64_t)((B + G * NL - 1) / (G * NL)) * (G / 64); };
            // chunks whose survivors fit LDS can run stage 2 themselves (see chunk_k below)
            while (through_memory && g_opt.chunked != 0 && (NL > 1 || G > 256) &&
                   pow2_ceil((int64_t)G * NL * Kp) > kMaxFusedCandidates) {
                if (NL > 1) NL >>= 1; else G >>= 1;
            }
            auto workgroups = [&] { return rows * (int64_t)((B + G * NL - 1) / (G * NL)); };
            while ((waves() < kTargetWaves || workgroups() < kTargetWorkgroups) && (NL > 1 || G > 256)) {
                // (a chunk that runs its own stage 2 should hold a few times K survivors)
                if (through_memory && g_opt.chunked != 0 && (int64_t)G * NL * Kp < 8 * (int64_t)K) break;
                if (NL > 1) NL >>= 1; else G >>= 1;
            }
            chunked = G * NL < B;
        }
        // Short lists: half the lanes with twice the lists each (wider loads, fewer waves per row)
        // measured 3-5 % faster as long as the chip stays full and a lane holds at most 8 entries.
        if (!chunked && g_opt.lanes_per_row == 0 && G >= 128 && NL * 2 * KP <= 8 && B % (NL * 2) == 0 &&
            rows * (int64_t)(G / 2 / 64) >= kTargetWaves &&
            find_variant(dtype, KP, NL * 2, false, aligned_for) != nullptr &&
            find_variant(dtype, KP, NL * 2, false, aligned_for)->V > 1) {
            G >>= 1;
            NL <<= 1;
        }
    }
    // bf16 rows whose indices fit 16 bits: value and index share one 32-bit key
    // (such variants only exist for the plain fused route with at most 1024 candidates per row)
    bool packed_ok = dtype == ATK_BF16 && N <= 65536 && !stage1_only && !through_memory && owners == 1 && G >= 64 &&
                     pow2_ceil((int64_t)B * Kp) <= kWaveSortMaxKeys &&
                     g_opt.packed != 0;
    // sixteen packed lists in one lane: two wavefronts with eight lists per lane stream the row
    // faster (measured on 16384 rows of 14336 with 1024 buckets: 95 -> 90 us)
    // (not when that leaves a lane two-byte loads: 128 buckets at K' = 8, 133 against 113 us)
    if (packed_ok && G == 64 && NL * KP >= 16 && NL >= 4 && g_opt.lanes_per_row == 0) { G = 128; NL >>= 1; }
    if (packed_ok && G == 64 && NL == 1 && is_pow2(B) && rows >= 1024 &&
        g_opt.lanes_per_row == 0 && g_opt.subwave != 0) {
        // many short rows with only 64 buckets: rather than 2-byte loads from 64 lanes, a wavefront
        // works on several rows at once, each lane taking as many consecutive elements per load
        // as its registers allow (measured: a gain only in this case)
        for (int nl = maxNL < 8 ? maxNL : 8; nl > NL; nl >>= 1) {
            if (B % nl != 0 || B / nl < 8) continue;
            const Variant* v = find_variant(dtype, KP, nl, true, aligned_for);
            if (v && v->packed()) { NL = nl; G = B / nl; break; }
        }
    }
    pl.var = find_variant(dtype, KP, NL, packed_ok, aligned_for);
    if (!pl.var) { pl.status = ATK_UNSUPPORTED; return pl; }
    // Long lists with few buckets: sorted batches of 64-bit keys, one bucket per lane, cost about a
    // third of the position-by-position update at K' = 32.
    // (16-bit rows with at most 65535 steps keep packed keys in their lists instead: K'+3 operations
    // per element against about 35 to 56 -- 256 x 262144 bf16, 256 buckets, K' = 16: 165 -> 85 us)
    const bool packed_lists = es == 2 && N / B <= 65535 && g_opt.packed != 0;
    if (!pl.var->packed() && owners == 1 && KP >= g_opt.batch_min_kp && B >= 64 && B <= 256 && !packed_lists) {
        for (const Variant& v : kVariants)
            if (v.rep == 2 && v.dtype == dtype && v.KP == KP) {
                pl.var = &v; G = pow2_ceil(B); NL = 1;
                break;
            }
    }
    const int V = pl.var->V;
    if (chunked && G * NL < B) { pl.chunk = G * NL; pl.nchunk = (B + pl.chunk - 1) / pl.chunk; }
    // Survivors beyond LDS, option "chunked": when the chunks divide the row evenly and each holds
    // at least 2K survivors that fit LDS, a chunk's workgroup runs stage 2 on its own survivors and only its K
    // greatest leave (a row's K greatest are among its chunks' K greatest); the exact kernel then
    // selects among nchunk*K instead of B*K'.
    const bool chunk_fused = through_memory && g_opt.chunked != 0 && pl.chunk > 0 && G >= 256 && B % pl.chunk == 0 &&
                             pow2_ceil((int64_t)pl.chunk * Kp) <= kMaxFusedCandidates &&
                             (int64_t)pl.chunk * Kp >= 2 * (int64_t)K && !pl.var->packed() && pl.var->rep != 2;
    if (chunk_fused) pl.chunk_k = K;
    pl.owners = owners;
    pl.S = owners > 1 ? G * V : B;
    pl.nsteps = (int)(N / pl.S);
    pl.seg = owners > 1 ? pow2_ceil((int64_t)owners * KP) : 0;
    pl.Cpad = pow2_ceil((int64_t)(chunk_fused ? pl.chunk : B) * Kp);

    // rows per workgroup: fill 256 lanes when one row needs fewer
    int rpw = G >= 256 ? 1 : 256 / G;
    while (rpw > 1 && rpw / 2 >= rows) rpw >>= 1;
    // LDS: [candidates of every row of the workgroup][auxiliary: partial lists of shared
    // buckets, later reused as scratch of the selection]
    const bool wave_tail = !stage1_only && G >= 64 && pl.Cpad <= kWaveSortMaxKeys;
    const bool to_memory = stage1_only || (through_memory && !chunk_fused);
    // More candidates than one wavefront sorts: one row per workgroup, so that stage 2 is the
    // selection (rows sharing a workgroup would fall back to a full LDS sort of all their
    // candidates: 16384 x 4096 with 1024 buckets, K' = 4: 2500 us against 120 us)
    if (!to_memory && G >= 64 && pl.Cpad > kWaveSortMaxKeys) rpw = 1;
    auto lds_for = [&](int r) {
        size_t cand = 0, aux = 0;
        if (owners > 1) { cand = (size_t)r * pl.Cpad; aux = (size_t)r * B * pl.seg; }
        else if (pl.var->packed()) cand = (size_t)r * pl.Cpad / 2 + 1;     // 32-bit keys
        else if (!to_memory) cand = (size_t)r * pl.Cpad;
        if (!to_memory && !pl.var->packed() && r == 1 && pl.Cpad > 256 &&
            aux * 8 < (size_t)kSelectScratchBytes)
            aux = (kSelectScratchBytes + 7) / 8;
        return (cand + aux) * 8;
    };
    while (rpw > 1 && lds_for(rpw) > kLdsBudget) rpw >>= 1;
    // The kernel addresses a lane's row by a 32-bit byte offset from the workgroup's first row.
    // Never launch less than a wavefront: when so few rows may share a workgroup that their
    // lanes do not fill one, a row gets more lanes than it has buckets (the extra ones idle).
    while (rpw > 1 && (uint64_t)rpw * (uint64_t)row_stride * es >= (1ull << 31)) rpw >>= 1;
    if (G * rpw < 64) {
        if ((uint64_t)(64 / G) * (uint64_t)row_stride * es < (1ull << 31)) rpw = 64 / G;
        else if (owners == 1) G = 64 / rpw;
        else { pl.status = ATK_UNSUPPORTED; return pl; }   // shared buckets fix the lane count
    }
    pl.G = G;
    pl.rows_per_wg = rpw;
    pl.lds = lds_for(rpw);
    pl.aux_offset = (size_t)rpw * pl.Cpad;
    pl.tail = rpw == 1 ? 2 : (wave_tail ? 1 : 0);
    pl.block = G * rpw;
    pl.grid = (int)((rows + rpw - 1) / rpw);
    pl.fused = !to_memory && pl.lds <= kLdsBudget;
    if (pl.lds > kLdsBudget) { pl.status = ATK_UNSUPPORTED; return pl; }   // (cannot happen)
    if (through_memory) {
        // survivors (or every chunk's K greatest) go through memory: int32 indices, then values
        // (input dtype); the exact kernel then selects among them
        pl.workspace = (size_t)rows * (chunk_fused ? (size_t)pl.nchunk * K : (size_t)B * Kp) * (es + 4);
        pl.fused = false;
        // ... or, stage 2 by ranking: every wavefront's survivors leave as one sorted run of keys
        // and the second launch places each key by counting the keys above it, many workgroups
        // per row (64 x 2^20, K = 1024: 62 against 96 us at (8192, 4), 80 / 130 at (16384, 2)).
        // What it costs grows with the count of runs, 64 to 1024 keys long.
        const int per_lane = pow2_ceil((int64_t)NL * Kp);
        const int64_t nruns = (int64_t)pl.nchunk * (G / 64);
        if (!chunk_fused && g_opt.rank_finish != 0 && owners == 1 && G >= 64 && pl.var->rep != 2 &&
            per_lane <= 16 && rows > 0) {
            const int run_len = 64 * per_lane, log_head = rank_log_head(K, nruns, log2_of(run_len));
            int per_wg = 1;
            while (per_wg < nruns && rows * ((nruns + per_wg - 1) / per_wg) > g_opt.rank_wgs) per_wg <<= 1;
            // LDS reads per thread of a placing workgroup, half of every head being in play
            const int64_t reads = (int64_t)per_wg * ((int64_t)1 << log_head) / 2 * nruns * (log_head + 1) / 256;
            const size_t ws_runs = (size_t)rows * nruns * run_len * 8;
            // (LDS of a placing workgroup: the heads, a rank word per key of its own runs)
            const size_t rank_lds = ((size_t)nruns << log_head) * 8 + (size_t)per_wg * run_len * 4 + 256;
            if ((nruns << log_head) <= kRankMaxHeadKeys && reads <= 1024 && ws_runs <= ws_avail &&
                rank_lds <= kLdsBudget && (size_t)pl.block * per_lane * 8 <= kLdsBudget) {
                pl.run_len = run_len;
                pl.rank_runs_per_wg = per_wg;
                pl.lds = (size_t)pl.block * per_lane * 8;
                pl.workspace = ws_runs;
            }
        }
        if (pl.run_len == 0 && K > kExactMaxK) { pl.status = ATK_UNSUPPORTED; return pl; }
    }

    // Very few rows: give every workgroup a slab of 32 buckets of one row over all steps, with m
    // lanes per bucket taking every m-th step.  A lane then reads 128-byte runs (32 four-byte
    // elements) that lie B elements apart, which costs bandwidth but puts rows * B / 32
    // workgroups on the chip, and unlike segments along the row it leaves nothing to merge:
    // the workgroup ends with the final K' keys of its buckets and the second launch is stage 2
    // alone.
    if (pl.fused && owners == 1 && G >= 64 && rows > 0 && B % kSlabBuckets == 0 &&
        pl.var->rep != 2 && g_opt.slab != 0) {
        const int64_t steps = N / B;
        int m = g_opt.slab_owners > 0 ? g_opt.slab_owners : 8;
        while (m > 1 && (steps % m != 0 || steps / m < 4 || m * KP > 64 || m * kSlabBuckets > kMaxLanes)) m >>= 1;
        const Variant* v = find_variant(dtype, KP, 1, false, [](int V) { return V == 1; });
        const size_t in_bytes = (size_t)rows * N * es;
        const size_t ws = (size_t)rows * Kp * B * 8;
        // measured against the other routes on 1..128 rows of 2^16..2^20 elements (GPU time with
        // the queue kept full): a gain of 5-55 % inside these limits; beyond them the strided
        // runs cost more than the extra workgroups bring
        // Stage 2 spread over several workgroups per row: every slab's keys leave as a sorted
        // run and the second launch places each key by counting the keys above it, which
        // costs in proportion to the count of runs.  Slabs are therefore widened until a run
        // has 128 keys, and 256 while there are more than 32 runs (K' = 2: 64 or 128 buckets,
        // K' = 1: 128), with fewer lanes per bucket so that the workgroup keeps 256 lanes.
        // Measured on 8 x 262144, K = 1024 (GPU time per call): 15.4 against 22.9 us at
        // (1024, 4), 13.7 / 20.7 at (2048, 2), 15.0 / 23.0 at (4096, 2), 14.5 / 25.1 at
        // (8192, 1), 23.0 / 36.1 at (512, 8), 22.2 / 31.3 at (8192, 2).  The gain shrinks as
        // rows are added (there are then enough single-workgroup finishes to fill the chip)
        // and is gone where a workgroup would have to place the keys of more than two runs
        // (1 to 64 rows of 2^16 to 2^20 elements, K = 64 to 1024: 64 rows at (1024, 4) 42.6
        // against 28.8 us).
        const int kp2 = (int)pow2_ceil(Kp);
        int slab_w = kSlabBuckets;
        if (g_opt.slab_width >= kSlabBuckets && B % g_opt.slab_width == 0) {
            slab_w = g_opt.slab_width;
        } else {
            while ((slab_w * kp2 < 128 || (slab_w * kp2 < 256 && B / slab_w > 32)) &&
                   slab_w < 128 && B % (2 * slab_w) == 0)
                slab_w *= 2;
        }
        int mr = m;
        while (mr > 2 && slab_w * mr > (g_opt.slab_owners > 0 ? kMaxLanes : 256)) mr >>= 1;
        const int run_len = slab_w * kp2;
        const int64_t nruns = B / slab_w;
        const size_t ws_runs = (size_t)rows * nruns * run_len * 8;
        const bool ranked = g_opt.rank_finish != 0 && run_len <= 256 && slab_w * mr <= kMaxLanes &&
                            pow2_ceil((int64_t)mr * KP) <= 16 * mr && (nruns << rank_log_head(K, nruns, log2_of(run_len))) <= kRankMaxHeadKeys &&
                            rows * nruns <= 1024 && ws_runs <= ws_avail;
        const bool few = rows <= 64 && (ranked || rows * (B / kSlabBuckets) <= 2048) && B >= 256 &&
                         !pl.var->packed() && (size_t)N * es >= kSlabMinRowBytes &&
                         (size_t)(N / B) * es <= 4096 && in_bytes <= kSlabMaxBytes;
        if (m > 1 && v && v->V == 1 && v->R == 1 && (ws <= ws_avail || ranked) &&
            (g_opt.slab == 2 || few)) {
            pl.var = v;
            pl.rows_per_wg = 1;
            pl.grid = (int)rows;
            pl.aux_offset = 0;
            auto shape = [&](int slab_width, int owners_) {
                pl.slab_w = slab_width;
                pl.G = pl.block = slab_width * owners_;
                pl.owners = owners_;
                pl.S = owners_ * B;
                pl.nsteps = (int)(N / pl.S);
                pl.seg = pow2_ceil((int64_t)owners_ * KP);
                pl.lds = (size_t)slab_width * pl.seg * 8;
            };
            if (ranked) {
                shape(slab_w, mr);
                pl.run_len = run_len;
                pl.rank_runs_per_wg = rows * nruns <= 512 ? 1 : 2;
                pl.lds += (size_t)run_len * 8;
                pl.workspace = ws_runs;
            } else {
                shape(kSlabBuckets, m);
                pl.workspace = ws;
            }
            return pl;
        }
    }

    // Too few rows to fill the chip: cut every row into segments streamed by separate
    // workgroups (aim: at least 2 waves on each of the 1024 SIMDs), merged by a finishing launch.
    if (pl.fused && owners == 1 && G >= 64 && rows > 0 && !pl.var->packed()) {
        const int64_t waves = (int64_t)pl.grid * (pl.block / 64);
        int want = (int)((kTargetWaves + waves - 1) / waves);
        // (... and a workgroup on every CU: 128 rows of 1024 lanes are 2048 waves on half the chip)
        if (pl.grid * 2 <= kTargetWorkgroups && want < kTargetWorkgroups / pl.grid) want = (int)(kTargetWorkgroups / pl.grid);
        const int max_by_len = pl.nsteps / kMinSegmentSteps;
        if (want > max_by_len) want = max_by_len;
        if (want > kMaxSegments) want = kMaxSegments;
        // worth it only for real streams, and only while the partial lists stay a small
        // fraction of the bytes streamed (half of them when most of the chip would idle)
        const size_t in_bytes = (size_t)rows * N * es;
        const size_t per_seg = (size_t)rows * Kp * B * 8;
        size_t ws_cap = waves * 2 <= kTargetWaves ? in_bytes / 2 : in_bytes / 8;
        if (ws_cap > ws_avail) ws_cap = ws_avail;
        if ((size_t)want > ws_cap / per_seg) want = (int)(ws_cap / per_seg);
        if (in_bytes < kMinSplitBytes) want = 1;
        // Fewer segments than would fill the chip can still be faster: the finishing launch
        // merges nseg*K' keys per bucket, sixteen loads at a time, and few rows make it pure
        // latency.  Rough per-row model in microseconds (constants measured on 8 x 262144 rows):
        // a workgroup streams ~45 GB/s on its own, the second launch and the round trip through
        // memory cost ~6, every batch of sixteen keys per bucket pass ~3 (~1 from 8 rows on, more
        // when a row's batch is more than a latency's worth of bytes).
        // The stream itself is the slower of two things: a row's own rate (its lanes' loads in
        // flight: a row of fewer than 256 lanes streams in proportion to its lanes) and the chip's
        // (every wavefront keeps 64 x U x R x V elements in flight for about 1.5 us; about 5 TB/s
        // once there are enough of them, and about 28 GB/s per CU that has a workgroup).  Measured: 8 x 2^24 with 64 buckets 484 -> 180 us (32 ->
        // 128 segments), 32 x 2^22 253 -> 118 us, 12 x 2^20 119 -> 47 us.
        if (want > 1) {
            const double row_bytes = (double)N * es;
            const double lanes_share = G >= 256 ? 1.0 : G / 256.0;
            const int dw = (pl.var->V * es + 3) / 4;
            int inflight = 32 / (pl.var->R * dw);
            inflight = inflight < 1 ? 1 : (inflight > 16 ? 16 : inflight);
            const double wave_rate = 64.0 * inflight * pl.var->R * pl.var->V * es / 1.5;      // bytes per us
            // one batch of a row: a memory latency, or its B x 16 keys at what one workgroup reads
            const double per_batch = std::max(rows >= 8 ? 1.0 : 3.0, B * 128.0 / 30e3);
            auto cost = [&](int n) {
                const double busy_cus = std::min<double>(256.0, (double)pl.grid * n);
                const double chip = std::min({5e6, (double)waves * n * wave_rate, busy_cus * 28e3});
                const double own = row_bytes / n / (45e3 * lanes_share);
                const double stream = std::max(own, (double)in_bytes / chip);
                if (n == 1) return stream;
                return stream + 6.0 + per_batch * ((n * Kp + 15) / 16);
            };
            int best = 1;
            for (int n = 2; n <= want; n = (n * 2 <= want || n == want) ? n * 2 : want)
                if (cost(n) < cost(best)) best = n;
            want = best;
        }
        const int forced = g_opt.segments;
        if (forced > 0 && (size_t)forced * per_seg <= ws_avail) want = forced;
        if (want > pl.nsteps) want = pl.nsteps;
        if (want > 1) {
            const int seg_steps = (pl.nsteps + want - 1) / want;
            const int nseg = (pl.nsteps + seg_steps - 1) / seg_steps;
            if (nseg > 1) {
                pl.nseg = nseg;
                pl.seg_steps = seg_steps;
                pl.workspace = (size_t)nseg * per_seg;
                pl.lds = 0;     // the streaming launch keeps nothing in LDS
            }
        }
    }
    return pl;
}

// The plan is a pure function of these arguments and the options, and callers in a loop repeat
// them: the last few plans of a thread are kept.
static const Plan& make_plan(const void* values, int dtype, int64_t rows, int64_t N, int64_t row_stride,
                             int K, int Kp, int B, bool stage1_only, size_t ws_avail = SIZE_MAX) {
    options_from_env_once();
    struct Key {
        unsigned generation; int dtype, K, Kp, B, align; bool stage1_only;
        int64_t rows, N, row_stride; size_t ws_avail;
        bool operator==(const Key& o) const {
            return generation == o.generation && dtype == o.dtype && K == o.K && Kp == o.Kp && B == o.B &&
                   align == o.align && stage1_only == o.stage1_only && rows == o.rows && N == o.N &&
                   row_stride == o.row_stride && ws_avail == o.ws_avail;
        }
    };
    constexpr int kSlots = 8;
    static thread_local Key keys[kSlots];
    static thread_local Plan plans[kSlots];
    static thread_local int used = 0, next = 0;
    // only the alignment of the base address enters the plan (which vector loads are legal)
    const Key key{g_opt_generation, dtype, K, Kp, B, (int)((uintptr_t)values & 15), stage1_only,
                  rows, N, row_stride, ws_avail};
    for (int i = 0; i < used; ++i)
        if (keys[i] == key) return plans[i];
    const int slot = used < kSlots ? used++ : (next = (next + 1) % kSlots);
    keys[slot] = key;
    Plan& pl = plans[slot];
    pl = compute_plan(values, dtype, rows, N, row_stride, K, Kp, B, stage1_only, ws_avail);
    // Value+step lists, long buckets: the variant that sets an element aside when it beats its
    // list's least entry and inserts it later (wavefront-uniform branch, rarely taken) instead of
    // updating the list with every element.  Measured: lists of 8 entries from 128 steps a row
    // on (1024 x 65536, 256 buckets: 81 -> 75 us; 512 x 262144: 160 -> 126 us), lists of 3 and 4
    // from 768 steps (256 x 2^20, 1024 buckets, K' = 4: 170 -> 166 us; at 500 steps and fewer, or
    // with one list per lane -- one branch per element then -- 1-4 % slower), from 256 steps for
    // 16-bit rows, which reach the vector ALU's limit at half the operations per element (4096 x
    // 131072 bf16, 256 buckets, K' = 4: 304 -> 241 us); never lists of 2 (bf16: 99 -> 118 us).
    // Option "defer": 0 never, 2 wherever such a variant exists.
    // 16-bit rows on the value+step lists (too long for keys that hold the position, or off the plain
    // fused route): the variant whose lists hold packed keys of value and step -- K'+3 operations
    // per element instead of 4K'-1 -- and which builds the general keys from them afterwards.
    // The step must fit 16 bits.  (4096 x 131072 bf16, 256 buckets, K' = 4: 241 -> 150 us.)
    if (pl.status == ATK_OK && !pl.route_exact && pl.var && pl.var->rep == 0 && elem_size(pl.var->dtype) == 2 &&
        pl.nsteps <= 65535 && g_opt.packed != 0) {
        for (const Variant& v : kVariants)
            if (v.rep == 5 && v.dtype == pl.var->dtype && v.KP == pl.var->KP && v.V == pl.var->V && v.R == pl.var->R) {
                pl.var = &v;
                break;
            }
    }
    if (pl.status == ATK_OK && !pl.route_exact && pl.var && pl.var->rep == 0 && g_opt.defer != 0) {
        const int steps = pl.nseg > 1 ? pl.seg_steps : pl.nsteps;
        const int lists = pl.var->V * pl.var->R, kp = pl.var->KP;
        const bool pays = kp >= 6 ? steps >= 128
                                  : (kp >= 3 && lists >= 2 && steps >= (elem_size(pl.var->dtype) == 2 ? 256 : 768));
        if (pays || g_opt.defer == 2)
            for (const Variant& v : kVariants)
                if (v.rep == 4 && v.dtype == pl.var->dtype && v.KP == pl.var->KP && v.V == pl.var->V && v.R == pl.var->R) {
                    pl.var = &v;
                    pl.defer_from = 8 * v.KP;
                    break;
                }
    }
    return pl;
}

static ApproxParams params_from(const Plan& pl, const void* values, int64_t rows, int64_t N,
                                int64_t row_stride, int K, int Kp, int B) {
    ApproxParams p{};
    p.values = values;
    p.row_stride = row_stride;
    p.rows = (int)rows; p.N = (int)N; p.K = K; p.Kprime = Kp; p.B = B;
    p.G = pl.G; p.log2G = ilog2(pl.G);
    p.rows_per_wg = pl.rows_per_wg;
    p.S = pl.S; p.nsteps = pl.nsteps; p.owners = pl.owners; p.seg = pl.seg; p.Cpad = pl.Cpad;
    p.aux_offset = (int)pl.aux_offset; p.tail = pl.tail;
    p.chunk = pl.chunk;
    p.defer_from = pl.defer_from;
    return p;
}

// The mask that reverses the order of an element type (kernel dtype), xor-ed onto its (widened)
// bit pattern: the sign bit of a floating type, every bit of an integer.  0 for the K greatest.
static uint32_t flip_mask(int dtype, bool smallest) {
    if (!smallest) return 0;
    return (dtype == ATK_I32 || dtype == ATK_U32) ? 0xffffffffu : 0x80000000u;
}

static int hip_fail(hipError_t e) {
    g_last_hip_error = hipGetErrorString(e);
    return ATK_HIP_ERROR;
}

static int exact_threads(int64_t N) {
    if (g_opt.exact_threads) return g_opt.exact_threads;
    int t = pow2_ceil((N + 63) / 64);     // about 64 elements per lane, more lanes for long rows
    if (t < 64) t = 64;
    if (t > 1024) t = 1024;
    return t;
}

// `payload` non-null: `values` are survivors [rows, N] with their original positions in
// `payload`, taken from the rows of `orig` (stride `orig_stride`), which is only read to tell
// the two zeros apart.
static int run_exact(const void* values, const int32_t* payload, int dtype, int64_t rows, int64_t N,
                     int64_t row_stride, int K, void* out_vals, int32_t* out_idx, hipStream_t st,
                     const void* orig = nullptr, int64_t orig_stride = 0, uint32_t flip = 0,
                     const int32_t* row_mask = nullptr) {
    if (K > kExactMaxK) return ATK_UNSUPPORTED;
    TopkParams tp{};
    tp.flip = flip;
    tp.row_mask = row_mask;
    tp.values = values; tp.payload = payload; tp.row_stride = row_stride;
    tp.orig_values = orig; tp.orig_stride = orig_stride;
    tp.rows = (int)rows; tp.N = (int)N; tp.K = K;
    // LDS key buffer: room for 4K keys (members + candidates of the threshold digit) within
    // [1024, 4096] -- a small buffer lets more rows share a CU -- and 2K keys for larger K
    tp.cap = pow2_ceil(4 * (int64_t)K);
    if (tp.cap < 1024) tp.cap = 1024;
    if (tp.cap > 4096) tp.cap = K <= 2048 ? 4096 : pow2_ceil(2 * (int64_t)K);
    if (tp.cap > kExactCap) tp.cap = kExactCap;
    int threads = exact_threads(N);
    // One pass with a rising threshold where it pays: rows long enough that a second pass costs
    // more than the compactions of the buffer and the drained load pipeline at every look at
    // the fill (measured: 1.6x faster on rows of 2^20 elements, even at 256000, slower from 65536
    // down; option "onepass" = 2 forces it for tests).  The buffer must take a round of the whole workgroup (one
    // vector load per lane) on top of what a compaction leaves, at most 1024 keys.
    if (g_opt.onepass != 0 && K <= 1024 && (N >= kOnepassMinN || g_opt.onepass == 2) && threads >= 256) {
        int t1 = threads;
        if (elem_size(dtype) == 2 && !payload && t1 > 512) t1 = 512;     // eight elements per vector
        const int round = t1 * (payload ? 1 : 16 / elem_size(dtype));
        int cap1 = pow2_ceil(1024 + (int64_t)round);
        if (cap1 < tp.cap) cap1 = tp.cap;
        if (cap1 <= 8192 && cap1 <= 16 * t1) { tp.cap = cap1; tp.onepass = 1; threads = t1; }
    }
    // A short row goes into registers once (all of its loads in flight together) and every pass
    // runs from there.
    const int ve = 16 / elem_size(dtype);
    if (g_opt.reg_rows != 0 && !payload && !tp.onepass && g_opt.exact_threads == 0 && N % ve == 0 &&
        N <= (int64_t)kRegRowThreads * ve * kRegRowVectors && N * elem_size(dtype) >= 4096) {
        tp.reg_row = 1;
        threads = kRegRowThreads;
    }
    tp.out_vals = out_vals; tp.out_idx = out_idx;
    hipError_t e = launch_topk_exact(tp, dtype, threads, st);
    return e == hipSuccess ? ATK_OK : hip_fail(e);
}

}  // namespace atk

using namespace atk;

// ---- matmul-fused path (Section 7.3): plan ---------------------------------------------------------
namespace {

struct MipsPlan {
    int status = ATK_OK;
    int KP = 0, nslab = 0, nqt = 0, nseg = 1, seg_steps = 0, Cpad = 0;
    size_t workspace = 0;
};

constexpr int kMipsTargetWorkgroups = 512;   // 2 wavefronts per SIMD on 256 CUs
constexpr int kMipsMinSegmentSteps = 64;     // shorter walks only refill lists

MipsPlan make_mips_plan(int dtype, int64_t Q, int64_t N, int64_t D, int K, int Kprime, int B) {
    options_from_env_once();
    MipsPlan pl;
    if (Q < 0 || N <= 0 || N > kMaxN || D <= 0) { pl.status = ATK_INVALID_ARG; return pl; }
    if ((pl.status = validate_method(N, K, Kprime, B))) return pl;
    if ((dtype != ATK_BF16 && dtype != ATK_F16) || (D != 64 && D != 128 && D != 256) || B % kMipsSlab || Kprime > 4 ||
        (int64_t)B * Kprime > 16384 || Q > 0x7fffffffLL / 2) {
        pl.status = ATK_UNSUPPORTED;
        return pl;
    }
    pl.KP = Kprime;
    pl.nslab = B / kMipsSlab;
    const int qtile = kMipsQueryTile * mips_subtiles(pl.KP, (int)D);
    pl.nqt = (int)((Q + qtile - 1) / qtile);
    const int nsteps = (int)(N / B);
    const int64_t pairs = (int64_t)pl.nslab * (pl.nqt > 0 ? pl.nqt : 1);
    int nseg = (int)((kMipsTargetWorkgroups + pairs - 1) / pairs);
    nseg = std::min(nseg, std::max(1, nsteps / kMipsMinSegmentSteps));
    nseg = std::max(1, std::min(nseg, 16));
    const int forced = g_opt.mips_segments;                      // developer option
    if (forced >= 1 && forced <= 64 && forced <= nsteps) nseg = forced;
    pl.seg_steps = (nsteps + nseg - 1) / nseg;
    pl.nseg = (nsteps + pl.seg_steps - 1) / pl.seg_steps;
    pl.Cpad = (int)pow2_ceil((int64_t)B * Kprime);
    pl.workspace = (size_t)Q * pl.nseg * Kprime * B * 8;
    return pl;
}

}  // namespace

namespace {

// ---- exact Top-K through the two-stage kernels plus a certificate ------------------------------
// Where rows are long against K, the exact entry points run the approximate path at a (B, K')
// for which a bucket rarely holds more than K' of the K greatest, then the certificate kernel
// (certify.hip) proves the rows exact or repairs them from the few buckets in doubt, and the
// radix-selection kernel takes whatever rows that kernel gave up on.
struct CertPlan { int B = 0, Kprime = 0; };      // B == 0: not applicable

// Expected number of buckets per row that hold at least kp of the K greatest elements, placement
// at random: B * P[Binomial(K, 1/B) >= kp] (the balls-in-buckets model of Section 6.2).
static double expected_full_buckets(int K, int B, int kp) {
    const double q = 1.0 / B;
    double term = std::pow(1.0 - q, K), below = 0.0;          // P[X = i], i = 0 ...
    for (int i = 0; i < kp; ++i) {
        below += term;
        term *= (double)(K - i) / (i + 1) * q / (1.0 - q);
    }
    return B * std::fmax(0.0, 1.0 - below);
}

constexpr int kCertKprime = 4;              // the fast list length (one maximum and three medians per element)
constexpr int kCertMinK = 8;                // below, K' = 4 would be K' >= K
constexpr int kCertMinRowPerSurvivor = 16;  // N >= 16 B K': otherwise stage 2 costs more than a second pass
constexpr int kCertMaxScan = 65536;         // elements a repairing workgroup reads again

static CertPlan certified_params(int dtype, int64_t rows, int64_t N, int K) {
    struct Slot { int64_t rows, N; int K, es; unsigned gen; CertPlan cp; };
    thread_local Slot last{0, 0, 0, 0, 0, {}};
    options_from_env_once();
    const int es = elem_size(dtype);
    if (last.rows == rows && last.N == N && last.K == K && last.es == es && last.gen == g_opt_generation) return last.cp;
    CertPlan cp;
    if (g_opt.certified != 0 && K < kCertMinK && (K <= 4 || rows <= 64)) {
        // Very small K: lists of K' = K entries keep the whole Top-K by construction (Section 1: the
        // method is exact there), so the two-stage kernels give the exact result with nothing to
        // certify.  Survivors (B x K, K rounded up to a power of two) at
        // most a sixteenth of the row, between 256 and 4096, and at most 1024 where that keeps
        // 16-bit rows on the packed-key kernels.  Lists of more than four entries only where the
        // rows are too few for the radix kernel to fill the chip (it takes a workgroup per row).
        // Measured against the radix kernel: 8 x 2^23 fp32, K = 1: 69 against 447 us; 1 x 2^24: 65 /
        // 708; 16384 x 4096: 69 / 113; 50000 x 1024 bf16: 28 / 369.
        int64_t survivors = N / 16 < 256 ? 256 : (N / 16 > 4096 ? 4096 : N / 16);
        if (es == 2 && N <= 65536 && survivors > kWaveSortMaxKeys) survivors = kWaveSortMaxKeys;
        // (rows of fewer than 4096 elements: 64 buckets, the shape for which a wavefront takes several
        // rows at once -- 100000 x 512: 146 against 693 us, bf16 34 against 443 us)
        const bool tiny = N < 4096;
        const int64_t most = tiny ? 64 : survivors / pow2_ceil(K);
        auto fits = [&](int64_t B) { return N % B == 0 && N / B >= (tiny ? 2 : 16) && N / B >= K; };
        for (int64_t B = pow2_floor(most); B >= 64 && B * 4 >= most && !cp.B; B >>= 1)     // a power of two near the budget,
            if (fits(B)) { cp.B = (int)B; cp.Kprime = K; }
        for (int64_t B = most; B >= 64 && !cp.B; --B)                                        // else the greatest divisor of N
            if (fits(B)) { cp.B = (int)B; cp.Kprime = K; }
    }
    if (g_opt.certified != 0 && K >= kCertMinK && K <= kWaveSortMaxKeys) {
        // smallest B (fewest survivors) at which nearly every row is certified at once; failing
        // that, the smallest at which a row needs about one bucket repaired.  Powers of two first
        // (the fast kernels), then any divisor of N.
        int chosen = 0;
        for (int pass = 0; pass < 2 && !chosen; ++pass) {
            int fallback = 0;
            for (int64_t B = 64; B <= kCertifyMaxB; B = pass ? B + 1 : B << 1) {
                if (B * kCertKprime * kCertMinRowPerSurvivor > N) break;
                if (N % B || N / B <= kCertKprime || B * kCertKprime < K) continue;
                const double e = expected_full_buckets(K, (int)B, kCertKprime);
                if (e <= 0.05) { fallback = (int)B; break; }
                if (e <= 1.5 && !fallback) fallback = (int)B;
            }
            chosen = fallback;
        }
        if (chosen) { cp.B = chosen; cp.Kprime = kCertKprime; }
        // Short rows of 16-bit elements: the packed-key kernels run stage 2 on up to 1024 survivors
        // at streaming speed whatever the row length, so the rule above (rows long against the
        // survivors) need not hold; K' = 8 then keeps buckets in doubt rare where K' = 4 cannot
        // (c2: K = 287 of 14336 at (128, 8): 0.3 buckets per row).
        if (!chosen && es == 2 && N <= 65536 && g_opt.packed != 0) {
            double best = 1.5;
            for (int kp = 4; kp <= 8; kp += 4)
                for (int64_t B = kWaveSortMaxKeys / kp; B >= 16; B >>= 1) {
                    if (N % B || N / B <= kp || B * kp < K) continue;
                    const double e = expected_full_buckets(K, (int)B, kp);
                    if (e <= best) { best = e; cp.B = (int)B; cp.Kprime = kp; }
                    if (e <= 0.05) break;
                }
        }
    }
    last = {rows, N, K, es, g_opt_generation, cp};
    return cp;
}

// two words per row: rows left to the radix kernel, rows the two-stage launch left open
static size_t certified_lists_bytes(int64_t rows) { return 2 * (((size_t)rows * 4 + 255) & ~(size_t)255); }

static int approx_impl(const void* values, int dtype, int64_t rows, int64_t N, int64_t row_stride,
                       int K, int Kprime, int B, void* out_vals, int32_t* out_idx,
                       void* workspace, size_t workspace_bytes, void* stream, bool smallest,
                       int32_t* cert_flags = nullptr);

// dtype: the kernel's (fp16 already mapped).  Arguments validated by the caller.  A workspace that
// is absent or too small for the certified route only selects the radix-selection kernel.
static int exact_dispatch(const void* values, int dtype, int64_t rows, int64_t N, int64_t row_stride, int K,
                          void* out_vals, int32_t* out_idx, void* workspace, size_t workspace_bytes,
                          hipStream_t st, bool smallest) {
    const uint32_t flip = flip_mask(dtype, smallest);
    const CertPlan cp = certified_params(dtype, rows, N, K);
    if (cp.B && cp.Kprime >= K)          // exact by construction: the two-stage call is the whole job
        return approx_impl(values, dtype, rows, N, row_stride, K, cp.Kprime, cp.B, out_vals, out_idx,
                           (uintptr_t)workspace % 8 == 0 ? workspace : nullptr, workspace_bytes, (void*)st, smallest);
    const size_t lists = certified_lists_bytes(rows);
    if (cp.B && workspace && (uintptr_t)workspace % 8 == 0 && workspace_bytes >= lists) {
        const size_t rest = workspace_bytes - lists;
        size_t need;
        bool tail_certifies;        // the packed-key variants take the certificate in their own tail
        {
            const Plan& pl = make_plan(values, dtype, rows, N, row_stride, K, cp.Kprime, cp.B, false, rest);
            need = (pl.status == ATK_OK && !pl.route_exact) ? pl.workspace : SIZE_MAX;
            tail_certifies = need != SIZE_MAX && pl.fused && pl.var->packed();
        }
        if (need <= rest) {
            int32_t* open_rows = tail_certifies ? (int32_t*)((char*)workspace + lists / 2) : nullptr;
            int rc = approx_impl(values, dtype, rows, N, row_stride, K, cp.Kprime, cp.B, out_vals, out_idx,
                                 (char*)workspace + lists, rest, (void*)st, smallest, open_rows);
            if (rc) return rc;
            CertifyParams c{};
            c.values = values; c.row_stride = row_stride;
            c.rows = (int)rows; c.N = (int)N; c.K = K; c.Kprime = cp.Kprime; c.B = cp.B;
            c.flip = flip;
            c.cap = (int)pow2_ceil(2 * (int64_t)K);
            if (c.cap < 1024) c.cap = 1024;
            c.max_scan = kCertMaxScan;
            c.rows_per_wg = (rows >= 4096 && cp.B <= 1024) ? kCertifyRowsPerWg : 1;
            c.out_vals = out_vals; c.out_idx = out_idx;
            c.hard_rows = (int32_t*)workspace;
            c.open_rows = open_rows;
            hipError_t e = launch_certify(c, dtype, st);
            if (e != hipSuccess) return hip_fail(e);
            return run_exact(values, nullptr, dtype, rows, N, row_stride, K, out_vals, out_idx, st,
                             nullptr, 0, flip, c.hard_rows);
        }
    }
    return run_exact(values, nullptr, dtype, rows, N, row_stride, K, out_vals, out_idx, st, nullptr, 0, flip);
}

static int approx_impl(const void* values, int dtype, int64_t rows, int64_t N, int64_t row_stride,
                       int K, int Kprime, int B, void* out_vals, int32_t* out_idx,
                       void* workspace, size_t workspace_bytes, void* stream, bool smallest,
                       int32_t* cert_flags) {
    int rc = validate_common(values, dtype, rows, N, row_stride);
    if (rc) return rc;
    dtype = kernel_dtype(dtype);       // fp16 -> the bf16 kernels
    rc = validate_method(N, K, Kprime, B);
    if (rc) return rc;
    if (rows > 0 && (!out_vals || !out_idx)) return ATK_INVALID_ARG;
    if ((uintptr_t)out_vals % elem_size(dtype) || (uintptr_t)out_idx % 4) return ATK_INVALID_ARG;
    const Plan& pl = make_plan(values, dtype, rows, N, row_stride, K, Kprime, B, false,
                               workspace ? workspace_bytes : 0);
    if (pl.status) return pl.status;
    if (pl.route_exact && K > kExactMaxK) return ATK_UNSUPPORTED;
    if (pl.workspace > 0 && (!workspace || workspace_bytes < pl.workspace))
        return ATK_WORKSPACE_TOO_SMALL;
    if ((uintptr_t)workspace % 8) return ATK_INVALID_ARG;
    if (rows == 0) return ATK_OK;
    hipStream_t st = (hipStream_t)stream;
    const uint32_t flip = flip_mask(dtype, smallest);
    if (pl.route_exact)
        return exact_dispatch(values, dtype, rows, N, row_stride, K, out_vals, out_idx, workspace,
                              workspace_bytes, st, smallest);

    ApproxParams p = params_from(pl, values, rows, N, row_stride, K, Kprime, B);
    p.flip = flip;
    p.cert_flags = cert_flags;      // (only the packed-key variants of the fused route look at it)
    if (pl.slab_w > 0) {
        // slab path: the final K' keys of every bucket through the workspace, then stage 2
        p.mode = 3;
        p.slab_w = pl.slab_w;
        p.part_keys = (uint64_t*)workspace;
        p.run_len = pl.run_len;
        hipError_t e = pl.var->fn(p, pl.grid, pl.block, pl.lds, st);
        if (e != hipSuccess) return hip_fail(e);
        if (pl.run_len > 0) {
            RankFinishParams r{};
            r.runs = (const uint64_t*)workspace; r.values = values; r.row_stride = row_stride;
            r.rows = (int)rows; r.K = K; r.nruns = B / pl.slab_w;
            r.log_run = log2_of(pl.run_len);
            r.runs_per_wg = pl.rank_runs_per_wg;
            r.log_head = rank_log_head(K, r.nruns, r.log_run);
            r.flip = flip;
            r.out_vals = out_vals; r.out_idx = out_idx;
            e = launch_rank_finish(r, dtype, st);
            return e == hipSuccess ? ATK_OK : hip_fail(e);
        }
        FinishParams f{};
        f.part_keys = (const uint64_t*)workspace; f.values = values; f.row_stride = row_stride;
        f.rows = (int)rows; f.K = K; f.Kprime = Kprime; f.B = B; f.nseg = 1; f.Cpad = pl.Cpad;
        f.flip = flip;
        f.out_vals = out_vals; f.out_idx = out_idx;
        e = launch_finish(f, dtype, pl.var->KP, st);
        return e == hipSuccess ? ATK_OK : hip_fail(e);
    }
    if (pl.nseg > 1) {
        // split path: partial lists of every (row, segment) through the workspace
        p.mode = 2;
        p.nseg = pl.nseg; p.seg_steps = pl.seg_steps;
        p.part_keys = (uint64_t*)workspace;
        hipError_t e = pl.var->fn(p, pl.grid, pl.block, 0, st);
        if (e != hipSuccess) return hip_fail(e);
        FinishParams f{};
        f.part_keys = (const uint64_t*)workspace; f.values = values; f.row_stride = row_stride;
        f.rows = (int)rows; f.K = K; f.Kprime = Kprime; f.B = B; f.nseg = pl.nseg; f.Cpad = pl.Cpad;
        f.flip = flip;
        f.out_vals = out_vals; f.out_idx = out_idx;
        e = launch_finish(f, dtype, pl.var->KP, st);
        return e == hipSuccess ? ATK_OK : hip_fail(e);
    }
    if (pl.fused) {
        p.mode = 0;
        p.out_vals = out_vals; p.out_idx = out_idx;
        hipError_t e = pl.var->fn(p, pl.grid, pl.block, pl.lds, st);
        return e == hipSuccess ? ATK_OK : hip_fail(e);
    }
    if (pl.chunk_k > 0) {
        // every bucket chunk's K greatest [rows, nchunk, K] through the workspace, then exact Top-K
        const int64_t C = (int64_t)pl.nchunk * K;
        char* ws = (char*)workspace;
        int32_t* part_idx = (int32_t*)ws;
        void* part_vals = ws + (size_t)rows * C * 4;
        p.mode = 0;
        p.out_vals = part_vals; p.out_idx = part_idx;
        hipError_t e = pl.var->fn(p, pl.grid, pl.block, pl.lds, st);
        if (e != hipSuccess) return hip_fail(e);
        return run_exact(part_vals, part_idx, dtype, rows, C, C, K, out_vals, out_idx, st, values, row_stride, flip);
    }
    if (pl.run_len > 0) {
        // unfused, stage 2 by ranking: sorted runs of keys through the workspace
        p.mode = 4;
        p.run_len = pl.run_len;
        p.part_keys = (uint64_t*)workspace;
        hipError_t e = pl.var->fn(p, pl.grid, pl.block, pl.lds, st);
        if (e != hipSuccess) return hip_fail(e);
        RankFinishParams r{};
        r.runs = (const uint64_t*)workspace; r.values = values; r.row_stride = row_stride;
        r.rows = (int)rows; r.K = K; r.nruns = pl.nchunk * (pl.G / 64);
        r.log_run = log2_of(pl.run_len);
        r.log_head = rank_log_head(K, r.nruns, r.log_run);
        r.runs_per_wg = pl.rank_runs_per_wg;
        r.flip = flip;
        r.out_vals = out_vals; r.out_idx = out_idx;
        e = launch_rank_finish(r, dtype, st);
        return e == hipSuccess ? ATK_OK : hip_fail(e);
    }
    // unfused: survivors [rows, K', B] through the workspace, then exact Top-K over them
    const int64_t C = (int64_t)B * Kprime;
    char* ws = (char*)workspace;
    int32_t* surv_idx = (int32_t*)ws;                                  // 4-byte part first
    void* surv_vals = ws + (size_t)rows * C * 4;
    p.mode = 1;
    p.surv_vals = surv_vals; p.surv_idx = surv_idx;
    p.surv_aligned = ((uintptr_t)surv_vals % 16 == 0 && (uintptr_t)surv_idx % 16 == 0) ? 1 : 0;
    hipError_t e = pl.var->fn(p, pl.grid, pl.block, pl.lds, st);
    if (e != hipSuccess) return hip_fail(e);
    return run_exact(surv_vals, surv_idx, dtype, rows, C, C, K, out_vals, out_idx, st, values, row_stride, flip);
}

}  // namespace

extern "C" {

int atk_approx_topk(const void* values, int dtype, int64_t rows, int64_t N, int64_t row_stride,
                    int K, int Kprime, int B, void* out_vals, int32_t* out_idx,
                    void* workspace, size_t workspace_bytes, void* stream) {
    return approx_impl(values, dtype, rows, N, row_stride, K, Kprime, B, out_vals, out_idx, workspace,
                       workspace_bytes, stream, false);
}

int atk_approx_mink(const void* values, int dtype, int64_t rows, int64_t N, int64_t row_stride,
                    int K, int Kprime, int B, void* out_vals, int32_t* out_idx,
                    void* workspace, size_t workspace_bytes, void* stream) {
    return approx_impl(values, dtype, rows, N, row_stride, K, Kprime, B, out_vals, out_idx, workspace,
                       workspace_bytes, stream, true);
}

int atk_approx_topk_noalloc(const void* values, int dtype, int64_t rows, int64_t N, int64_t row_stride,
                            int K, int Kprime, int B, void* out_vals, int32_t* out_idx, void* stream) {
    // what the call would need as a workspace, given that at most the scratch array is on offer
    // (routes that only use a workspace to go faster fall back by themselves when it is too small)
    int rc = validate_common(values, dtype, rows, N, row_stride);
    if (rc) return rc;
    rc = validate_method(N, K, Kprime, B);
    if (rc) return rc;
    const Plan& pl = make_plan(values, kernel_dtype(dtype), rows, N, row_stride, K, Kprime, B, false,
                               kScratchBytes);
    if (pl.status) return pl.status;
    if (pl.workspace > kScratchBytes) return ATK_WORKSPACE_TOO_SMALL;   // survivors beyond the array
    void* ws = nullptr;
    if (pl.workspace > 0 && rows > 0) {
        hipError_t e;
        ws = scratch_on_current_device(&e);
        if (!ws) return hip_fail(e);
    }
    return atk_approx_topk(values, dtype, rows, N, row_stride, K, Kprime, B, out_vals, out_idx,
                           ws, ws ? kScratchBytes : 0, stream);
}

int atk_recall_params(int dtype, int64_t rows, int64_t N, int K, double recall_target, int* Kprime_out,
                      int* B_out, double* expected_recall_out) {
    if (kernel_dtype(dtype) < 0) return ATK_UNSUPPORTED;
    if (rows < 0) return ATK_INVALID_ARG;
    if (N <= 0 || N > kMaxN || K < 1 || K > N || !Kprime_out || !B_out) return ATK_INVALID_ARG;
    if (!(recall_target > 0.0) || recall_target > 1.0) return ATK_INVALID_ARG;
    options_from_env_once();
    // the answer is a pure function of the arguments and the options, and callers in a loop
    // repeat them (the sweep evaluates Theorem 1 a few hundred times): the last one is kept
    struct Slot { int dtype; int64_t rows, N; int K; double target; unsigned gen; int rc, kp, b; double r; };
    thread_local Slot last{-1, 0, 0, 0, 0.0, 0, 0, 0, 0, 0.0};
    const int kd = kernel_dtype(dtype);
    if (!(last.dtype == kd && last.rows == rows && last.N == N && last.K == K && last.target == recall_target &&
          last.gen == g_opt_generation)) {
        struct Ctx { int dtype; int64_t rows, N; int K; } ctx{kd, rows, N, K};
        // only configurations that atk_approx_topk runs are candidates
        auto runs = [](void* c, int kp, int64_t B) {
            const Ctx& x = *(const Ctx*)c;
            if (B > 0x7fffffff || validate_method(x.N, x.K, kp, (int)B)) return false;
            return make_plan(nullptr, x.dtype, x.rows, x.N, x.N, x.K, kp, (int)B, false).status == ATK_OK;
        };
        // ceilings below which stage 1 stays memory-bound on this chip: K' <= 4 for 32-bit elements,
        // K' <= 8 for 16-bit ones; buckets in multiples of a wavefront
        const int ceiling = elem_size(kd) == 2 ? 8 : 4;
        int kp = 0, b = 0;
        double r = 0.0;
        // On this chip the list length is what stage 1 pays for, and stage 2 is cheap while the
        // survivors are few against the row: the shortest lists for which some B within a
        // survivor budget reaches the target -- a sixteenth of the row, between 512 and 4096,
        // at most 1024 where that keeps 16-bit rows on the packed-key kernels -- and for that K'
        // the smallest sufficient power of two (doubled up to 1024 within the budget), else the
        // smallest sufficient divisor.  Measured
        // against the fewest-survivors rule: 256 x 2^20, K = 128, target 0.95: (1, 2048) 163 us
        // against (4, 64) 188 us; 4096 x 32768 bf16, K = 100: (1, 1024) 48 us against (4, 64) 102 us.
        int64_t budget = N / 16 < 512 ? 512 : (N / 16 > 4096 ? 4096 : N / 16);
        if (elem_size(kd) == 2 && N <= 65536 && budget > kWaveSortMaxKeys) budget = kWaveSortMaxKeys;
        for (int k = 1; k <= ceiling && k <= K && !kp; ++k) {
            int64_t first = 0, first_pow2 = 0;
            for (int64_t B = 64; B * k <= budget && B <= N / k; B += 64) {
                if (N % B || B * k < K || !runs(&ctx, k, B)) continue;
                if (first && (B & (B - 1))) continue;                  // after the first: powers of two only
                const double e = atk_expected_recall(N, B, K, k);
                if (e < recall_target) continue;
                if (!first) first = B;
                if ((B & (B - 1)) == 0) { first_pow2 = B; break; }
            }
            int64_t pick = first_pow2 ? first_pow2 : first;
            // (a power of two below 1024 leaves a lane single-element loads: doubled while the budget
            // allows -- 256 x 2^20, K = 128, target 0.99: (2, 1024) 162 us against (2, 512) 182 us)
            while (first_pow2 && pick < 1024 && 2 * pick * k <= budget && N % (2 * pick) == 0 &&
                   N / (2 * pick) >= k && runs(&ctx, k, 2 * pick))
                pick *= 2;
            if (pick) { kp = k; b = (int)pick; r = atk_expected_recall(N, pick, K, k); }
        }
        int rc = ATK_OK;
        if (!kp)        // nothing within the budget: the fewest survivors (Section 6.3's rule)
            rc = select_params_impl(N, K, recall_target, ceiling, 64, runs, &ctx, &kp, &b, &r);
        if (!rc && kp == K && b == 1 && K > kExactMaxK) rc = ATK_UNSUPPORTED;   // exact fallback out of range
        last = {kd, rows, N, K, recall_target, g_opt_generation, rc, kp, b, r};
    }
    if (last.rc) return last.rc;
    *Kprime_out = last.kp;
    *B_out = last.b;
    if (expected_recall_out) *expected_recall_out = last.r;
    return ATK_OK;
}

static int exact_impl(const void* values, int dtype, int64_t rows, int64_t N, int64_t row_stride, int K,
                      void* out_vals, int32_t* out_idx, void* workspace, size_t workspace_bytes,
                      void* stream, bool smallest);

static int recall_impl(const void* values, int dtype, int64_t rows, int64_t N, int64_t row_stride, int K,
                       double recall_target, void* out_vals, int32_t* out_idx, void* workspace,
                       size_t workspace_bytes, void* stream, int* Kprime_used, int* B_used, bool smallest) {
    int kp = 0, b = 0;
    int rc = atk_recall_params(dtype, rows, N, K, recall_target, &kp, &b, nullptr);
    if (rc) return rc;
    if (Kprime_used) *Kprime_used = kp;
    if (B_used) *B_used = b;
    if (kp == K && b == 1)   // nothing approximate reaches the target: the exact result
        return exact_impl(values, dtype, rows, N, row_stride, K, out_vals, out_idx, workspace, workspace_bytes,
                          stream, smallest);
    return approx_impl(values, dtype, rows, N, row_stride, K, kp, b, out_vals, out_idx, workspace,
                       workspace_bytes, stream, smallest);
}

int atk_approx_topk_recall(const void* values, int dtype, int64_t rows, int64_t N,
                           int64_t row_stride, int K, double recall_target, void* out_vals,
                           int32_t* out_idx, void* workspace, size_t workspace_bytes,
                           void* stream, int* Kprime_used, int* B_used) {
    return recall_impl(values, dtype, rows, N, row_stride, K, recall_target, out_vals, out_idx, workspace,
                       workspace_bytes, stream, Kprime_used, B_used, false);
}

int atk_approx_mink_recall(const void* values, int dtype, int64_t rows, int64_t N,
                           int64_t row_stride, int K, double recall_target, void* out_vals,
                           int32_t* out_idx, void* workspace, size_t workspace_bytes,
                           void* stream, int* Kprime_used, int* B_used) {
    return recall_impl(values, dtype, rows, N, row_stride, K, recall_target, out_vals, out_idx, workspace,
                       workspace_bytes, stream, Kprime_used, B_used, true);
}

static int exact_impl(const void* values, int dtype, int64_t rows, int64_t N, int64_t row_stride, int K,
                      void* out_vals, int32_t* out_idx, void* workspace, size_t workspace_bytes,
                      void* stream, bool smallest) {
    int rc = validate_common(values, dtype, rows, N, row_stride);
    if (rc) return rc;
    dtype = kernel_dtype(dtype);       // fp16 -> the bf16 kernels
    if (K < 1 || (int64_t)K > N) return ATK_INVALID_ARG;
    if (rows > 0 && (!out_vals || !out_idx)) return ATK_INVALID_ARG;
    if ((uintptr_t)out_vals % elem_size(dtype) || (uintptr_t)out_idx % 4) return ATK_INVALID_ARG;
    if (K > kExactMaxK) return ATK_UNSUPPORTED;
    if (rows == 0) return ATK_OK;
    return exact_dispatch(values, dtype, rows, N, row_stride, K, out_vals, out_idx, workspace,
                          workspace_bytes, (hipStream_t)stream, smallest);
}

int atk_topk(const void* values, int dtype, int64_t rows, int64_t N, int64_t row_stride, int K,
             void* out_vals, int32_t* out_idx, void* workspace, size_t workspace_bytes,
             void* stream) {
    return exact_impl(values, dtype, rows, N, row_stride, K, out_vals, out_idx, workspace, workspace_bytes,
                      stream, false);
}

int atk_mink(const void* values, int dtype, int64_t rows, int64_t N, int64_t row_stride, int K,
             void* out_vals, int32_t* out_idx, void* workspace, size_t workspace_bytes, void* stream) {
    return exact_impl(values, dtype, rows, N, row_stride, K, out_vals, out_idx, workspace, workspace_bytes,
                      stream, true);
}

int atk_describe_topk_plan(int dtype, int64_t rows, int64_t N, int K, char* buf, size_t buflen) {
    if (!buf || buflen == 0) return ATK_INVALID_ARG;
    buf[0] = 0;
    dtype = kernel_dtype(dtype);
    if (dtype < 0 || rows < 0 || N <= 0 || N > kMaxN || K < 1 || K > N) return ATK_INVALID_ARG;
    if (K > kExactMaxK) return ATK_UNSUPPORTED;
    options_from_env_once();
    const CertPlan cp = certified_params(dtype, rows, N, K);
    if (cp.B) {
        const Plan& pl = make_plan(nullptr, dtype, rows, N, N, K, cp.Kprime, cp.B, false);
        if (pl.status == ATK_OK && !pl.route_exact && cp.Kprime >= K) {
            std::snprintf(buf, buflen, "two-stage B=%d K'=K=%d workspace=%zu", cp.B, cp.Kprime, pl.workspace);
            return ATK_OK;
        }
        if (pl.status == ATK_OK && !pl.route_exact) {
            std::snprintf(buf, buflen, "certified B=%d K'=%d workspace=%zu (else radix threads=%d)", cp.B, cp.Kprime,
                          certified_lists_bytes(rows) + pl.workspace, exact_threads(N));
            return ATK_OK;
        }
    }
    std::snprintf(buf, buflen, "radix threads=%d", exact_threads(N));
    return ATK_OK;
}

int atk_approx_topk_stage1(const void* values, int dtype, int64_t rows, int64_t N,
                           int64_t row_stride, int Kprime, int B, void* surv_vals,
                           int32_t* surv_idx, void* stream) {
    int rc = validate_common(values, dtype, rows, N, row_stride);
    if (rc) return rc;
    dtype = kernel_dtype(dtype);       // fp16 -> the bf16 kernels
    // stage 1 has no K of its own: any K in [K', B*K'] makes the same survivors
    rc = validate_method(N, Kprime, Kprime, B);
    if (rc) return rc;
    if (rows > 0 && (!surv_vals || !surv_idx)) return ATK_INVALID_ARG;
    if ((uintptr_t)surv_vals % elem_size(dtype) || (uintptr_t)surv_idx % 4) return ATK_INVALID_ARG;
    const Plan& pl = make_plan(values, dtype, rows, N, row_stride, Kprime, Kprime, B, true);
    if (pl.status) return pl.status;
    if (rows == 0) return ATK_OK;
    ApproxParams p = params_from(pl, values, rows, N, row_stride, Kprime, Kprime, B);
    p.mode = 1;
    p.surv_vals = surv_vals; p.surv_idx = surv_idx;
    p.surv_aligned = ((uintptr_t)surv_vals % 16 == 0 && (uintptr_t)surv_idx % 16 == 0) ? 1 : 0;
    hipError_t e = pl.var->fn(p, pl.grid, pl.block, pl.lds, (hipStream_t)stream);
    return e == hipSuccess ? ATK_OK : hip_fail(e);
}

size_t atk_workspace_bytes(int op, int dtype, int64_t rows, int64_t N, int K, int Kprime, int B) {
    dtype = kernel_dtype(dtype);
    if (dtype < 0) return SIZE_MAX;
    if (rows < 0 || N <= 0 || N > kMaxN) return SIZE_MAX;
    if (op == ATK_OP_TOPK) {
        if (K < 1 || K > N) return SIZE_MAX;
        options_from_env_once();
        const CertPlan cp = certified_params(dtype, rows, N, K);
        if (!cp.B) return 0;
        const Plan& pl = make_plan(nullptr, dtype, rows, N, N, K, cp.Kprime, cp.B, false);
        if (pl.status != ATK_OK || pl.route_exact) return 0;
        return cp.Kprime >= K ? pl.workspace : certified_lists_bytes(rows) + pl.workspace;
    }
    if (op == ATK_OP_STAGE1) return validate_method(N, Kprime, Kprime, B) ? SIZE_MAX : 0;
    if (op != ATK_OP_APPROX_TOPK) return SIZE_MAX;
    if (validate_method(N, K, Kprime, B)) return SIZE_MAX;
    // alignment of the real buffers is not known here; assume the allocator's (>= 16 bytes)
    const Plan& pl = make_plan(nullptr, dtype, rows, N, N, K, Kprime, B, false);
    if (pl.status) return SIZE_MAX;
    // K' = K beyond the list lengths: the exact Top-K, which is faster with its own workspace
    if (pl.route_exact) return atk_workspace_bytes(ATK_OP_TOPK, dtype, rows, N, K, 0, 0);
    return pl.workspace;
}

// ---- matmul-fused path (Section 7.3): entry points ---------------------------------------------
size_t atk_mips_workspace_bytes(int dtype, int64_t Q, int64_t N, int64_t D, int K, int Kprime, int B) {
    MipsPlan pl = make_mips_plan(dtype, Q, N, D, K, Kprime, B);
    return pl.status ? SIZE_MAX : pl.workspace;
}

int atk_mips_approx_topk(const void* queries, const void* database, int dtype, int64_t Q, int64_t N,
                         int64_t D, int K, int Kprime, int B, float* out_vals, int32_t* out_idx,
                         void* workspace, size_t workspace_bytes, void* stream) {
    MipsPlan pl = make_mips_plan(dtype, Q, N, D, K, Kprime, B);
    if (pl.status) return pl.status;
    if (Q == 0) return ATK_OK;
    if (!queries || !database || !out_vals || !out_idx) return ATK_INVALID_ARG;
    if ((uintptr_t)queries % 16 || (uintptr_t)database % 16 || (uintptr_t)out_vals % 4 ||
        (uintptr_t)out_idx % 4)
        return ATK_INVALID_ARG;
    if (!workspace || workspace_bytes < pl.workspace) return ATK_WORKSPACE_TOO_SMALL;
    if ((uintptr_t)workspace % 8) return ATK_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;

    MipsParams p{};
    p.queries = (const uint16_t*)queries; p.database = (const uint16_t*)database;
    p.f16 = dtype == ATK_F16;
    p.Q = (int)Q; p.N = (int)N; p.D = (int)D; p.Kprime = Kprime; p.B = B;
    p.nsteps = (int)(N / B); p.nseg = pl.nseg; p.seg_steps = pl.seg_steps;
    p.nslab = pl.nslab; p.nqt = pl.nqt;
    p.part_keys = (uint64_t*)workspace;
    hipError_t e = launch_mips_stage1(p, pl.KP, st);
    if (e != hipSuccess) return hip_fail(e);

    FinishParams f{};
    f.part_keys = (const uint64_t*)workspace; f.values = nullptr; f.row_stride = 0;
    f.rows = (int)Q; f.K = K; f.Kprime = Kprime; f.B = B; f.nseg = pl.nseg; f.Cpad = pl.Cpad;
    f.out_vals = out_vals; f.out_idx = out_idx;
    e = launch_finish(f, kFinishScores, pl.KP, st);
    return e == hipSuccess ? ATK_OK : hip_fail(e);
}

int atk_mips_approx_topk_recall(const void* queries, const void* database, int dtype, int64_t Q,
                                int64_t N, int64_t D, int K, double recall_target, float* out_vals,
                                int32_t* out_idx, void* workspace, size_t workspace_bytes,
                                void* stream, int* Kprime_used, int* B_used) {
    // (the sweep costs a few hundred microseconds of host time: the last answer is kept)
    struct Slot { int64_t N; int K; double target; int rc, kp, b; };
    thread_local Slot last{0, 0, 0.0, 0, 0, 0};
    if (!(last.N == N && last.K == K && last.target == recall_target && N > 0)) {
        int kp0 = 0, b0 = 0;
        const int rc0 = atk_mips_select_params(N, K, recall_target, &kp0, &b0, nullptr);
        last = {N, K, recall_target, rc0, kp0, b0};
    }
    if (last.rc) return last.rc;
    const int kp = last.kp, b = last.b;
    if (Kprime_used) *Kprime_used = kp;
    if (B_used) *B_used = b;
    return atk_mips_approx_topk(queries, database, dtype, Q, N, D, K, kp, b, out_vals, out_idx,
                                workspace, workspace_bytes, stream);
}

int atk_mips_describe_plan(int dtype, int64_t Q, int64_t N, int64_t D, int K, int Kprime, int B,
                           char* buf, size_t buflen) {
    if (!buf || buflen == 0) return ATK_INVALID_ARG;
    buf[0] = 0;
    MipsPlan pl = make_mips_plan(dtype, Q, N, D, K, Kprime, B);
    if (pl.status) return pl.status;
    std::snprintf(buf, buflen,
                  "mfma32x32x16 KP=%d slabs=%d query_tiles=%d segments=%d steps_per_segment=%d "
                  "grid=%d block=256 cand=%d workspace=%zu",
                  pl.KP, pl.nslab, pl.nqt, pl.nseg, pl.seg_steps, pl.nslab * pl.nqt * pl.nseg,
                  pl.Cpad, pl.workspace);
    return ATK_OK;
}

int atk_describe_plan(int dtype, int64_t rows, int64_t N, int K, int Kprime, int B, char* buf,
                      size_t buflen) {
    if (!buf || buflen == 0) return ATK_INVALID_ARG;
    buf[0] = 0;
    dtype = kernel_dtype(dtype);
    if (dtype < 0) return ATK_UNSUPPORTED;
    if (rows < 0 || N <= 0 || N > kMaxN) return ATK_INVALID_ARG;
    int rc = validate_method(N, K, Kprime, B);
    if (rc) return rc;
    const Plan& pl = make_plan(nullptr, dtype, rows, N, N, K, Kprime, B, false);
    if (pl.status) return pl.status;
    if (pl.route_exact) {
        std::snprintf(buf, buflen, "exact(K'=K) threads=%d", exact_threads(N));
        return ATK_OK;
    }
    std::snprintf(buf, buflen,
                  "%s%s KP=%d V=%d R=%d lanes_per_row=%d rows_per_wg=%d block=%d grid=%dx%d step=%d "
                  "steps=%d owners=%d seg=%d cand=%d tail=%d lds=%zu workspace=%zu",
                  pl.slab_w > 0 ? "slab" : pl.nseg > 1 ? "split" : (pl.fused ? "fused" : (pl.chunk_k > 0 ? "chunked" : "unfused")),
                  pl.var->packed() ? " packed" : (pl.var->rep == 2 ? " batched" : (pl.var->rep == 4 ? " deferred" : (pl.var->rep == 5 ? " lists32" : ""))), pl.var->KP, pl.var->V,
                  pl.var->R, pl.G, pl.rows_per_wg, pl.block, pl.grid,
                  pl.slab_w > 0 ? B / pl.slab_w : (pl.nseg > 1 ? pl.nseg : pl.nchunk), pl.S, pl.nsteps,
                  pl.owners, pl.seg, pl.Cpad, pl.tail, pl.lds, pl.workspace);
    if (pl.run_len > 0) {
        // second launch: workgroups per row x keys each of them places
        const size_t n = std::strlen(buf);
        const int nruns = pl.slab_w > 0 ? B / pl.slab_w : pl.nchunk * (pl.G / 64);
        std::snprintf(buf + n, buflen - n, " rank_finish=%dx%d",
                      (nruns + pl.rank_runs_per_wg - 1) / pl.rank_runs_per_wg, pl.rank_runs_per_wg * pl.run_len);
    }
    return ATK_OK;
}

int atk_set_option(const char* name, int value) {
    if (!name) return ATK_INVALID_ARG;
    options_from_env_once();
    const Options defaults;
    struct Entry { const char* name; int Options::*field; };
    static const Entry entries[] = {
        {"lanes_per_row", &Options::lanes_per_row}, {"segments", &Options::segments},
        {"slab", &Options::slab}, {"rank_finish", &Options::rank_finish}, {"slab_width", &Options::slab_width}, {"rank_wgs", &Options::rank_wgs}, {"defer", &Options::defer}, {"slab_owners", &Options::slab_owners}, {"packed", &Options::packed}, {"subwave", &Options::subwave},
        {"batch_min_kp", &Options::batch_min_kp}, {"mips_segments", &Options::mips_segments},
        {"unfused", &Options::unfused}, {"onepass", &Options::onepass}, {"chunked", &Options::chunked},
        {"exact_threads", &Options::exact_threads}, {"certified", &Options::certified}, {"reg_rows", &Options::reg_rows},
    };
    for (const Entry& e : entries) {
        if (std::strcmp(name, e.name) != 0) continue;
        int v = value < 0 ? defaults.*(e.field) : value;
        if (e.field == &Options::lanes_per_row && (v > kMaxLanes || (v & (v - 1)))) return ATK_INVALID_ARG;
        if (e.field == &Options::slab_owners && (v > 32 || (v & (v - 1)))) return ATK_INVALID_ARG;
        if (e.field == &Options::slab_width && v != 0 && (v < 32 || v > 1024 || (v & (v - 1)))) return ATK_INVALID_ARG;
        if (e.field == &Options::exact_threads && v != 0 && (v < 64 || v > 1024 || (v & (v - 1)))) return ATK_INVALID_ARG;
        g_opt.*(e.field) = v;
        ++g_opt_generation;
        return ATK_OK;
    }
    return ATK_INVALID_ARG;
}

const char* atk_status_string(int status) {
    switch (status) {
        case ATK_OK: return "ATK_OK";
        case ATK_INVALID_ARG: return "ATK_INVALID_ARG";
        case ATK_UNSUPPORTED: return "ATK_UNSUPPORTED";
        case ATK_WORKSPACE_TOO_SMALL: return "ATK_WORKSPACE_TOO_SMALL";
        case ATK_HIP_ERROR: return "ATK_HIP_ERROR";
        default: return "ATK_UNKNOWN_STATUS";
    }
}

const char* atk_last_hip_error(void) { return g_last_hip_error.c_str(); }

const char* atk_version(void) { return "0.1.0"; }

}  // extern "C"
