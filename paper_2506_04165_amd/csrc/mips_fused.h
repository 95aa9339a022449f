// Matmul-fused stage 1 (Section 7.3; appendix "Matmul-fused implementation"): the score matrix
// queries x database^T is produced tile by tile on the matrix cores and consumed by the K'-list
// update in the same registers; it never reaches memory.  See mips_fused.hip.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace atk {

struct MipsParams {
    const uint16_t* queries;    // [Q, D] bf16 or fp16, vectors contiguous
    const uint16_t* database;   // [N, D] same type, vectors contiguous
    int f16;                    // 1: the vectors are IEEE binary16, 0: bfloat16
    int Q, N, D, Kprime, B;
    int nsteps;                 // N / B: elements per bucket
    int nseg;                   // parts the element range of every bucket is cut into
    int seg_steps;              // steps per part (the last one may be shorter)
    int nslab;                  // B / 32: bucket slabs
    int nqt;                    // query tiles: ceil(Q / (128 * sub-tiles per wavefront))
    uint64_t* part_keys;        // [Q, nseg, K', B] keys, 0 = empty entry
};

constexpr int kMipsSlab = 32;        // buckets per workgroup
constexpr int kMipsQueryTile = 128;  // queries per workgroup and sub-tile (4 wavefronts x 32)

// 32-query sub-tiles a wavefront computes per step for lists of length KP and dimension D
// (p.nqt must be ceil(Q / (kMipsQueryTile * this))): two while the registers allow it
constexpr int mips_subtiles(int KP, int D) { return (KP == 1 && D <= 128) ? 2 : 1; }

// KP: compiled list length (1 to 4, = Kprime); D one of 64, 128, 256.
hipError_t launch_mips_stage1(const MipsParams& p, int KP, hipStream_t stream);

}  // namespace atk
