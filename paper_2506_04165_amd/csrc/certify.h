// Exactness certificate and repair for a two-stage result (see certify.hip): turns the output of
// the approximate path into the exact Top-K.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace atk {

struct CertifyParams {
    const void* values;       // [rows, row_stride] elements, the rows the result was taken from
    int64_t row_stride;
    int rows, N, K, Kprime, B;
    uint32_t flip;            // order-reversing mask of the call (0: Top-K), see ApproxParams
    int cap;                  // LDS key buffer (keys): a power of two >= 2K, at least 1024
    int max_scan;             // most elements a workgroup re-reads from the row before it gives up
    int rows_per_wg;          // 1, or kCertifyRowsPerWg (many short rows with few buckets: every wavefront
                              // of a workgroup certifies four rows by itself)
    void* out_vals;           // [rows, K] in: the two-stage result; out: the exact one
    int32_t* out_idx;
    int32_t* hard_rows;       // [rows] out: 1 where the row has to be done by the exact kernel, else 0
    const int32_t* open_rows; // optional [rows]: 0 where the two-stage launch has already certified the row
                              // (ApproxParams::cert_flags), which is then not looked at
};

constexpr int kCertifyMaxB = 4096;       // buckets the LDS counters hold
constexpr int kCertifyRowsPerWg = 4;
constexpr int kCertifyMaxFlagged = 128;  // buckets a workgroup repairs before it gives up

size_t certify_lds_bytes(const CertifyParams& p);
hipError_t launch_certify(const CertifyParams& p, int dtype, hipStream_t stream);

}  // namespace atk
