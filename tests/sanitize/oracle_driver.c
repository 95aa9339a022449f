/*
 * Driver for running the C oracle under AddressSanitizer and UndefinedBehaviorSanitizer.
 * Built by tests/test_sanitizers.py together with oracle/atk_oracle.c (both with
 * -fsanitize=address,undefined) and fed requests on stdin; results go to stdout as raw bytes so
 * that the test can compare them with what the ordinary build of the oracle returns.
 *
 * Request: nine int64 words  op dtype rows N row_stride K Kprime B D,  then the input bytes.
 *   op 0  approx_topk   input values[rows, row_stride]          -> vals[rows,K], idx[rows,K]
 *   op 1  topk          same                                     -> vals[rows,K], idx[rows,K]
 *   op 2  stage1        same                                     -> vals[rows,K',B], idx[rows,K',B]
 *   op 3  mips          queries[rows, D] then database[N, D]     -> scores[rows,K], idx[rows,K]
 * Reply: one int64 status, then (status 0 only) the two output arrays.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int atk_oracle_stage1(const void *, int, int64_t, int64_t, int64_t, int64_t, int64_t, void *, int32_t *);
int atk_oracle_approx_topk(const void *, int, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, void *, int32_t *);
int atk_oracle_topk(const void *, int, int64_t, int64_t, int64_t, int64_t, void *, int32_t *);
int atk_oracle_mips_approx_topk(const uint16_t *, const uint16_t *, int, int64_t, int64_t, int64_t, int64_t,
                                int64_t, int64_t, float *, int32_t *);

static void *read_exact(size_t n)
{
    /* exactly n bytes, so that the sanitizer sees any access one element past the end */
    void *p = malloc(n ? n : 1);
    if (!p || fread(p, 1, n, stdin) != n) { fprintf(stderr, "driver: short read\n"); exit(3); }
    return p;
}

int main(void)
{
    int64_t h[9];
    while (fread(h, sizeof(int64_t), 9, stdin) == 9) {
        const int64_t op = h[0], dtype = h[1], rows = h[2], N = h[3], stride = h[4], K = h[5],
                      Kp = h[6], B = h[7], D = h[8];
        const size_t es = (dtype == 1 || dtype == 2) ? 2 : 4;
        int64_t status;
        size_t nout = (size_t)rows * (size_t)(op == 2 ? Kp * B : K);
        void *ov = malloc((nout ? nout : 1) * 4);
        int32_t *oi = malloc((nout ? nout : 1) * 4);
        size_t out_es = es;
        if (op == 3) {
            uint16_t *q = read_exact((size_t)rows * D * 2), *d = read_exact((size_t)N * D * 2);
            status = atk_oracle_mips_approx_topk(q, d, (int)dtype, rows, N, D, K, Kp, B, ov, oi);
            out_es = 4;
            free(q); free(d);
        } else {
            /* the last row ends at N, not at row_stride: no byte beyond it is allocated */
            void *x = read_exact(rows ? ((size_t)(rows - 1) * stride + N) * es : 0);
            if (op == 0) status = atk_oracle_approx_topk(x, (int)dtype, rows, N, stride, K, Kp, B, ov, oi);
            else if (op == 1) status = atk_oracle_topk(x, (int)dtype, rows, N, stride, K, ov, oi);
            else status = atk_oracle_stage1(x, (int)dtype, rows, N, stride, Kp, B, ov, oi);
            free(x);
        }
        fwrite(&status, sizeof status, 1, stdout);
        if (status == 0) {
            fwrite(ov, out_es, nout, stdout);
            fwrite(oi, 4, nout, stdout);
        }
        free(ov); free(oi);
    }
    return 0;
}
