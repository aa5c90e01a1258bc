/* Plain C11 user of the C ABI: builds a host-only plan of a small matrix, reads its statistics,
 * decodes it back and compares with the input.  Exit status 0 = all checks passed. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "rsh_spmm.h"

#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "check failed, line %d: %s\n", __LINE__, #cond); return 1; } } while (0)

int main(void) {
    enum { ROWS = 40, COLS = 50 };
    int64_t row_ptr[ROWS + 1];
    int32_t col_idx[ROWS * 6];
    uint16_t val[ROWS * 6];
    int64_t nnz = 0;
    for (int i = 0; i < ROWS; ++i) {           /* a band of 1..6 entries per row, row 7 empty */
        row_ptr[i] = nnz;
        int len = i == 7 ? 0 : 1 + i % 6;
        for (int j = 0; j < len; ++j) {
            col_idx[nnz] = (int32_t)((i + 2 * j) % COLS);
            val[nnz] = (uint16_t)(0x3c00 + i + j);   /* binary16 values a little above 1.0 */
            ++nnz;
        }
        /* columns must ascend inside a row */
        for (int64_t a = row_ptr[i] + 1; a < nnz; ++a)
            for (int64_t b = a; b > row_ptr[i] && col_idx[b - 1] > col_idx[b]; --b) {
                int32_t tc = col_idx[b]; col_idx[b] = col_idx[b - 1]; col_idx[b - 1] = tc;
                uint16_t tv = val[b]; val[b] = val[b - 1]; val[b - 1] = tv;
            }
    }
    row_ptr[ROWS] = nnz;

    rsh_csr_t csr = {ROWS, COLS, nnz, row_ptr, col_idx, val};
    rsh_plan_opts_t opts;
    CHECK(rsh_plan_opts_default(&opts) == RSH_OK);
    opts.upload = 0;                            /* no GPU needed */
    opts.threads = 1;
    rsh_plan_t *plan = NULL;
    CHECK(rsh_plan_create(&csr, 32, &opts, &plan) == RSH_OK && plan != NULL);

    rsh_plan_stats_t st;
    CHECK(rsh_plan_stats(plan, &st) == RSH_OK);
    CHECK(st.nnz_tile + st.nnz_irregular == nnz);

    int64_t rp2[ROWS + 1];
    int32_t ci2[ROWS * 6];
    uint16_t v2[ROWS * 6];
    uint8_t path[ROWS * 6];
    CHECK(rsh_plan_decode(plan, rp2, ci2, v2, path) == RSH_OK);
    CHECK(memcmp(rp2, row_ptr, sizeof row_ptr) == 0);
    CHECK(memcmp(ci2, col_idx, (size_t)nnz * sizeof(int32_t)) == 0);
    CHECK(memcmp(v2, val, (size_t)nnz * sizeof(uint16_t)) == 0);

    CHECK(rsh_spmm(plan, (const void *)16, (void *)16, NULL) == RSH_ERR_NOT_UPLOADED);
    CHECK(rsh_plan_create(&csr, 0, &opts, &plan) == RSH_ERR_UNSUPPORTED_N);
    int32_t a = 0, b = 0;
    CHECK(rsh_struct_sizes(&a, &b) == RSH_OK && a == (int32_t)sizeof(rsh_plan_opts_t) && b == (int32_t)sizeof(rsh_plan_stats_t));
    CHECK(strlen(rsh_status_string(RSH_ERR_INVALID_CSR)) > 0);
    printf("c abi ok: %lld entries, %lld in fragments, %lld irregular\n", (long long)nnz, (long long)st.nnz_tile,
           (long long)st.nnz_irregular);
    return 0;
}
