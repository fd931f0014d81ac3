/* Plain-C (C99) user of the library: checks that include/mfreduce.h compiles as C,
 * that the shared library links, and that argument errors come back as status
 * codes without touching a GPU.  Built and run by tests/test_host_boundary.py. */
#include <stdio.h>
#include <string.h>

#include "mfreduce.h"

int main(void)
{
    int block = 0, R = 0, grid = -7;
    unsigned long long plan[7];
    mfr_tuning t;
    memset(&t, 0, sizeof t);
    if (mfr_version() < 100) return 1;
    if (strcmp(mfr_strerror(MFR_OK), "success") != 0) return 2;
    if (mfr_get_default_tuning(&block, &R, &grid) != MFR_OK || block < 64 || R < 1 || grid != MFR_GRID_AUTO) return 3;
    if (mfr_sum_f16((const mfr_half *)0, 5, (float *)4096, (hipStream_t)0) != MFR_ERR_INVALID_ARG) return 4;
    if (mfr_sum_f16((const mfr_half *)4096, 5, (float *)0, (hipStream_t)0) != MFR_ERR_INVALID_ARG) return 5;
    t.block_threads = 100;
    if (mfr_sum_f16_ex((const mfr_half *)4096, 5, (float *)4096, &t, (hipStream_t)0) != MFR_ERR_INVALID_ARG) return 6;
    t.block_threads = 256;
    t.chain_R = 4;
    if (mfr_plan_for(100003, 4096 + 6, &t, plan) != MFR_OK || plan[0] != 3) return 7;
    if (mfr_plan_ex(100003, 4096 + 8, MFR_DTYPE_F32, &t, plan) != MFR_OK || plan[0] != 2) return 8;
    if (mfr_sum_f16_recurrence((const mfr_half *)4096, 5, (float *)4096, 0, (hipStream_t)0) != MFR_ERR_INVALID_ARG) return 9;
    if (mfr_sum_f16_f64((const mfr_half *)4096, 5, (double *)4100, (hipStream_t)0) != MFR_ERR_INVALID_ARG) return 10;
    if (mfr_sum_rows_ex((const void *)4096, MFR_DTYPE_F16, 4, 100, 99, (float *)4096, (const mfr_tuning *)0,
                        (hipStream_t)0) != MFR_ERR_INVALID_ARG) return 11;
    printf("c abi ok, version %d\n", mfr_version());
    return 0;
}
