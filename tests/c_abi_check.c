/* A C translation unit that uses the library through include/pk.h alone: host-side calls only (no GPU needed). */
#include <stdio.h>
#include <string.h>

#include "pk.h"

int main(void) {
    pk_plan plan;
    if (pk_version() < 1) return 1;
    if (pk_gemm_rs_plan(8, 8192, 8192, 28672, PK_BF16, &plan) != PK_OK) return 2;
    if (plan.tile_m != 256 || plan.tile_n != 256 || plan.flags_per_slot != 4 * 32 || plan.local_k != 3584) return 3;
    if (pk_ag_gemm_plan(8, 8192, 28672, 8192, PK_BF16, &plan) != PK_OK || plan.local_n != 3584) return 4;
    if (plan.workspace_bytes < PK_WS_FLAG_BYTES + 256 * 256 * 4) return 9;
    if (pk_gemm_ar_plan(8, 8192, 8192, 28672, PK_BF16, &plan) != PK_OK || plan.ar_flags_per_slot != (1024 / PK_AR_ROWS) * 32)
        return 5;
    if (pk_gemm_rs_plan(3, 256, 256, 512, PK_BF16, &plan) != PK_ERR_SHAPE) return 6;
    if (pk_gemm_rs(2, 5, 256, 256, 512, PK_BF16, (void*)0x1000, (void*)0x2000, NULL, NULL, (void*)0x3000, (void*)0x4000,
                   (uint32_t*)0x5000, (uint32_t*)0x6000, 1u, (void*)0x7000, PK_PHASE_ALL, 0, PK_PARTIAL_F32, PK_B_ROW_MAJOR, NULL, 0,
                   (uint32_t*)0x8000, 0, NULL) != PK_ERR_RANK)
        return 7;
    if (strcmp(pk_status_str(PK_OK), pk_status_str(PK_ERR_SHAPE)) == 0) return 8;
    printf("c abi ok, version %d\n", pk_version());
    return 0;
}
