/* A plain C99 caller of include/lba.h (host-only entry points: no GPU needed).  Built and run by
 * tests/test_abi_cpu.py with -std=c99 -Wall -Wextra -Werror against paper_2401_14110_amd/liblba_hip.so. */
#include <stdio.h>
#include <string.h>

#include "lba.h"

int main(void) {
    lba_qfmt qprod = {5, 7, 15, LBA_ROUND_FLOOR}, qacc = {4, 7, 7, LBA_ROUND_FLOOR};
    lba_plan_info info;
    memset(&info, 0, sizeof info);
    if (lba_mask_words(4, 5, 33) != 40 || lba_mask_words_level2(4, 5, 513) != 40) return 1;
    if (strcmp(lba_strerror(LBA_OK), "ok") != 0 || lba_strerror(12345) == NULL) return 2;
    if (lba_plan_query(100352, 64, 576, qprod, qacc, LBA_ORDER_SEQ, 0, &info) != LBA_OK) return 3;
    if (info.kernel != 0 || info.tile_m * info.grid_x < 100352) return 4;
    /* validation comes before any device work: a bad format with bogus pointers must come back clean */
    qacc.man_bits = 24;
    if (lba_gemm((const uint8_t*)0x1000, (const uint8_t*)0x1000, (float*)0x1000, 8, 8, 8, qprod, qacc,
                 LBA_ORDER_SEQ, NULL) != LBA_ERR_FORMAT) return 5;
    qacc.man_bits = 7;
    if (lba_gemm_bwd_chunked(NULL, NULL, NULL, NULL, NULL, NULL, NULL, 0, 8, 8, qprod, qacc, NULL) != LBA_OK) return 6;
    if (lba_gemm_bwd((const uint8_t*)0x1000, (const uint8_t*)0x1000, NULL, (uint32_t*)0x1000, NULL, 8, 8, 8, qprod, qacc,
                     LBA_ORDER_CHUNK16, NULL) != LBA_ERR_UNSUPPORTED) return 7;
    printf("c caller ok: %d x %d tiles, %d workgroups\n", info.tile_m, info.tile_n, info.grid_x * info.grid_y);
    return 0;
}
