/* Plain C99 translation unit that includes the public header and calls the
 * argument-validation paths of the C ABI: checks that ud.h is a valid C header
 * (no C++, no HIP types) and that the library links from C.  No GPU needed. */
#include <stdio.h>
#include <string.h>

#include "ud.h"

int main(void)
{
    ud_table *t = NULL;
    ud_tuning plan;
    int64_t bad = 0;
    if (ud_alloc_table(0, 4, UD_F32, UD_TABLE_COHERENT, &t) != UD_ERR_INVALID_ARG)
        return 1;
    if (ud_gather(NULL, 4, 4, UD_F32, NULL, UD_I64, 0, NULL, NULL) != UD_OK)
        return 2;
    if (ud_gather((const void *)0x1000, 4, 4, UD_F32, NULL, UD_I64, 1, (void *)0x2000, NULL) != UD_ERR_INVALID_ARG)
        return 3;
    if (ud_scatter((void *)0x1000, 4, 4, UD_F16_TO_F32, (const void *)0x3000, UD_I64, 1, (const void *)0x2000, NULL) != UD_ERR_INVALID_ARG)
        return 4;
    if (ud_gather_plan((const void *)0x10000, 602, UD_F32, &plan) != UD_OK || plan.lanes_per_row != 64 || plan.chunks_per_lane != 3)
        return 5;
    if (strcmp(ud_status_str(UD_ERR_INDEX_OUT_OF_RANGE), "UD_ERR_INDEX_OUT_OF_RANGE") != 0)
        return 6;
    if (ud_free_table(NULL) != UD_OK || ud_cache_free(NULL) != UD_OK)
        return 7;
    if (ud_gather_noalloc(NULL, 4, 4, UD_F32, NULL, UD_I64, 0, NULL, NULL) != UD_OK)
        return 8;
    if (ud_gather_noalloc((const void *)0x1000, 4, 4, UD_F32, NULL, UD_I64, 1, (void *)0x2000, NULL) != UD_ERR_INVALID_ARG)
        return 9;
    if (strlen(ud_build_id()) == 0)
        return 10;
    (void)bad;
    printf("c abi ok\n");
    return 0;
}
