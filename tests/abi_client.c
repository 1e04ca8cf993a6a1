/* Plain-C client of the library's C ABI: includes the header as C99 and calls the
 * host-only entry points.  Built and run by tests/test_library_host.py (no GPU). */
#include <stdio.h>
#include <string.h>

#include "dssync.h"

int main(void) {
    int32_t sizes[2] = {4, 4}, perm[8], off[3];
    int32_t seen[8] = {0};
    int i;
    if (ds_partition(0u, 0u, 8, sizes, 2, perm, off) != DS_OK) return 1;
    for (i = 0; i < 8; ++i) {
        if (perm[i] < 0 || perm[i] > 7 || seen[perm[i]]) return 2;
        seen[perm[i]] = 1;
    }
    if (off[0] != 0 || off[1] != 4 || off[2] != 8) return 3;
    if (ds_partition(0u, 0u, 8, sizes, 1, perm, off) != DS_ERR_BAD_SIZES) return 4;
    if (ds_padded_ld(1000) != 1280 || ds_padded_ld(-1) != 0) return 5;
    if (strncmp(ds_status_string(DS_ERR_ALIGN), "DS_ERR_ALIGN", 12) != 0) return 6;
    /* a GPU entry point with a bad argument reports it before touching any device */
    if (ds_group_sync(NULL, NULL, DS_F32, 0, 0, 0, 8, perm, off, 2, 0.1f, NULL) != DS_ERR_NULL) return 7;
    printf("abi ok: perm");
    for (i = 0; i < 8; ++i) printf(" %d", (int)perm[i]);
    printf("\n");
    return 0;
}
