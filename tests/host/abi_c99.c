/* The C ABI from a plain C99 program: the header must compile as C, and the host-only entry points must be callable
 * without a GPU.  Built and run by tests/test_abi_host.py. */
#include <stdio.h>
#include <string.h>

#include "spd.h"

int main(void)
{
    spd_shape shape;
    spd_kv_view view;
    int32_t lens[3] = {700, 0, 40};
    spd_work_item items[256];
    int64_t n_items = 0;
    int32_t chunk = 0;
    int rc;

    memset(&shape, 0, sizeof shape);
    memset(&view, 0, sizeof view);
    shape.dtype = SPD_BF16;
    shape.n_q_heads = 32;
    shape.n_kv_heads = 8;
    shape.head_dim = 128;
    shape.scale = 0.0883883f;

    if (strcmp(spd_strerror(SPD_OK), "ok") != 0)
        return 1;
    view.n_users = -1;
    if (spd_validate_partial(&shape, (const void *)0x1000, &view, (const float *)0x2000, (const float *)0x3000) !=
        SPD_ERR_LEN)
        return 2;
    rc = spd_build_schedule(&shape, 3, lens, 256, 0, items, 256, &n_items, &chunk);
    if (rc != SPD_OK || n_items <= 0)
        return 3;
    if (spd_partial_attn_private(NULL, &shape, NULL, &view, NULL, NULL, NULL) != SPD_ERR_NULL)
        return 4;
    printf("c99 ok: %lld work items, chunk %d tokens\n", (long long)n_items, (int)chunk);
    return 0;
}
