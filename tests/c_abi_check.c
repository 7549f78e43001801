/* Plain C user of the library: the header must compile as C99, and the
 * host-only device must plan the worked example of tests/golden/plan_small.txt. */
#include <stdio.h>
#include <string.h>
#include "rdev.h"

#define CHECK(cond) do { if (!(cond)) { printf("FAILED line %d: %s (%s)\n", __LINE__, #cond, rdev_last_error()); return 1; } } while (0)

int main(void) {
    rdev_device_t *dev = NULL;
    rdev_plan_t *plan = NULL;
    uint32_t a0, a1, n;
    rdev_tensor_desc t[5];
    rdev_placement p;
    rdev_region r;
    uint64_t base, stat, heap_off, heap_bytes;
    static const uint64_t want[5][5] = { /* data_offset, bytes, flag_offset, meta_offset, region_bytes */
        {0, 12, 16, 0, 256}, {256, 300, 560, 0, 512}, {0, 0, 892, 768, 256}, {0, 7936, 7936, 0, 8192}, {1024, 0, 1024, 0, 256}};
    uint32_t i;

    CHECK(sizeof(rdev_meta) == RDEV_META_BYTES && sizeof(rdev_frag) == 32);
    CHECK(rdev_open(&dev, RDEV_HOST_ONLY) == RDEV_OK);
    CHECK(rdev_register_arena(dev, (void *)0x700000000000ull, 1u << 20, 0, &a0) == RDEV_OK);
    CHECK(rdev_register_arena(dev, (void *)0x710000000000ull, 1u << 20, 0, &a1) == RDEV_OK);
    memset(t, 0, sizeof t);
    t[0].tensor_id = 0; t[0].dtype = RDEV_F32; t[0].ndims = 1; t[0].dims[0] = 3;   t[0].dst_arena = a0;
    t[1].tensor_id = 1; t[1].dtype = RDEV_U8;  t[1].ndims = 1; t[1].dims[0] = 300; t[1].dst_arena = a0;
    t[2].tensor_id = 2; t[2].dtype = RDEV_F32; t[2].ndims = 2; t[2].dims[0] = -1; t[2].dims[1] = 4; t[2].dst_arena = a0;
    t[3].tensor_id = 3; t[3].dtype = RDEV_F64; t[3].ndims = 2; t[3].dims[0] = 32; t[3].dims[1] = 31; t[3].dst_arena = a1;
    t[4].tensor_id = 4; t[4].dtype = RDEV_I16; t[4].ndims = 1; t[4].dims[0] = 0;   t[4].dst_arena = a0;
    CHECK(rdev_plan(dev, t, 5, NULL, &plan) == RDEV_OK);
    CHECK(rdev_plan_count(plan, &n) == RDEV_OK && n == 5);
    for (i = 0; i < 5; ++i) {
        CHECK(rdev_plan_get(plan, i, &p) == RDEV_OK);
        CHECK(p.tensor_id == i && p.kind == (i == 2 ? RDEV_DYNAMIC : RDEV_STATIC));
        CHECK(p.data_offset == want[i][0] && p.bytes == want[i][1] && p.flag_offset == want[i][2] &&
              p.meta_offset == want[i][3] && p.region_bytes == want[i][4]);
    }
    CHECK(rdev_plan_arena_info(plan, a0, &base, &stat, &heap_off, &heap_bytes) == RDEV_OK);
    CHECK(base == 0 && stat == 1280 && heap_off == 1280 && heap_bytes == 0);
    CHECK(rdev_alloc_region(dev, a0, 100, 256, &r) == RDEV_OK && r.offset == 1280);
    CHECK(rdev_write_batch(dev, plan, NULL, 0, RDEV_ZEROCOPY, 1, NULL) == RDEV_E_HIP);   /* no GPU behind this device */
    CHECK(strlen(rdev_last_error()) > 0);
    CHECK(rdev_close(dev) == RDEV_E_BUSY);
    CHECK(rdev_plan_free(plan) == RDEV_OK);
    CHECK(rdev_free_region(dev, &r) == RDEV_OK);
    CHECK(rdev_close(dev) == RDEV_OK);
    printf("c abi ok\n");
    return 0;
}
