/* Test-only: a plain C program that links the library and calls its host-only entry points,
 * to show that the boundary is usable without Python or C++.  Prints "ok" and returns 0. */
#include <stdio.h>
#include <string.h>

#include "tokencake_kv.h"

int main(void)
{
    if (strcmp(tc_strerror(TC_OK), "ok") != 0) return 1;
    if (tc_fnv1a64("a", 1, TC_FNV_BASIS) != 0xAF63DC4C8601EC8Cull) return 2;
    if (tc_upload_budget(40, 30, 10) != 20 || tc_gradual_reserve(20, 10, 20) != 5) return 3;

    tc_index *ix = NULL;
    if (tc_index_create(&ix) != TC_OK) return 4;
    uint64_t keys[3] = {10, 11, 12};
    int32_t blocks[3] = {7, 3, 9};
    static char records[3 * 256];
    if (tc_index_insert(ix, keys, blocks, records, 256, 3) != TC_OK) return 5;
    uint64_t q[3] = {10, 99, 12};
    tc_index_hit hit[3];
    uint32_t hits = 0;
    if (tc_index_lookup(ix, q, 3, hit, &hits) != TC_OK || hits != 1 || hit[0].cpu_record != records) return 6;
    if (tc_index_insert(ix, keys, blocks, records, 256, 1) != TC_ERR_DUP) return 7;
    if (tc_index_destroy(ix) != TC_OK) return 8;

    tc_req_state r = {TC_RUNNING, 0, 0, 0};
    int action = -1;
    if (tc_lifecycle_step(&r, TC_EV_CALL_START, &action) != TC_OK || r.state != TC_PENDING_OFFLOAD) return 9;
    if (tc_create(NULL, NULL, NULL) != TC_ERR_INVAL) return 10;
    puts("ok");
    return 0;
}
