/* A plain C program against include/kun.h: the header must compile as C, and the host-only entry
 * points must work when called from C through the dynamic linker (no Python, no GPU work).
 * Built and run by tests/test_host_boundary.py. */
#include <math.h>
#include <stdio.h>
#include <string.h>

#include "kun.h"

#define CHECK(cond)                                                \
    do {                                                           \
        if (!(cond)) {                                             \
            printf("FAILED line %d: %s\n", __LINE__, #cond);       \
            return 1;                                              \
        }                                                          \
    } while (0)

int main(void) {
    /* pool arithmetic on made-up (never dereferenced) device addresses: 8 KV heads of 128 dims, bf16 */
    kun_kv_pool* pool = NULL;
    char* base0 = (char*)0x100000000ull;
    char* base1 = (char*)0x900000000ull;
    CHECK(kun_kv_pool_create(&pool, base0, 10 * 65536 + 100, KUN_BF16, 8, 128, 16) == KUN_OK);
    size_t bb = 0;
    CHECK(kun_kv_pool_block_bytes(pool, &bb) == KUN_OK && bb == 65536);
    int64_t first = -1, added = -1, n = 0;
    CHECK(kun_kv_pool_extend(pool, base1, 3 * 65536, &first, &added) == KUN_OK && first == 10 && added == 3);
    CHECK(kun_kv_pool_num_blocks(pool, &n) == KUN_OK && n == 13);
    int range = -1;
    size_t off = 0;
    void* addr = NULL;
    CHECK(kun_kv_pool_resolve(pool, 11, &range, &off, &addr) == KUN_OK);
    CHECK(range == 1 && off == 65536 && addr == (void*)(base1 + 65536));
    CHECK(kun_kv_pool_resolve(pool, 13, &range, &off, &addr) == KUN_ERR_BLOCK_OOB);
    CHECK(kun_kv_pool_extend(pool, base1 + 65536, 65536, NULL, NULL) == KUN_ERR_OVERLAP);
    kun_kv_pool* bad = NULL;
    CHECK(kun_kv_pool_create(&bad, base0 + 8, 65536, KUN_BF16, 8, 128, 16) == KUN_ERR_MISALIGNED && bad == NULL);
    CHECK(strcmp(kun_status_string(KUN_ERR_OVERLAP), kun_status_string(KUN_OK)) != 0);
    /* blocks of 64 tokens */
    kun_kv_pool* pool64 = NULL;
    CHECK(kun_kv_pool_create(&pool64, base0, 4 * 262144, KUN_BF16, 8, 128, 64) == KUN_OK);
    CHECK(kun_kv_pool_block_bytes(pool64, &bb) == KUN_OK && bb == 262144);
    CHECK(kun_kv_pool_destroy(pool64) == KUN_OK);
    CHECK(kun_kv_pool_destroy(pool) == KUN_OK);

    /* cost model: a chunk of c tokens after p prior ones costs alpha (p c + (c c + c) / 2) + beta c + gamma */
    kun_cost_model m = {2.0, 3.0, 5.0};
    CHECK(fabs(kun_cost_chunk(&m, 10, 4) - (2.0 * (40 + 10) + 12.0 + 5.0)) < 1e-9);
    kun_chunk q[2] = {{0, 10, 4}, {1, 0, 2}};
    CHECK(fabs(kun_cost_microbatch(&m, q, 2) - (117.0 + (2.0 * 3 + 6.0 + 5.0) - 5.0)) < 1e-9);

    /* drop plan: four single instances, 8 layers of 1 byte, demand of one copy: instances 0 and 1 merge */
    int32_t group[4], kf[4], ke[4], members[6], sizes[6];
    int64_t dropped[4], freed = 0;
    int n_merges = 0, met = 0;
    CHECK(kun_drop_plan(4, NULL, 8, 1, 8, group, kf, ke, dropped, members, sizes, &n_merges, &freed, &met) == KUN_OK);
    CHECK(n_merges == 1 && freed == 8 && met == 1);
    CHECK(group[0] == group[1] && group[2] != group[0] && group[3] != group[0] && group[2] != group[3]);
    CHECK(kf[0] == 0 && ke[0] == 4 && kf[1] == 4 && ke[1] == 8 && dropped[0] == 4 && dropped[2] == 0);
    printf("c abi ok\n");
    return 0;
}
