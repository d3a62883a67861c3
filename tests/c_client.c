/* A C99 client of the library's boundary, host-only calls: it shows that include/mpa.h and
 * include/mpa_sched.h are C headers and that libmpa.so links from C.  It forms one batch with the
 * scheduler, asks the planner how the attention call would decompose it, and prints what it got as
 * "key value" lines that tests/test_c_client.py checks against the Python binding. */
#include <stdio.h>
#include <stdlib.h>

#include "mpa.h"
#include "mpa_sched.h"

#define CHECK(call)                                                              \
    do {                                                                         \
        int st_ = (call);                                                        \
        if (st_ != MPA_OK) {                                                     \
            fprintf(stderr, "%s -> %s\n", #call, mpa_status_string(st_));        \
            return 1;                                                            \
        }                                                                        \
    } while (0)

int main(void)
{
    if (mpa_abi_version() != MPA_ABI_VERSION) {
        fprintf(stderr, "library built from another header version\n");
        return 4;
    }
    mpa_config cfg = {40, 40, 128, 32, MPA_BF16};
    mpa_ctx *ctx = NULL;
    CHECK(mpa_create(&ctx, &cfg));
    mpa_config bad = cfg;
    bad.head_dim = 96;
    mpa_ctx *none = NULL;
    printf("create_bad %d\n", mpa_create(&none, &bad));
    printf("status_string %s\n", mpa_status_string(MPA_ERR_WORKSPACE));

    mpa_sched_config sc;
    sc.block_size = 32;
    sc.num_blocks = 256;
    sc.pivot_forward_size = 768;
    sc.max_batch_tokens = 4096;
    sc.pivot_time = 0.05;
    sc.max_batch_time = 0.1;
    sc.gamma = 0.75;
    sc.preempt_max_time = 0.0;
    sc.preempt_probability = 0.0;
    sc.num_swap_blocks = 0;
    mpa_sched *s = NULL;
    CHECK(mpa_sched_create(&s, &sc, NULL));
    CHECK(mpa_sched_add_request(s, 7, 1000, 4, 1.0, 0.1, 0.0));
    CHECK(mpa_sched_add_request(s, 8, 100, 2, 1.0, 0.1, 0.0));
    mpa_sched_batch info;
    CHECK(mpa_sched_next_batch(s, 0.0, &info));
    printf("num_seqs %d\nnum_tokens %d\ntoken_budget %d\n", info.num_seqs, info.num_tokens, info.token_budget);
    if (info.num_seqs < 1 || info.num_seqs > 8) return 2;
    int64_t ids[8];
    int32_t cs[9], ctxl[8];
    int64_t *slots = (int64_t *)malloc(sizeof(int64_t) * (size_t)info.num_tokens);
    int32_t stride = info.max_blocks_per_seq;
    int32_t *table = (int32_t *)malloc(sizeof(int32_t) * (size_t)info.num_seqs * (size_t)stride);
    if (!slots || !table) return 3;
    CHECK(mpa_sched_batch_arrays(s, ids, cs, ctxl, slots, table, stride));
    for (int i = 0; i < info.num_seqs; ++i)
        printf("seq %lld %d %d %d\n", (long long)ids[i], cs[i], cs[i + 1], ctxl[i]);
    printf("slot_first %lld\nslot_last %lld\n", (long long)slots[0], (long long)slots[info.num_tokens - 1]);

    size_t ws = mpa_workspace_bytes_for_batch(ctx, cs, ctxl, info.num_seqs);
    size_t ws_max = mpa_workspace_bytes(ctx, 8, 4096, 8192);
    printf("workspace %zu\nworkspace_bound_holds %d\n", ws, ws_max >= ws);
    int32_t counts[4];
    int32_t items[8 * 64];
    int64_t n = mpa_plan_describe(ctx, cs, ctxl, info.num_seqs, items, 64, counts);
    printf("plan_items %lld\nplan_counts %d %d %d %d\n", (long long)n, counts[0], counts[1], counts[2], counts[3]);
    /* a null q must be refused before anything touches a device */
    printf("attention_null %d\n", mpa_mixed_paged_attention(ctx, NULL, NULL, NULL, NULL, stride, cs, ctxl, info.num_seqs,
                                                            info.num_tokens, 0.0f, NULL, NULL, 0, NULL));
    free(slots);
    free(table);
    CHECK(mpa_sched_destroy(s));
    CHECK(mpa_destroy(ctx));
    return 0;
}
