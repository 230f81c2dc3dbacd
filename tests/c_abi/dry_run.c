/* Host-only use of the C ABI from plain C: proves that include/blitz_layer.h and include/blitz_plan.h compile
 * as C, that the library links without any Python or PyTorch in the process, and that the calls which need
 * no GPU (size queries, a dry-run instance with its slot bookkeeping and argument checks, the scheduling
 * simulation, the scale planner) behave as the header says.  Prints one line per check; exit status 0 = all passed. */
#include <stdio.h>
#include <string.h>

#include "blitz_layer.h"
#include "blitz_plan.h"

static int failures = 0;
#define CHECK(cond)                                                     \
    do {                                                                \
        if (!(cond)) {                                                  \
            printf("FAILED line %d: %s\n", __LINE__, #cond);            \
            ++failures;                                                 \
        }                                                               \
    } while (0)

int main(void) {
    bz_config cfg;
    bz_sizes sz;
    bz_layer_layout lay;
    bz_instance* inst = NULL;
    memset(&cfg, 0, sizeof cfg);
    cfg.n_layers = 2; cfg.hidden = 256; cfg.n_q_heads = 4; cfg.n_kv_heads = 4; cfg.head_dim = 64; cfg.ffn = 688;
    cfg.rms_eps = 1e-5f; cfg.rope_base = 10000.0f;
    cfg.max_seqs = 4; cfg.max_seq_len = 128; cfg.max_tokens = 64; cfg.kv_tokens = 256;
    cfg.flags = BZ_FLAG_DRY_RUN;

    CHECK(bz_query_sizes(&cfg, &sz) == BZ_OK);
    CHECK(sz.layer_bytes == 1582080u);                    /* 2 * (256*64*16 + 3*256*688 + 2*256) */
    CHECK(sz.layer_stride % 256 == 0 && sz.weights_arena_bytes == 2 * sz.layer_stride);
    CHECK(bz_layer_layout_of(&cfg, &lay) == BZ_OK && lay.g1 == 0 && lay.wq == 512 && lay.total == sz.layer_bytes);
    CHECK(strcmp(bz_strerror(BZ_ENOTREADY), "layer not resident yet") == 0);
#ifdef EXPECT_FP32_DEBUG
    CHECK((bz_build_info() & BZ_BUILD_FP32_DEBUG) != 0 && sz.act_elem_bytes == 4);
#else
    CHECK((bz_build_info() & BZ_BUILD_FP32_DEBUG) == 0 && sz.act_elem_bytes == 2);
#endif

    cfg.head_dim = 96;                                    /* unsupported head size */
    CHECK(bz_query_sizes(&cfg, &sz) == BZ_EINVAL);
    cfg.head_dim = 64;

    CHECK(bz_create(&cfg, &inst) == BZ_OK && inst != NULL);
    CHECK(bz_frontier(inst) == 0);
    CHECK(bz_kv_reserve(inst, 0, 100) == BZ_OK);          /* rounded up to 128 positions */
    CHECK(bz_kv_free_tokens(inst) == 128);
    CHECK(bz_kv_reserve(inst, 0, 10) == BZ_EBUSY);
    CHECK(bz_kv_reserve(inst, 1, 129) == BZ_ECAPACITY);
    CHECK(bz_kv_release(inst, 0) == BZ_OK && bz_kv_free_tokens(inst) == 256);
    CHECK(bz_layer_ready(inst, 5) == BZ_EINVAL);
    CHECK(bz_wait_layer(inst, 0) == BZ_ENOTLOADED);
    CHECK(bz_load_layer(inst, 0, &cfg, 12) == BZ_EINVAL); /* wrong size */
    CHECK(bz_wait_stream(inst, NULL) == BZ_ESTATE);       /* a dry-run instance enqueues nothing */
    CHECK(bz_destroy(inst) == BZ_OK);

    {   /* batch descriptions are validated before any GPU call */
        bz_batch* b = NULL;
        int32_t q_bad[3] = {0, 5, 3}, slot[2] = {0, 1}, kv[2] = {0, 0}, slot_dup[2] = {1, 1}, q_ok[3] = {0, 5, 6};
        bz_batch_desc d;
        d.n_seqs = 2; d.q_start = q_bad; d.seq_slot = slot; d.kv_len_before = kv;
        CHECK(bz_batch_create(&d, &b) == BZ_EINVAL && b == NULL);
        d.q_start = q_ok; d.seq_slot = slot_dup;
        CHECK(bz_batch_create(&d, &b) == BZ_EINVAL);
        CHECK(bz_batch_storage_bytes(4, 64, 128) > 0 && bz_batch_storage_bytes(4, 64, 128) % 32 == 0);
        CHECK(bz_batch_rebuild(NULL, &d, NULL) == BZ_EINVAL);
    }
    {   /* section 5.2's worked example through the scheduler's own decision code */
        int32_t T[7];
        double fin[7];
        CHECK(bz_zz_simulate(BZ_ZZ_ZIGZAG, 7, 7, 6.0, 1.0, T, fin) == BZ_OK);
        CHECK(T[0] == 1 && T[1] == 2 && T[2] == 2 && fin[1] == 12.0 && fin[2] == 17.0);
        CHECK(bz_zz_simulate(BZ_ZZ_BEST_EFFORT, 7, 7, 6.0, 1.0, T, fin) == BZ_OK);
        CHECK(T[0] == 1 && T[5] == 1 && fin[5] == 37.0);
        CHECK(bz_zz_simulate(2, 7, 7, 6.0, 1.0, T, fin) == BZ_EINVAL);
        {   /* a time per layer and request (section 5.4): 4 layers, one every 3, source free at 2, times (1, 2) */
            const double w[2] = {1.0, 2.0}, bad[2] = {1.0, 0.0};
            CHECK(bz_zz_simulate_weighted(BZ_ZZ_ZIGZAG, 4, 2, 3.0, 2.0, w, T, fin) == BZ_OK);
            CHECK(T[0] == 1 && T[1] == 2 && fin[0] == 5.0 && fin[1] == 9.0);
            CHECK(bz_zz_simulate_weighted(BZ_ZZ_ZIGZAG, 4, 2, 3.0, 2.0, bad, T, fin) == BZ_EINVAL);
        }
    }
    {   /* scale plan: one source, two spare nodes under the same leaf -> one chain S -> T1 -> T2, slower target last */
        bz_plan_node nodes[3];
        bz_plan_hop hops[2];
        int n_hops = 0, n_chains = 0, interferes = 1;
        memset(nodes, 0, sizeof nodes);
        nodes[0].id = 0; nodes[0].n_gpus = 1; nodes[0].gpu_bw = 25e9; nodes[0].leaf = 0; nodes[0].role = BZ_PLAN_SOURCE;
        nodes[1].id = 1; nodes[1].n_gpus = 1; nodes[1].gpu_bw = 12.5e9; nodes[1].leaf = 0; nodes[1].role = BZ_PLAN_SPARE;
        nodes[2].id = 2; nodes[2].n_gpus = 1; nodes[2].gpu_bw = 25e9; nodes[2].leaf = 0; nodes[2].role = BZ_PLAN_SPARE;
        CHECK(bz_plan_generate(nodes, 3, 2, 1.0, 4, 1e9, hops, 2, &n_hops, &n_chains, &interferes) == BZ_OK);
        CHECK(n_hops == 2 && n_chains == 1 && interferes == 0);
        CHECK(hops[0].from == 0 && hops[0].to == 2 && hops[1].from == 2 && hops[1].to == 1 && hops[1].is_tail == 1);
    }
    printf(failures ? "%d check(s) failed\n" : "all checks passed\n", failures);
    return failures ? 1 : 0;
}
