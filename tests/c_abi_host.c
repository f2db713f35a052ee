/* The boundary used from plain C, host-only calls (no GPU needed): a pool over
 * a made-up device range, two models that share a tensor, plan -> commit ->
 * release, and the error codes of the obvious mistakes.  Prints "ok" and
 * exits 0 when every check holds. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include "tangram.h"

#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "line %d: %s\n", __LINE__, #cond); return 1; } } while (0)

int main(void) {
    void *base = (void *)((uintptr_t)1 << 40);
    void *host = (void *)((uintptr_t)1 << 41);
    tg_pool *pool = NULL;
    CHECK(tg_pool_create(base, 4096, 256, &pool) == TG_OK && pool != NULL);
    CHECK(tg_pool_create(base, 4096, 24, &pool) == TG_ERR_INVALID);
    CHECK(tg_pool_create(NULL, 4096, 256, &pool) == TG_ERR_INVALID);

    tg_tensor_desc a[2] = {{700, 0x1111, 0}, {256, 0x2222, 768}};
    tg_model_desc ma = {1, host, 1024, 2, 0, a};
    tg_load_plan *plan = NULL;
    CHECK(tg_plan(pool, &ma, 0, NULL, &plan) == TG_OK && plan != NULL);
    const tg_plan_op *ops = NULL;
    uint32_t n = 0;
    uint64_t reused = 1, transfer = 1;
    CHECK(tg_plan_ops(plan, &ops, &n, &reused, &transfer) == TG_OK);
    CHECK(n == 2 && reused == 0 && transfer == 956);
    CHECK(ops[0].kind == TG_OP_H2D && ops[0].dst_off == 0 && ops[0].src_off == 0 && ops[0].nbytes == 700);
    CHECK(ops[1].kind == TG_OP_H2D && ops[1].dst_off == 768 && ops[1].src_off == 768);
    void *ptrs[2] = {NULL, NULL};
    CHECK(tg_commit(pool, plan, ptrs) == TG_OK);
    CHECK(ptrs[0] == base && ptrs[1] == (char *)base + 768);
    CHECK(tg_commit(pool, plan, ptrs) == TG_ERR_INVALID);          /* a plan is used once */
    tg_plan_free(plan);

    tg_stats st;
    CHECK(tg_pool_stats(pool, &st) == TG_OK);
    CHECK(st.capacity == 4096 && st.free_bytes == 4096 - 1024 && st.n_entries == 2 && st.n_active == 2);
    CHECK(tg_plan(pool, &ma, 0, NULL, &plan) == TG_ERR_INVALID);   /* model 1 is running */
    CHECK(tg_release(pool, 1, 0) == TG_OK);
    CHECK(tg_release(pool, 7, 0) == TG_ERR_NOTFOUND);

    /* model 2 shares the first tensor (same fingerprint and length) */
    tg_tensor_desc b[2] = {{700, 0x1111, 256}, {512, 0x3333, 1024}};
    tg_model_desc mb = {2, host, 2048, 2, 0, b};
    uint64_t reuse = 0;
    double est = 0.0;
    CHECK(tg_reuse_size(pool, &mb, 100.0, &reuse, &est) == TG_OK && reuse == 700 && est == 5.12);
    CHECK(tg_plan(pool, &mb, TG_PLAN_ALIAS, NULL, &plan) == TG_OK);
    CHECK(tg_plan_ops(plan, &ops, &n, &reused, &transfer) == TG_OK);
    CHECK(reused == 700 && transfer == 512);
    CHECK(ops[0].kind == TG_OP_REUSE && ops[0].dst_off == 0 && ops[0].src_off == 0);
    tg_plan_summary info;
    CHECK(tg_plan_info(plan, &info) == TG_OK && info.alias == 1 && info.copy_bytes == 0 && info.n_moves == 0);
    CHECK(info.n_reused == 1 && info.n_tensors == 2);
    {   /* argument checks of the extended assemble come before anything touches the device */
        tg_assemble_args args;
        memset(&args, 0, sizeof args);
        CHECK(tg_assemble_ex(pool, plan, NULL, ptrs) == TG_ERR_INVALID);
        args.flags = 8u;
        CHECK(tg_assemble_ex(pool, plan, &args, ptrs) == TG_ERR_INVALID);
        CHECK(tg_assemble_ex(NULL, plan, &args, ptrs) == TG_ERR_INVALID);
        /* the load in steps: none of its calls does anything to a plan whose load has not begun */
        {
            tg_feed_row row = {1, 0, 0};
            uint32_t ticket = 99;
            CHECK(tg_assemble_begin(pool, plan, NULL) == TG_ERR_INVALID);
            CHECK(tg_assemble_async(pool, NULL, &args) == TG_ERR_INVALID);
            CHECK(tg_assemble_feed(pool, plan, host, 4096, &row, 1, &ticket) == TG_ERR_INVALID && ticket == 99);
            CHECK(tg_assemble_feed_wait(pool, plan, 0) == TG_ERR_INVALID);
            CHECK(tg_assemble_wait(pool, plan, ptrs) == TG_ERR_INVALID);
        }
    }
    {   /* launch shape and profiling belong to the pool; the plan keeps its own timing */
        tg_tuning def, cur;
        tg_timing tm;
        CHECK(tg_default_tuning(&def) == TG_OK && def.fingerprint_unroll == 8 && def.gather_unroll == 4);
        CHECK(def.h2d_kernel_max_bytes == 65536 && def.h2d_group_bytes == 0 && def.fuse_verify == 1);
        CHECK(tg_pool_get_tuning(pool, &cur) == TG_OK && memcmp(&cur, &def, sizeof def) == 0);
        cur.gather_unroll = 8;
        cur.h2d_group_bytes = 8u << 20;
        CHECK(tg_pool_set_tuning(pool, &cur) == TG_OK);
        CHECK(tg_pool_get_tuning(pool, &def) == TG_OK && def.gather_unroll == 8 && def.h2d_group_bytes == (8u << 20));
        CHECK(tg_pool_set_tuning(pool, NULL) == TG_ERR_INVALID && tg_default_tuning(NULL) == TG_ERR_INVALID);
        CHECK(tg_pool_set_profiling(pool, 1) == TG_OK && tg_pool_set_profiling(NULL, 1) == TG_ERR_INVALID);
        CHECK(tg_plan_timing(plan, &tm) == TG_OK && tm.plan_host_ms > 0.0f && tm.gather_ms == 0.0f && tm.feeds == 0);
        CHECK(tg_plan_timing(NULL, &tm) == TG_ERR_INVALID);
    }
    {   /* a model without a host image: rows only */
        tg_load_plan *bare = NULL;
        tg_tensor_desc d[1] = {{300, 0x5555, 123456789}};
        tg_model_desc md = {9, NULL, 0, 1, 0, d};
        tg_model_desc bad = {9, NULL, 64, 1, 0, d};
        CHECK(tg_plan(pool, &md, 0, NULL, &bare) == TG_OK);
        CHECK(tg_plan_ops(bare, &ops, &n, NULL, NULL) == TG_OK && n == 1 && ops[0].src_off == 123456789);
        CHECK(tg_assemble(pool, bare, 0, NULL, NULL, NULL) == TG_ERR_INVALID);   /* nothing to copy from */
        tg_plan_free(bare);
        CHECK(tg_plan(pool, &bad, 0, NULL, &bare) == TG_ERR_INVALID);
        CHECK(tg_plan(pool, &md, TG_PLAN_CONFIRM, NULL, &bare) == TG_ERR_INVALID);
        CHECK(tg_plan_ops(plan, &ops, &n, NULL, NULL) == TG_OK);
    }
    {
        CHECK(tg_commit(pool, plan, ptrs) == TG_OK && ptrs[0] == base);
        tg_plan_free(plan);
    }

    /* the Region List and the Tensor Mapping can be read out */
    {
        tg_region regs[8];
        tg_entry rows[8];
        uint32_t nr = 0, ne = 0;
        CHECK(tg_pool_regions(pool, NULL, 0, &nr) == TG_OK && nr == 4);
        CHECK(tg_pool_regions(pool, regs, 8, &nr) == TG_OK && nr == 4);
        CHECK(regs[0].off == 0 && regs[0].len == 768 && regs[0].free == 0);
        CHECK(regs[3].free == 1 && regs[3].off + regs[3].len == 4096);
        CHECK(tg_pool_entries(pool, rows, 8, &ne) == TG_OK && ne == 3);
        CHECK(rows[0].off == 0 && rows[0].nbytes == 700 && rows[0].fp == 0x1111 && rows[0].n_owners == 2 &&
              rows[0].active_refs == 1);
        CHECK(tg_pool_entries(pool, rows, 1, &ne) == TG_OK && ne == 3);
        CHECK(tg_pool_entries(pool, NULL, 1, &ne) == TG_ERR_INVALID);
    }

    /* too big for what is left, and flags nobody defined */
    tg_tensor_desc c[1] = {{4096, 0x4444, 0}};
    tg_model_desc mc = {3, host, 4096, 1, 0, c};
    CHECK(tg_plan(pool, &mc, 0, NULL, &plan) == TG_ERR_NOSPACE);
    CHECK(tg_plan(pool, &mc, 1u << 9, NULL, &plan) == TG_ERR_INVALID);
    c[0].nbytes = 0;
    CHECK(tg_plan(pool, &mc, 0, NULL, &plan) == TG_ERR_INVALID);

    CHECK(tg_release(pool, 2, TG_RELEASE_EVICT) == TG_OK);
    CHECK(tg_release(pool, 1, TG_RELEASE_EVICT) == TG_OK);
    CHECK(tg_pool_stats(pool, &st) == TG_OK && st.free_bytes == 4096 && st.n_entries == 0 && st.n_free_regions == 1);
    CHECK(strcmp(tg_strerror(TG_ERR_STALE), "plan is stale") == 0);
    CHECK(tg_pool_destroy(pool) == TG_OK);
    puts("ok");
    return 0;
}
