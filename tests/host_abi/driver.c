/* Drives every entry point of include/cs.h through its argument checks and its host-side bookkeeping
 * (plan cache, multi-operator tables, scratch limits, allocation failures), built for the host alone with
 * the address and undefined-behaviour sanitizers.  Plain C: the header has to compile as C99. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include "cs.h"

extern size_t hip_standin_live_allocations;
extern size_t hip_standin_fail_after;
extern int standin_launches;

static int failures = 0;
#define EXPECT(call, want) do { cs_status st_ = (call); if (st_ != (want)) { \
    fprintf(stderr, "line %d: %s returned %d, expected %d (%s)\n", __LINE__, #call, (int)st_, (int)(want), ctx ? cs_last_error(ctx) : ""); ++failures; } } while (0)

int main(void) {
    cs_ctx* ctx = NULL;
    /* creation */
    EXPECT(cs_create(NULL, 0, NULL, 0), CS_EINVAL);
    EXPECT(cs_create(&ctx, 5, NULL, 0), CS_EHIP);
    EXPECT(cs_create(&ctx, -1, NULL, 0), CS_EHIP);
    hip_standin_fail_after = 0;
    EXPECT(cs_create(&ctx, 0, NULL, 0), CS_ENOMEM);
    hip_standin_fail_after = (size_t)-1;
    EXPECT(cs_create(&ctx, 0, NULL, 1 << 20), CS_OK);
    if (!ctx) return 2;
    if (strlen(cs_last_error(ctx)) != 0) ++failures;
    if (strcmp(cs_last_error(NULL), "no context") != 0) ++failures;

    float* buf = aligned_alloc(256, 1 << 16);
    int32_t* ibuf = aligned_alloc(256, 1 << 16);
    char* odd = (char*)buf + 4;                               /* not 16-byte aligned */
    cs_op op = { CS_GAUSS, 7u, 1u, 64, 1024 };
    cs_op bad_ens = op; bad_ens.ens = 9;
    cs_op bad_m = op; bad_m.m = 0;
    cs_op srht_rows = { CS_SRHT, 7u, 1u, 4096, 1000 };        /* more rows than the padded transform has */
    cs_op srht_big = { CS_SRHT, 7u, 1u, 64, 100000 };
    cs_dict dct = { buf, 16, 64, 1 };
    cs_dict ident = { NULL, 16, 64, 64 };
    cs_dict bad_n = { buf, 17, 64, 1 };
    cs_dict bad_rb = { NULL, 16, 64, 1 };
    cs_dict odd_psi = { (const float*)odd, 16, 64, 1 };

    /* sketch */
    EXPECT(cs_sketch(NULL, &op, buf, 1, buf), CS_EINVAL);
    EXPECT(cs_sketch(ctx, NULL, buf, 1, buf), CS_EINVAL);
    EXPECT(cs_sketch(ctx, &bad_ens, buf, 1, buf), CS_EINVAL);
    EXPECT(cs_sketch(ctx, &bad_m, buf, 1, buf), CS_EINVAL);
    EXPECT(cs_sketch(ctx, &srht_rows, buf, 1, buf), CS_EINVAL);
    EXPECT(cs_sketch(ctx, &srht_big, buf, 1, buf), CS_EINVAL);
    EXPECT(cs_sketch(ctx, &op, buf, -1, buf), CS_EINVAL);
    EXPECT(cs_sketch(ctx, &op, NULL, 1, buf), CS_EINVAL);
    EXPECT(cs_sketch(ctx, &op, (const float*)odd, 1, buf), CS_EALIGN);
    EXPECT(cs_sketch(ctx, &op, buf, 0, buf), CS_OK);
    EXPECT(cs_sketch(ctx, &op, buf, 3, buf), CS_OK);
    cs_op ops2[2] = { op, op }; ops2[1].stream_id = 2;
    cs_op ops_mixed[2] = { op, op }; ops_mixed[1].m = 65;
    EXPECT(cs_sketch_multi(ctx, 0, ops2, buf, 1, buf), CS_EINVAL);
    EXPECT(cs_sketch_multi(ctx, 2, NULL, buf, 1, buf), CS_EINVAL);
    EXPECT(cs_sketch_multi(ctx, 2, ops_mixed, buf, 1, buf), CS_EINVAL);
    EXPECT(cs_sketch_multi(ctx, 2, ops2, buf, 1, buf), CS_OK);

    /* plans and recovery */
    EXPECT(cs_plan(ctx, &op, NULL), CS_EINVAL);
    EXPECT(cs_plan(ctx, &op, &bad_n), CS_EINVAL);
    EXPECT(cs_plan(ctx, &op, &bad_rb), CS_EINVAL);
    EXPECT(cs_plan(ctx, &op, &odd_psi), CS_EALIGN);
    hip_standin_fail_after = 2;                               /* third allocation of the plan fails */
    size_t live = hip_standin_live_allocations;
    EXPECT(cs_plan(ctx, &op, &dct), CS_ENOMEM);
    hip_standin_fail_after = (size_t)-1;
    if (hip_standin_live_allocations != live) { fprintf(stderr, "a failed plan leaked device memory\n"); ++failures; }
    EXPECT(cs_plan(ctx, &op, &dct), CS_OK);
    EXPECT(cs_plan(ctx, &op, &dct), CS_OK);                   /* cached */
    EXPECT(cs_recover_support(ctx, &op, &dct, 0, buf, 1, ibuf, buf, buf, buf), CS_EINVAL);
    EXPECT(cs_recover_support(ctx, &op, &dct, 17, buf, 1, ibuf, buf, buf, buf), CS_EINVAL);
    EXPECT(cs_recover_support(ctx, &op, &ident, 1, buf, 1, ibuf, buf, buf, buf), CS_EILLPOSED);
    EXPECT(cs_recover_support(ctx, &op, &dct, 4, buf, 1, NULL, buf, buf, buf), CS_EINVAL);
    EXPECT(cs_recover_support(ctx, &op, &dct, 4, buf, 1, ibuf, (float*)odd, buf, buf), CS_EALIGN);
    EXPECT(cs_recover_support(ctx, &op, &dct, 4, buf, -2, ibuf, buf, buf, buf), CS_EINVAL);
    EXPECT(cs_recover_support(ctx, &op, &dct, 4, buf, 0, ibuf, buf, buf, buf), CS_OK);
    EXPECT(cs_recover_support(ctx, &op, &dct, 4, buf, 2, ibuf, NULL, NULL, NULL), CS_OK);
    cs_dict dcts2[2] = { dct, dct };
    EXPECT(cs_recover_support_multi(ctx, 2, ops2, NULL, 4, buf, 1, ibuf, buf, buf, buf), CS_EINVAL);
    EXPECT(cs_recover_support_multi(ctx, 2, ops_mixed, dcts2, 4, buf, 1, ibuf, buf, buf, buf), CS_EINVAL);
    EXPECT(cs_recover_support_multi(ctx, 2, ops2, dcts2, 4, buf, 1, ibuf, buf, buf, buf), CS_OK);
    EXPECT(cs_recover_support_multi(ctx, 2, ops2, dcts2, 4, buf, 1, ibuf, buf, buf, buf), CS_OK);   /* table reused */
    EXPECT(cs_plan_drop(ctx, &ops2[1], &dct), CS_OK);         /* takes the table with it */
    EXPECT(cs_plan_drop(ctx, &ops2[1], &dct), CS_OK);
    EXPECT(cs_plan_drop(ctx, NULL, &dct), CS_EINVAL);
    EXPECT(cs_recover_support_multi(ctx, 2, ops2, dcts2, 4, buf, 1, ibuf, buf, buf, buf), CS_OK);
    EXPECT(cs_recover_support_iht(ctx, &op, &dct, 4, 0, buf, 1, ibuf, buf, buf, buf), CS_EINVAL);
    EXPECT(cs_recover_support_iht(ctx, &op, &dct, 4, 3, buf, 1, ibuf, buf, buf, buf), CS_OK);
    EXPECT(cs_recover_support_inc(ctx, &op, &dct, 4, buf, 1, ibuf, NULL, 0.f, 5, ibuf, buf, buf, buf), CS_EINVAL);
    EXPECT(cs_recover_support_inc(ctx, &op, &dct, 4, buf, 1, ibuf, NULL, -1.f, 1, ibuf, buf, buf, buf), CS_EINVAL);
    EXPECT(cs_recover_support_inc(ctx, &op, &dct, 4, buf, 1, NULL, NULL, 0.f, 1, ibuf, buf, buf, buf), CS_EINVAL);
    EXPECT(cs_recover_support_inc(ctx, &op, &dct, 4, buf, 1, ibuf, NULL, 0.f, 1, ibuf, buf, buf, buf), CS_OK);
    EXPECT(cs_recover_support_inc_carry(ctx, &op, &dct, 4, buf, 1, ibuf, 5, (uint32_t*)ibuf, ibuf, buf, buf, buf), CS_EINVAL);
    EXPECT(cs_recover_support_inc_carry(ctx, &op, &dct, 4, buf, 1, ibuf, 1, NULL, ibuf, buf, buf, buf), CS_EINVAL);
    EXPECT(cs_recover_support_inc_carry(ctx, &op, &dct, 4, buf, 1, ibuf, 1, (uint32_t*)((char*)ibuf + 4), ibuf, buf, buf, buf), CS_EALIGN);
    EXPECT(cs_recover_support_inc_carry(ctx, &op, &dct, 4, buf, 1, ibuf, 1, (uint32_t*)ibuf, ibuf, buf, buf, buf), CS_OK);
    if (cs_inc_state_words(4) != 24 || cs_inc_state_words(0) != 0) { printf("cs_inc_state_words\n"); return 1; }

    /* execution calls */
    EXPECT(cs_block_ffn(ctx, 7, buf, buf, buf, 256, 16, 64, buf, 1, ibuf, 4, 0, buf), CS_EINVAL);
    EXPECT(cs_block_ffn(ctx, CS_BF16, buf, buf, buf, 250, 16, 64, buf, 1, ibuf, 4, 0, buf), CS_EINVAL);
    EXPECT(cs_block_ffn(ctx, CS_BF16, buf, buf, buf, 256, 16, 64, buf, 1, ibuf, 17, 0, buf), CS_EINVAL);
    EXPECT(cs_block_ffn(ctx, CS_BF16, buf, buf, buf, 256, 16, 64, buf, 70000, ibuf, 4, 0, buf), CS_EINVAL);
    EXPECT(cs_block_ffn(ctx, CS_BF16, buf, NULL, buf, 256, 16, 64, buf, 1, ibuf, 4, 0, buf), CS_EINVAL);
    EXPECT(cs_block_ffn(ctx, CS_BF16, buf, buf, buf, 256, 16, 64, odd, 1, ibuf, 4, 0, buf), CS_EALIGN);
    EXPECT(cs_block_ffn(ctx, CS_BF16, buf, buf, buf, 256, 16, 64, buf, 0, ibuf, 4, 0, buf), CS_OK);
    EXPECT(cs_block_ffn(ctx, CS_BF16, buf, buf, buf, 256, 16, 64, buf, 2, NULL, 0, 0, buf), CS_OK);     /* empty support: zero fill */
    EXPECT(cs_block_ffn(ctx, CS_BF16, buf, buf, buf, 256, 16, 64, buf, 2, ibuf, 4, 0, buf), CS_OK);
    EXPECT(cs_block_ffn(ctx, CS_BF16, buf, buf, buf, 4096, 172, 64, buf, 4000, ibuf, 43, 0, buf), CS_ENOMEM);   /* 1 MiB of scratch */
    EXPECT(cs_block_ffn_static(ctx, CS_BF16, buf, buf, buf, 256, 16, 64, buf, 2, ibuf, 4, 0, buf), CS_OK);
    EXPECT(cs_block_ffn_static(ctx, CS_BF16, buf, buf, buf, 4096, 172, 64, buf, 4000, ibuf, 43, 0, buf), CS_ENOMEM);
    EXPECT(cs_block_ffn_static(NULL, CS_BF16, buf, buf, buf, 256, 16, 64, buf, 2, ibuf, 4, 0, buf), CS_EINVAL);
    EXPECT(cs_head_attn(ctx, CS_BF16, buf, buf, buf, 2, 8, 100, 96, ibuf, 3, buf), CS_EINVAL);
    EXPECT(cs_head_attn(ctx, CS_BF16, buf, buf, buf, 2, 8, 0, 128, ibuf, 3, buf), CS_EINVAL);
    EXPECT(cs_head_attn(ctx, CS_BF16, buf, buf, buf, 2, 8, 100, 128, ibuf, 9, buf), CS_EINVAL);
    EXPECT(cs_head_attn(ctx, CS_BF16, buf, buf, buf, 2, 8, 100, 128, NULL, 3, buf), CS_EINVAL);
    EXPECT(cs_head_attn(ctx, CS_BF16, buf, buf, buf, 2, 8, 100, 128, ibuf, 3, odd), CS_EALIGN);
    EXPECT(cs_head_attn(ctx, CS_BF16, buf, buf, buf, 0, 8, 100, 128, ibuf, 3, buf), CS_OK);
    EXPECT(cs_head_attn(ctx, CS_BF16, buf, buf, buf, 2, 8, 100, 128, ibuf, 3, buf), CS_OK);
    EXPECT(cs_head_attn(ctx, CS_BF16, buf, buf, buf, 60000, 32, 100, 128, ibuf, 32, buf), CS_ENOMEM);

    /* joint selection, entropy, budget, gather, probe */
    cs_op tok = { CS_RADEMACHER, 3u, 9u, 32, 512 };
    EXPECT(cs_joint_select(ctx, &tok, buf, 0, &op, &dct, buf, 4, ibuf, ibuf, buf, buf), CS_EINVAL);
    EXPECT(cs_joint_select(ctx, &tok, buf, 513, &op, &dct, buf, 4, ibuf, ibuf, buf, buf), CS_EINVAL);
    EXPECT(cs_joint_select(ctx, &tok, buf, 100, &op, &dct, buf, 4, NULL, ibuf, buf, buf), CS_EINVAL);
    EXPECT(cs_joint_select(ctx, &tok, buf, 100, &op, &dct, buf, 4, ibuf, ibuf, NULL, NULL), CS_OK);
    EXPECT(cs_joint_select_coupled(ctx, &tok, buf, 100, &op, &dct, NULL, 4, ibuf, ibuf, buf, buf, buf), CS_EINVAL);
    EXPECT(cs_joint_select_coupled(ctx, &tok, buf, 100, &op, &dct, buf, 4, ibuf, ibuf, NULL, NULL, NULL), CS_OK);
    EXPECT(cs_softmax_entropy(ctx, buf, 2, 0, buf), CS_EINVAL);
    EXPECT(cs_softmax_entropy(ctx, buf, 70000, 10, buf), CS_EINVAL);
    EXPECT(cs_softmax_entropy(ctx, buf, 2, 1000, buf), CS_OK);
    if (cs_uds_budget(256, 0.5f, 2.0f, 64, 512) != 512) ++failures;
    if (cs_uds_budget(256, 0.5f, 0.5f, 64, 512) != 320) ++failures;
    if (cs_uds_budget(256, 0.5f, 0.5f, 600, 512) != -1) ++failures;
    if (cs_uds_budget(256, 0.5f, 0.0f / 0.0f, 64, 512) != -1) ++failures;
    EXPECT(cs_gather_rows(ctx, CS_BF16, buf, 100, 250, ibuf, 4, buf), CS_EINVAL);
    EXPECT(cs_gather_rows(ctx, CS_BF16, buf, 100, 256, ibuf, 0, buf), CS_OK);
    EXPECT(cs_gather_rows(ctx, CS_BF16, buf, 100, 256, ibuf, 4, buf), CS_OK);
    EXPECT(cs_stream_read(ctx, odd, 64, (uint32_t*)ibuf), CS_EALIGN);
    EXPECT(cs_stream_read(ctx, buf, 0, NULL), CS_OK);
    EXPECT(cs_stream_read(ctx, buf, 4096, (uint32_t*)ibuf), CS_OK);
    EXPECT(cs_set_stream(ctx, NULL), CS_OK);
    EXPECT(cs_set_stream(NULL, NULL), CS_EINVAL);
    EXPECT(cs_set_union_hint(ctx, CS_UNION_DENSE), CS_OK);
    EXPECT(cs_set_union_hint(ctx, 3), CS_EINVAL);
    EXPECT(cs_set_union_hint(NULL, CS_UNION_AUTO), CS_EINVAL);
    EXPECT(cs_set_union_hint(ctx, CS_UNION_AUTO), CS_OK);

    /* many plans: the cache grows and moves; everything is released at the end */
    for (uint32_t s = 100; s < 140; ++s) {
        cs_op o = op; o.stream_id = s;
        EXPECT(cs_plan(ctx, &o, &dct), CS_OK);
    }
    for (uint32_t s = 100; s < 140; s += 3) {
        cs_op o = op; o.stream_id = s;
        EXPECT(cs_plan_drop(ctx, &o, &dct), CS_OK);
    }
    cs_destroy(ctx);
    cs_destroy(NULL);
    if (hip_standin_live_allocations != 0) { fprintf(stderr, "%zu device allocations leaked\n", hip_standin_live_allocations); ++failures; }
    if (standin_launches == 0) ++failures;
    free(buf); free(ibuf);
    if (failures) { fprintf(stderr, "%d failures\n", failures); return 1; }
    printf("host ABI checks passed (%d launches requested)\n", standin_launches);
    return 0;
}
