/* A plain C99 client of the resharding library: everything it does goes through the
 * declarations of reshard.h alone (host-side calls only, so it runs without a GPU).
 * It prints one line per fact; the Python test compares the lines with what the
 * ctypes binding reports for the same workload. */
#include <stdio.h>
#include <string.h>

#include "reshard.h"

int main(void) {
    reshard_model_spec spec;
    reshard_layout src, dst;
    reshard_plan *plan = NULL;
    reshard_plan_info info;
    reshard_mem_stats_t st;
    reshard_desc d0;
    int64_t cls[3];
    int i, n, rc;

    memset(&spec, 0, sizeof spec);
    memset(&src, 0, sizeof src);
    memset(&dst, 0, sizeof dst);
    /* the toy dense decoder: 2 layers, hidden 256, 4 query / 2 KV heads of 64, FFN 688, vocabulary 1024 */
    spec.struct_size = sizeof spec;
    spec.family = RESHARD_DENSE_GQA;
    spec.L = 2; spec.H = 256; spec.nq = 4; spec.nkv = 2; spec.d = 64; spec.I = 688; spec.V = 1024;
    spec.has_embeddings = 1;
    spec.elem_bytes = 2;
    src.struct_size = sizeof src;
    src.kind = RESHARD_TRAIN; src.tp = 2; src.pp = 1; src.ep = 1;
    src.tp_rank_filter = src.ep_rank_filter = -1;
    dst = src;
    dst.kind = RESHARD_GEN; dst.tp = 1;

    /* error paths first: they must not crash and must leave a message */
    rc = reshard_plan_create(&spec, &src, &dst, NULL);
    printf("create_null_out %d %d\n", rc, (int)(strlen(reshard_last_error()) > 0));
    src.tp = 3;
    rc = reshard_plan_create(&spec, &src, &dst, &plan);
    printf("create_tp3 %d %d\n", rc, plan == NULL);
    src.tp = 2;
    spec.struct_size = 4;
    rc = reshard_plan_create(&spec, &src, &dst, &plan);
    printf("create_bad_size %d\n", rc);
    spec.struct_size = sizeof spec;

    rc = reshard_plan_create(&spec, &src, &dst, &plan);
    printf("create %d\n", rc);
    if (rc != RESHARD_OK) return 1;
    for (i = 0; i < 2; ++i) {
        n = reshard_plan_num_bufs(plan, i);
        printf("num_bufs %d %d\n", i, n);
        for (int b = 0; b < n; ++b)
            printf("buf %d %d %lld %d\n", i, b, (long long)reshard_plan_buf_bytes(plan, i, b), reshard_plan_buf_used(plan, i, b));
    }
    rc = reshard_plan_get_info(plan, &info);
    printf("info %d %lld %lld %lld\n", rc, (long long)info.num_descs, (long long)info.num_tiles, (long long)info.bytes_moved);
    rc = reshard_plan_desc(plan, 0, &d0);
    printf("desc0 %d %d %d %lld %lld %lld %lld\n", rc, d0.src_buf, d0.dst_buf, (long long)d0.src_off, (long long)d0.dst_off,
           (long long)d0.rows, (long long)d0.row_bytes);
    printf("desc_out_of_range %d\n", reshard_plan_desc(plan, info.num_descs, &d0));
    rc = reshard_plan_class_bytes(plan, 1, cls);
    printf("class_bytes %d %lld %lld %lld\n", rc, (long long)cls[0], (long long)cls[1], (long long)cls[2]);
    rc = reshard_mem_stats(plan, &st);
    printf("mem_stats %d %lld %lld %d\n", rc, (long long)st.src_live, (long long)st.dst_live, st.state);
    /* nothing is bound: the swap calls must refuse, not crash */
    printf("swap_out_unbound %d\n", reshard_swap_out(plan, NULL));
    printf("swap_in_unbound %d\n", reshard_swap_in(plan, NULL));
    printf("tensors %lld\n", (long long)reshard_plan_num_tensors(plan, 1));
    printf("eq3 %.1f\n", reshard_redundant_memory_bytes(2, 8e9, 4, 4e9, 2));
    printf("destroy %d\n", reshard_plan_destroy(plan));
    printf("version %s\n", reshard_version());
    return 0;
}
