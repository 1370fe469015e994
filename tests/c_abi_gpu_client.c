/* A GPU client of the resharding library written in plain C: device memory from the HIP
 * runtime, no Python and no tensor framework anywhere.  It reshards the toy dense workload
 * (TP2 -> TP1), swaps the sources out and back in, and writes the destination buffer and the
 * returned sources to a file; the Python test compares them with the CPU oracle run on the
 * same inputs.  Inputs: word i of source buffer b is (i * 2654435761 + b * 40503) >> 9,
 * truncated to 16 bits (the test generates the same words). */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "reshard.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 2; } } while (0)
#define CHECK_RS(x) do { int r_ = (x); if (r_ != RESHARD_OK) { fprintf(stderr, "reshard error %d (%s) at line %d\n", r_, reshard_last_error(), __LINE__); return 3; } } while (0)

int main(int argc, char **argv) {
    reshard_model_spec spec;
    reshard_layout src, dst;
    reshard_plan *plan = NULL;
    reshard_mem_stats_t st;
    void *sp[2] = {NULL, NULL}, *dp[1] = {NULL};
    const void *csp[2];
    uint16_t *host[2], *out;
    int64_t sbytes[2], dbytes;
    hipStream_t stream;
    FILE *f;
    int b;

    if (argc < 2) { fprintf(stderr, "usage: %s output-file\n", argv[0]); return 1; }
    memset(&spec, 0, sizeof spec);
    memset(&src, 0, sizeof src);
    spec.struct_size = sizeof spec;
    spec.family = RESHARD_DENSE_GQA;
    spec.L = 2; spec.H = 256; spec.nq = 4; spec.nkv = 2; spec.d = 64; spec.I = 688; spec.V = 1024;
    spec.has_embeddings = 1; spec.elem_bytes = 2;
    src.struct_size = sizeof src;
    src.kind = RESHARD_TRAIN; src.tp = 2; src.pp = 1; src.ep = 1; src.tp_rank_filter = src.ep_rank_filter = -1;
    dst = src;
    dst.kind = RESHARD_GEN; dst.tp = 1;
    CHECK_RS(reshard_plan_create(&spec, &src, &dst, &plan));
    if (reshard_plan_num_bufs(plan, 0) != 2 || reshard_plan_num_bufs(plan, 1) != 1) return 4;
    CHECK_HIP(hipSetDevice(0));
    CHECK_HIP(hipStreamCreate(&stream));
    for (b = 0; b < 2; ++b) {
        int64_t i, n;
        sbytes[b] = reshard_plan_buf_bytes(plan, 0, b);
        n = sbytes[b] / 2;
        host[b] = (uint16_t *)malloc((size_t)sbytes[b]);
        if (!host[b]) return 5;
        for (i = 0; i < n; ++i) host[b][i] = (uint16_t)(((uint64_t)i * 2654435761u + (uint64_t)b * 40503u) >> 9);
        CHECK_HIP(hipMalloc(&sp[b], (size_t)sbytes[b]));
        CHECK_HIP(hipMemcpy(sp[b], host[b], (size_t)sbytes[b], hipMemcpyHostToDevice));
        csp[b] = sp[b];
    }
    dbytes = reshard_plan_buf_bytes(plan, 1, 0);
    CHECK_HIP(hipMalloc(&dp[0], (size_t)dbytes));
    CHECK_HIP(hipMemset(dp[0], 0xA5, (size_t)dbytes));
    out = (uint16_t *)malloc((size_t)dbytes);
    if (!out) return 5;

    CHECK_RS(reshard_execute(plan, csp, dp, stream));          /* select and copy */
    CHECK_RS(reshard_swap_out(plan, stream));                  /* training copy to pinned host memory */
    CHECK_RS(reshard_swap_wait(plan));
    CHECK_RS(reshard_mark_src_released(plan));
    CHECK_RS(reshard_mem_stats(plan, &st));
    if (st.src_live != 0 || st.released != sbytes[0] + sbytes[1] || st.peak_device != sbytes[0] + sbytes[1] + dbytes) return 6;
    for (b = 0; b < 2; ++b) {                                  /* the caller really drops and re-creates it */
        CHECK_HIP(hipFree(sp[b]));
        CHECK_HIP(hipMalloc(&sp[b], (size_t)sbytes[b]));
        CHECK_HIP(hipMemset(sp[b], 0, (size_t)sbytes[b]));
        csp[b] = sp[b];
    }
    CHECK_RS(reshard_bind_src(plan, csp));
    CHECK_RS(reshard_swap_in(plan, stream));                   /* and back before the next update */
    CHECK_RS(reshard_swap_wait(plan));
    CHECK_HIP(hipStreamSynchronize(stream));

    f = fopen(argv[1], "wb");
    if (!f) return 7;
    CHECK_HIP(hipMemcpy(out, dp[0], (size_t)dbytes, hipMemcpyDeviceToHost));
    fwrite(out, 1, (size_t)dbytes, f);
    for (b = 0; b < 2; ++b) {
        CHECK_HIP(hipMemcpy(host[b], sp[b], (size_t)sbytes[b], hipMemcpyDeviceToHost));
        fwrite(host[b], 1, (size_t)sbytes[b], f);
    }
    fclose(f);
    CHECK_RS(reshard_plan_destroy(plan));
    printf("ok %lld %lld %lld\n", (long long)dbytes, (long long)sbytes[0], (long long)sbytes[1]);
    return 0;
}
