/*
 * A C consumer of the library: no Python, no PyTorch.  Allocates n rank buffers
 * with hipMalloc, fills them with small integers (so every summation order is
 * exact), runs the precondition, the completion rounds and the baselines through
 * the C ABI, and compares every element of every rank with a plain sum computed
 * here on the host.  Exit status 0 = all equal.
 *
 * usage: c_abi_smoke [n] [count]
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "stragglar.h"

#define HIP_OK(x)                                                                  \
    do {                                                                           \
        hipError_t e_ = (x);                                                       \
        if (e_ != hipSuccess) {                                                    \
            fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_));         \
            return 2;                                                              \
        }                                                                          \
    } while (0)
#define SAR_OK_(x)                                                                 \
    do {                                                                           \
        int s_ = (x);                                                              \
        if (s_ != SAR_OK) {                                                        \
            fprintf(stderr, "%s failed: %s\n", #x, stragglar_strerror(s_));        \
            return 3;                                                              \
        }                                                                          \
    } while (0)

static uint32_t lcg(uint32_t* s) { return *s = *s * 1664525u + 1013904223u; }

static uint16_t small_int_to_bf16(int v) { /* |v| <= 127 is exact in bf16 */
    float f = (float)v;
    uint32_t u;
    memcpy(&u, &f, 4);
    return (uint16_t)(u >> 16);
}

static int run_case(int n, size_t count, int dtype, int straggler) {
    const size_t eb = dtype == SAR_BF16 ? 2 : 4;
    const size_t bytes = count * eb;
    void* dev[SAR_MAX_RANKS];
    void* pristine = malloc(bytes * (size_t)n);
    void* back = malloc(bytes);
    long* want = (long*)calloc(count, sizeof(long));
    if (!pristine || !back || !want) return 4;
    uint32_t seed = 12345u + (uint32_t)(n * 131 + dtype * 7 + straggler);
    for (int r = 0; r < n; ++r) {
        for (size_t e = 0; e < count; ++e) {
            const int v = (int)(lcg(&seed) >> 24) % 15 - 7;       /* -7 .. 7 */
            want[e] += v;
            char* p = (char*)pristine + (size_t)r * bytes + e * eb;
            if (dtype == SAR_I32) { int32_t x = v; memcpy(p, &x, 4); }
            else if (dtype == SAR_F32) { float x = (float)v; memcpy(p, &x, 4); }
            else { uint16_t x = small_int_to_bf16(v); memcpy(p, &x, 2); }
        }
    }
    for (int r = 0; r < n; ++r) HIP_OK(hipMalloc(&dev[r], bytes));
    sar_plan* plan = NULL;
    SAR_OK_(stragglar_plan(n, straggler, count, dtype, &plan));

    hipStream_t stream;
    HIP_OK(hipStreamCreate(&stream));
    int failures = 0;
    const int pow2 = (n & (n - 1)) == 0;
    /* the same plan in every form a call can take: per-plan options, checked through the
       launch-form query; algo 4..6 repeat StragglAR as merged copies / single launch / split */
    for (int algo = 0; algo < 7; ++algo) {
        if (algo == 2 && !pow2) continue;
        sar_launch_form form;
        SAR_OK_(stragglar_plan_option_set(plan, SAR_TUNE_FUSE_ROUNDS, algo >= 5 ? 1 : 0));
        SAR_OK_(stragglar_plan_option_set(plan, SAR_TUNE_MERGE_COPIES, algo == 4 ? 1 : 0));
        SAR_OK_(stragglar_plan_option_set(plan, SAR_TUNE_FUSED_SPLIT, algo == 6 ? 1 : 0));
        SAR_OK_(stragglar_plan_launch_form(plan, SAR_SCHED_COMPLETION, &form));
        if (form.form != (algo == 4 ? 1 : algo == 5 ? 2 : algo == 6 ? (n > 2 ? 3 : 2) : 0) || form.launches < 1 ||
            form.bytes_stored != (unsigned long long)n * bytes) {
            fprintf(stderr, "n=%d algo=%d: launch form %d, %d launches, %llu bytes stored\n", n, algo, form.form, form.launches, form.bytes_stored);
            ++failures;
        }
        for (int r = 0; r < n; ++r)
            HIP_OK(hipMemcpy(dev[r], (char*)pristine + (size_t)r * bytes, bytes, hipMemcpyHostToDevice));
        if (algo == 0 || algo >= 4) {
            SAR_OK_(stragglar_phase1_reducescatter(plan, dev, stream));
            SAR_OK_(stragglar_phase2_complete(plan, dev, stream));
        } else if (algo == 1) {
            SAR_OK_(ring_allreduce(plan, dev, stream));
        } else if (algo == 2) {
            SAR_OK_(rhd_allreduce(plan, dev, stream));
        } else {
            SAR_OK_(broadcast_phase1_allreduce(plan, dev, stream));
            SAR_OK_(broadcast_phase2_complete(plan, dev, stream));
        }
        HIP_OK(hipStreamSynchronize(stream));
        for (int r = 0; r < n; ++r) {
            HIP_OK(hipMemcpy(back, dev[r], bytes, hipMemcpyDeviceToHost));
            for (size_t e = 0; e < count; ++e) {
                long got;
                if (dtype == SAR_I32) { int32_t x; memcpy(&x, (char*)back + e * 4, 4); got = x; }
                else if (dtype == SAR_F32) { float x; memcpy(&x, (char*)back + e * 4, 4); got = (long)x; }
                else { uint16_t h; memcpy(&h, (char*)back + e * 2, 2); uint32_t u = (uint32_t)h << 16; float x; memcpy(&x, &u, 4); got = (long)x; }
                if (got != want[e]) {
                    if (failures < 5)
                        fprintf(stderr, "n=%d dtype=%d algo=%d rank %d elem %zu: got %ld want %ld\n", n, dtype, algo, r, e, got, want[e]);
                    ++failures;
                }
            }
        }
    }
    stragglar_plan_destroy(plan);
    HIP_OK(hipStreamDestroy(stream));
    for (int r = 0; r < n; ++r) HIP_OK(hipFree(dev[r]));
    free(pristine); free(back); free(want);
    return failures ? 1 : 0;
}

int main(int argc, char** argv) {
    const int n_arg = argc > 1 ? atoi(argv[1]) : 0;
    const size_t count = argc > 2 ? (size_t)strtoull(argv[2], NULL, 10) : 7 * 12000 + 5;
    const int ns[] = {2, 4, 6, 8, 16};
    int bad = 0, cases = 0;
    for (size_t i = 0; i < sizeof(ns) / sizeof(ns[0]); ++i) {
        const int n = n_arg ? n_arg : ns[i];
        for (int dtype = SAR_I32; dtype <= SAR_BF16; ++dtype) {
            const int rc = run_case(n, count * (size_t)n, dtype, n / 2);
            if (rc > 1) return rc;
            bad += rc;
            ++cases;
        }
        if (n_arg) break;
    }
    printf("c_abi_smoke: %d cases, %d failed\n", cases, bad);
    return bad ? 1 : 0;
}
