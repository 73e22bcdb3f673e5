// Host-only check of the launch-policy code (no GPU is touched): for a grid of rank counts, buffer
// sizes, element types and launch options, stragglar_plan_launch_form must report a positive
// launch count and a positive byte count for every schedule - except the preconditions of two
// ranks, which have no ops.  Meant to be built with the address and undefined-behaviour
// sanitizers on the host side, which is what makes it worth running: every index into the
// schedules' per-chunk lists, group tables and model tables is exercised.
#include <cstdio>

#include "stragglar.h"

int main() {
    const int ns[] = {2, 8, 16, 32, 34, 64, 256};
    const size_t mibs[] = {1, 64, 256, 2048};
    long checked = 0;
    for (int n : ns)
        for (size_t mib : mibs)
            for (int dtype = 0; dtype < 3; dtype += 2) {
                sar_plan* p = nullptr;
                const size_t count = (mib << 20) / (dtype == SAR_BF16 ? 2 : 4) + 3;
                if (stragglar_plan(n, n / 3, count, dtype, &p) != SAR_OK) {
                    std::printf("plan failed: n=%d, %zu MiB\n", n, mib);
                    return 1;
                }
                for (int fuse = -1; fuse <= 1; ++fuse)
                    for (int split = -1; split <= 1; ++split)
                        for (int direct = -1; direct <= 1; ++direct)
                            for (int merge = 0; merge <= 1; ++merge) {
                                stragglar_plan_option_set(p, SAR_TUNE_FUSE_ROUNDS, fuse);
                                stragglar_plan_option_set(p, SAR_TUNE_FUSED_SPLIT, split);
                                stragglar_plan_option_set(p, SAR_TUNE_FUSED_DIRECT, direct);
                                stragglar_plan_option_set(p, SAR_TUNE_MERGE_COPIES, merge);
                                for (int which = 0; which < SAR_NUM_SCHEDULES; ++which) {
                                    if (which == SAR_SCHED_RHD && (n & (n - 1))) continue;
                                    sar_launch_form f;
                                    if (stragglar_plan_launch_form(p, which, &f) != SAR_OK) {
                                        std::printf("launch_form failed: n=%d which=%d\n", n, which);
                                        return 1;
                                    }
                                    const bool empty = n == 2 && (which == SAR_SCHED_PRECONDITION || which == SAR_SCHED_BCAST_PRECONDITION);
                                    if (empty ? (f.launches != 0 || f.bytes_stored != 0) : (f.launches <= 0 || f.bytes_stored == 0 || f.bytes_loaded == 0)) {
                                        std::printf("n=%d, %zu MiB, schedule %d: form %d, %d launches, %llu + %llu bytes\n", n, mib, which,
                                                    f.form, f.launches, f.bytes_loaded, f.bytes_stored);
                                        return 1;
                                    }
                                    ++checked;
                                }
                            }
                stragglar_plan_destroy(p);
            }
    std::printf("%ld launch forms ok\n", checked);
    return 0;
}
