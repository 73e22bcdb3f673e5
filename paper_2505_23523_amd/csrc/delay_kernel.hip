// Straggler emulation: a kernel that idles for a requested wall-clock time.
//
// Sec. 4.1 simulates a straggler by idling one rank for a number of clock
// cycles while the other ranks start the precondition.  Here the "late rank" is
// a stream: this kernel holds it (one wavefront, asleep most of the time) while
// the precondition runs on another stream of the same GPU.
//
// The wait is bounded twice: by the constant-rate wall clock and by an iteration
// limit derived from the requested time, so the wavefront always exits.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "launch.hpp"

namespace {

__global__ __launch_bounds__(64) void delay_kernel(uint64_t ticks, uint64_t max_iters) {
    const uint64_t t0 = wall_clock64();
    for (uint64_t it = 0; it < max_iters; ++it) {
        if (wall_clock64() - t0 >= ticks) break;
        __builtin_amdgcn_s_sleep(16);
    }
}

}  // namespace

int sar::enqueue_delay(uint64_t nanoseconds, void* hip_stream) {
    int dev = 0, khz = 0;
    if (hipGetDevice(&dev) != hipSuccess) return SAR_EDEVICE;
    if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess || khz <= 0)
        return SAR_EDEVICE;
    const uint64_t ticks = nanoseconds * uint64_t(khz) / 1000000u;
    // one iteration sleeps 16 * 64 clocks: at least ~0.3 us at any clock the part runs at;
    // the limit gives the clock test eight times the requested time before giving up
    const uint64_t max_iters = nanoseconds / 40u + 1000u;
    hipLaunchKernelGGL(delay_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(hip_stream), ticks, max_iters);
    return hipGetLastError() == hipSuccess ? SAR_OK : SAR_EDEVICE;
}

int sar::stream_wait_event(void* hip_stream, void* hip_event) {
    const hipError_t err =
        hipStreamWaitEvent(static_cast<hipStream_t>(hip_stream), static_cast<hipEvent_t>(hip_event), 0);
    return err == hipSuccess ? SAR_OK : SAR_EDEVICE;
}
