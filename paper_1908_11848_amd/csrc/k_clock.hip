// Device-side time for the wall-clock mode: the push timestamps Alg. 2 consumes are then real completion times of the
// workers' gradients, read from the GPU's constant-rate clock by a one-lane kernel behind each worker step, and a
// worker is made "slower" (Sec. V-C: a cluster of unequal GPUs) by a kernel that holds its stream until the iteration
// has lasted a given multiple of its real duration.  Waiting is bounded twice: by the clock (a cap on the extra time)
// and by an iteration count (in case the clock stood still), so every launch ends.
#include "common.hpp"
#include "../../include/dssp_kernels.h"

namespace {

constexpr int kSleepIterations = 1 << 16;       // x s_sleep(100), about 3 us each: ends after ~0.2 s whatever the clock says

__device__ __forceinline__ void publish(unsigned long long* p, unsigned long long v) {
    // may point to pinned host memory that the host polls
    __hip_atomic_store(p, v, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

__global__ void clock_stamp_kernel(unsigned long long* out_a, unsigned long long* out_b) {
    if (threadIdx.x == 0) {
        const unsigned long long t = wall_clock64();
        if (out_a) publish(out_a, t);
        if (out_b) publish(out_b, t);
    }
}

// start: tick at which the iteration began (written by clock_stamp_kernel earlier on the same stream).
// Leaves when (clock - start) >= permille / 1000 * (arrival - start), arrival = the tick this kernel started at, i.e.
// when everything enqueued before it had finished; never waits longer than max_extra ticks.
__global__ void clock_stretch_kernel(const unsigned long long* start, unsigned permille, unsigned long long max_extra,
                                     unsigned long long* arrival_out, unsigned long long* left_out) {
    if (threadIdx.x != 0) return;
    const unsigned long long t0 = *start, arrival = wall_clock64();
    const unsigned long long spent = arrival > t0 ? arrival - t0 : 0;
    unsigned long long extra = permille > 1000 ? spent / 1000 * (permille - 1000) + spent % 1000 * (permille - 1000) / 1000 : 0;
    if (extra > max_extra) extra = max_extra;
    const unsigned long long target = arrival + extra;
    unsigned long long now = arrival;
    for (int i = 0; i < kSleepIterations && now < target; ++i) {
        __builtin_amdgcn_s_sleep(100);
        now = wall_clock64();
    }
    if (arrival_out) publish(arrival_out, arrival);
    if (left_out) publish(left_out, now);
}

}  // namespace

extern "C" int dsspk_clock_khz(void) {
    int dev = 0, khz = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess) return -1;
    return khz > 0 ? khz : -1;
}

extern "C" int dsspk_clock_stamp(void* stream, uint64_t* out_a, uint64_t* out_b) {
    if (!out_a && !out_b) return -1;
    hipLaunchKernelGGL(clock_stamp_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, (unsigned long long*)out_a,
                       (unsigned long long*)out_b);
    return DSSPK_LAUNCH_RC();
}

extern "C" int dsspk_clock_stretch(void* stream, const uint64_t* start_dev, int permille, uint64_t max_extra_ticks,
                                   uint64_t* arrival_out, uint64_t* left_out) {
    if (!start_dev || permille < 0 || permille > 1000000 || (!arrival_out && !left_out)) return -1;
    hipLaunchKernelGGL(clock_stretch_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, (const unsigned long long*)start_dev,
                       (unsigned)permille, (unsigned long long)max_extra_ticks, (unsigned long long*)arrival_out,
                       (unsigned long long*)left_out);
    return DSSPK_LAUNCH_RC();
}
