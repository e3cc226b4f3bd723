// Which HIP streams share a hardware queue.
//
// A process gets a small number of hardware queues; the runtime deals streams onto them as it sees fit, and not
// evenly.  Work on two streams of one queue runs one after the other even when nothing orders it, and an event wait
// at the head of the queue holds up both.  K virtual workers spread unevenly over the queues (say 1, 2, 2 and 3 of
// 8) lose a tenth of the aggregate throughput against an even spread, so the caller needs to know the grouping.
// No call reports it; it is measured: a kernel that spins for a few milliseconds goes onto one stream, a kernel that
// reads the clock onto another, and if that reading is later than the end of the spin, the second waited for the first.
#include <hip/hip_runtime.h>

#include <vector>

#include "../../include/dssp.h"

namespace {

// Leaves after `ticks` of the constant-rate wall clock and notes when; the iteration count bounds it even if the
// clock stood still.
__global__ void spin_kernel(unsigned long long ticks, unsigned long long* left_at) {
    const unsigned long long t0 = wall_clock64();
    for (int i = 0; i < (1 << 16); ++i) {
        if (wall_clock64() - t0 >= ticks) break;
        __builtin_amdgcn_s_sleep(64);
    }
    if (threadIdx.x == 0) *left_at = wall_clock64();
}

__global__ void stamp_kernel(unsigned long long* ran_at) {
    if (threadIdx.x == 0) *ran_at = wall_clock64();
}

#define Q_TRY(x) do { if ((x) != hipSuccess) return DSSP_EHIP; } while (0)

// 1 if b's work waits for a's, 0 if not, < 0 on error.  Both streams are idle on entry and on return.  The answer
// comes from the device's own clock: the stamp on b is taken either well before the spin on a has ended or after it.
int waits_behind(hipStream_t a, hipStream_t b, unsigned long long ticks, unsigned long long* clocks_dev) {
    for (int round = 0; round < 2; ++round) {      // a host thread stalled between the two launches can fake one "yes"
        hipLaunchKernelGGL(spin_kernel, dim3(1), dim3(64), 0, a, ticks, clocks_dev);
        hipLaunchKernelGGL(stamp_kernel, dim3(1), dim3(64), 0, b, clocks_dev + 1);
        Q_TRY(hipGetLastError());
        Q_TRY(hipStreamSynchronize(b));
        Q_TRY(hipStreamSynchronize(a));
        unsigned long long t[2];
        Q_TRY(hipMemcpy(t, clocks_dev, sizeof t, hipMemcpyDeviceToHost));
        if (t[1] < t[0]) return 0;
    }
    return 1;
}

struct DeviceClocks {
    unsigned long long* p = nullptr;
    ~DeviceClocks() { if (p) (void)hipFree(p); }
};

}  // namespace

extern "C" int dssp_stream_queues(void* const* hip_streams, int n, int* queue_out, int* n_queues_out) {
    if (!hip_streams || !queue_out || n < 1 || n > 64) return DSSP_EINVAL;
    int dev = 0, khz = 0;
    Q_TRY(hipGetDevice(&dev));
    Q_TRY(hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev));
    if (khz <= 0) khz = 100000;
    const unsigned long long ticks = 2ull * (unsigned long long)khz;       // 2 ms
    DeviceClocks clocks;
    Q_TRY(hipMalloc(&clocks.p, 2 * sizeof(unsigned long long)));
    std::vector<hipStream_t> s(n);
    for (int i = 0; i < n; ++i) s[i] = (hipStream_t)hip_streams[i];
    // first use binds a stream to its queue and loads the kernels
    for (int i = 0; i < n; ++i) {
        hipLaunchKernelGGL(spin_kernel, dim3(1), dim3(64), 0, s[i], 1ull, clocks.p);
        hipLaunchKernelGGL(stamp_kernel, dim3(1), dim3(64), 0, s[i], clocks.p + 1);
        Q_TRY(hipGetLastError());
        Q_TRY(hipStreamSynchronize(s[i]));
    }
    std::vector<int> first;            // first stream found on each queue
    for (int i = 0; i < n; ++i) {
        int q = -1;
        for (int j = 0; j < i && q < 0; ++j)
            if (s[j] == s[i]) q = queue_out[j];
        for (size_t g = 0; g < first.size() && q < 0; ++g) {
            const int w = waits_behind(s[first[g]], s[i], ticks, clocks.p);
            if (w < 0) return w;
            if (w) q = (int)g;
        }
        if (q < 0) { q = (int)first.size(); first.push_back(i); }
        queue_out[i] = q;
    }
    if (n_queues_out) *n_queues_out = (int)first.size();
    return DSSP_OK;
}
