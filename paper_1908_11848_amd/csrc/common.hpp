// Shared by the kernel files: launch checks and small device helpers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define DSSPK_LAUNCH_RC() ((int)hipGetLastError())

typedef float floatx4 __attribute__((ext_vector_type(4)));

static inline int ceil_div(long a, long b) { return (int)((a + b - 1) / b); }

// Number of workgroups that keeps every CU of the chip busy a few times over for a
// bandwidth-bound grid-stride kernel (256 CUs in 8 XCDs; workgroups are dealt to XCDs
// round-robin, so a multiple of 8 keeps the XCDs evenly loaded).
static inline int stream_grid(long items_per_block_total, int cap = 256 * 8) {
    long g = items_per_block_total;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
}
