// Shared host-side helpers of the C-ABI entry points (validation, launch checks) and
// the vector types the gfx950 kernels use.  Device code only; nothing here is shared
// with the CPU oracle.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include <atomic>

#include "awq_mi355x.h"

#define AWQ_GROUP 128
#define AWQ_TILE_ROWS 16
#define AWQ_TILE_BYTES 1024

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

static inline bool awq_aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Weight-shape rules common to quantize / unpack / linear.
static inline int awq_check_weight_shape(int64_t N, int64_t K, int group)
{
    if (group != AWQ_GROUP) return AWQ_ERR_UNSUPPORTED_GROUP;
    if (N <= 0 || K <= 0 || (K % AWQ_GROUP) != 0 || (N % AWQ_TILE_ROWS) != 0) return AWQ_ERR_BAD_SHAPE;
    // index arithmetic inside the kernels is 32-bit for tile counts
    if (N > (int64_t)1 << 24 || K > (int64_t)1 << 24 || (N / 16) * (K / 128) > (int64_t)1 << 30)
        return AWQ_ERR_BAD_SHAPE;
    return AWQ_OK;
}

static inline int awq_launch_status()
{
    return hipGetLastError() == hipSuccess ? AWQ_OK : AWQ_ERR_HIP;
}

// "Done once on this device" flag for settings that belong to a (kernel, device) pair, such as a
// raised dynamic-LDS limit.  Setting such a thing twice is harmless, so a relaxed atomic flag is
// enough: two host threads may both set it, none reads a torn value.
struct AwqOncePerDevice {
    std::atomic<bool> done[64] = {};
    std::atomic<bool> &here()
    {
        int dev = 0;
        (void)hipGetDevice(&dev);
        return done[dev & 63];
    }
};

// Planner constants that experiments override through the environment exist only in the tuning
// build of the library (-DAWQ_TUNING_KNOBS, libawq_mi355x_knobs.so); the shipped library reads no
// environment variable and always takes the default.
#ifdef AWQ_TUNING_KNOBS
static inline int awq_knob(const char *name, int dflt)
{
    const char *e = getenv(name);
    return e ? atoi(e) : dflt;
}
#else
static inline int awq_knob(const char *, int dflt) { return dflt; }
#endif
