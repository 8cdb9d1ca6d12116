// Kernel launch with optional timing: when an event pair was armed (set_launch_events), it is attached to
// the dispatch itself, so the time between the two events is the kernel's own execution time.
#pragma once
#include <hip/hip_runtime.h>

#include <hip/hip_ext.h>

namespace ee {
bool take_launch_events(hipEvent_t* start, hipEvent_t* stop);  // true (and disarms) when a pair was armed
}

#define EE_LAUNCH_SM(kernel, grid, block, shmem, stream, ...)                                  \
    do {                                                                                       \
        hipEvent_t _a, _b;                                                                     \
        if (ee::take_launch_events(&_a, &_b)) {                                                \
            hipExtLaunchKernelGGL(kernel, grid, block, shmem, stream, _a, _b, 0, __VA_ARGS__); \
        } else {                                                                               \
            hipLaunchKernelGGL(kernel, grid, block, shmem, stream, __VA_ARGS__);               \
        }                                                                                      \
    } while (0)
#define EE_LAUNCH(kernel, grid, block, stream, ...) EE_LAUNCH_SM(kernel, grid, block, 0, stream, __VA_ARGS__)
