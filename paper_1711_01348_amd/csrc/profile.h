// Optional per-kernel timing with HIP events (tad_profile_begin / tad_profile_end).
// When a kernel name is armed, every launch of that kernel carries a pair of events that the runtime
// attaches to the dispatch itself (hipExtLaunchKernelGGL): they take the kernel's own begin and end
// timestamps on the stream it runs on and put no extra packet into the queue.
#pragma once
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

namespace tad {

struct ProfileScope {
    explicit ProfileScope(const char *name);
    hipEvent_t start, stop;   // null unless this launch is being timed
};

}  // namespace tad

// A launch is checked with hipGetLastError() right after it; an error left behind by an earlier, unrelated
// runtime call of this thread is discarded first so that it is not mistaken for a launch failure.
#define TAD_LAUNCH(name, kernel, grid, block, shmem, stream, ...)              \
    do {                                                                       \
        (void)hipGetLastError();                                               \
        tad::ProfileScope _ps(name);                                           \
        if (_ps.start)                                                         \
            hipExtLaunchKernelGGL(kernel, grid, block, shmem, stream, _ps.start, _ps.stop, 0, __VA_ARGS__); \
        else /* the plain launch: the form a stream capture records */         \
            hipLaunchKernelGGL(kernel, grid, block, shmem, stream, __VA_ARGS__); \
    } while (0)
