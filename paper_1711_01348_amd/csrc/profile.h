// Optional per-kernel timing with HIP events (tad_profile_begin / tad_profile_end).
// When a kernel name is armed, every launch of that kernel is bracketed by a pair of events recorded
// on the stream the kernel is launched on.
#pragma once
#include <hip/hip_runtime.h>

namespace tad {

struct ProfileScope {
    ProfileScope(const char *name, hipStream_t s);
    ~ProfileScope();
    int slot;
    hipStream_t stream;
};

}  // namespace tad

// A launch is checked with hipGetLastError() right after it; an error left behind by an earlier, unrelated
// runtime call of this thread is discarded first so that it is not mistaken for a launch failure.
#define TAD_LAUNCH(name, kernel, grid, block, shmem, stream, ...)              \
    do {                                                                       \
        (void)hipGetLastError();                                               \
        tad::ProfileScope _ps(name, stream);                                   \
        hipLaunchKernelGGL(kernel, grid, block, shmem, stream, __VA_ARGS__);   \
    } while (0)
