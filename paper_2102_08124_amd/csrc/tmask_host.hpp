// Host-side helpers shared by the translation units of libtmask.so.
#pragma once
#include <hip/hip_runtime.h>

namespace tmask {

// Records a thread-local, human-readable description of the failure and returns `code`.
int fail(int code, const char *fmt, ...);
int hip_fail(hipError_t e, const char *what);

// One-shot profiling events (tmask_profile_next): recorded around the main kernel of the next call.
extern thread_local hipEvent_t g_prof_start, g_prof_stop;

struct ProfileScope {
    hipStream_t stream;
    bool active;
    ProfileScope(hipStream_t s, bool last_chunk) : stream(s), active(last_chunk && g_prof_start && g_prof_stop)
    {
        if (active)
            (void)hipEventRecord(g_prof_start, stream);
    }
    ~ProfileScope()
    {
        if (active) {
            (void)hipEventRecord(g_prof_stop, stream);
            g_prof_start = g_prof_stop = nullptr;
        }
    }
};

// Compute units of the current device (256 if the query fails); asked once per thread and device.
inline int cu_count()
{
    static thread_local int cached_dev = -1, cached = 256;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess)
        return 256;
    if (dev != cached_dev) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;
        cached = n;
        cached_dev = dev;
    }
    return cached;
}

}  // namespace tmask
