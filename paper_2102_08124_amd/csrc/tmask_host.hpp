// Host-side helpers shared by the translation units of libtmask.so.
#pragma once
#include <hip/hip_runtime.h>

#include "../../include/tmask.h"
#include "tmask_device.hpp"

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

// Second-stage reductions (tmask_kernels.hip) for kernels of other translation units: first0[k] = index, inside the
// launch, of the first partial result of matrix k; first0[nb] = their number.
int launch_objective_reduce(double *const *objective, const uint32_t *first0, int nb, uint32_t partial0, const void *partials,
                            hipStream_t stream);
int launch_score_reduce(const uint32_t *first0, int nb, uint32_t partial0, const void *partials, tmask_score_out *out,
                        hipStream_t stream);

// The column-per-lane kernels (tmask_colwise.hip): M = 32, and matrices that miss the strip kernels' alignment.
// Arguments are validated by the callers.  solver: 0 = Algorithm 1, 1 = exact, 2 = row pruning; dense mode: 0 =
// Algorithm 1, 1 = row pruning, 2 = row pruning with mean absorption.
int cw_run_mask(int solver, const tmask_mat *mats, int n_mats, int dt, int N, int M, int mf, void *ws, hipStream_t stream);
int cw_run_score(const tmask_mat *mats, int n_mats, int dt, int N, int M, int mf, tmask_score_out *out, float *per_block_obj,
                 void *ws, hipStream_t stream);
int cw_run_pack(const tmask_pack_desc *descs, int n, int dt, int N, int M, int mf, hipStream_t stream);
int cw_run_dense(const tmask_mask_dense_desc *descs, int n, int dt, int N, int M, int mf, int mode, hipStream_t stream);
size_t cw_workgroups(int64_t rows, int64_t cols, int M);     // workgroups (= partial results) cw_run_mask uses for a matrix

// Fills the coarse index of a launch (see CoarseIndex): first0[k] = first workgroup of matrix k, n matrices,
// `total` workgroups.
inline void fill_coarse(CoarseIndex &ci, const uint32_t *first0, int n, uint32_t total)
{
    uint32_t shift = 0;
    while (total > 0 && ((total - 1u) >> shift) >= (uint32_t)kCoarse)
        shift++;
    ci.shift = shift;
    const uint32_t buckets = total ? ((total - 1u) >> shift) + 1u : 1u;
    uint32_t first[kCoarse + 1];
    int m = 0;
    for (uint32_t b = 0; b < buckets; b++) {
        const uint32_t t = b << shift;
        while (m + 1 < n && first0[m + 1] <= t)
            m++;
        first[b] = (uint32_t)m;
    }
    first[buckets] = (uint32_t)(n - 1);
    for (uint32_t b = 0; b < (uint32_t)kCoarse; b++)
        ci.e[b] = b < buckets ? (first[b] | (first[b + 1] << 16)) : 0u;
}

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
