// Evaluation of a gradient through its derived expressions (Sec. 5.3): the seed expressions first, then every part
// with the forward kernels of its own plan; the parts after the first are added to the result in a fixed order.
#include <hip/hip_runtime.h>

#include "derived.hpp"
#include "profile.h"

namespace tad {

template <class T>
__global__ __launch_bounds__(256) void k_add_inplace(T *__restrict__ dst, const T *__restrict__ src, long long n) {
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i < n) dst[i] += src[i];
}

}  // namespace tad

using namespace tad;

extern "C" int tad_eval_derived(const tad_derived *d, const void *const *args_dev, const void *df_dev, void *dx_dev,
                                void *ws_dev, size_t ws_bytes, void *stream) {
    if (!d || !args_dev || !df_dev || !dx_dev) return TAD_EINVAL;
    for (int q = 0; q < d->n_original; ++q)
        if (!args_dev[d->root[(size_t)q]]) return TAD_EINVAL;
    if (d->ws_bytes && (!ws_dev || ws_bytes < d->ws_bytes)) return TAD_ENOMEM;
    char *ws = static_cast<char *>(ws_dev);
    hipStream_t s = static_cast<hipStream_t>(stream);
    auto source = [&](int src) -> const void * {
        if (src == kSrcDf) return df_dev;
        if (src >= 0) return args_dev[d->root[(size_t)src]];
        for (const auto &seed : d->seeds)
            if (seed.seed == src) return ws + seed.out_offset;
        return nullptr;
    };
    const void *ptrs[TAD_MAX_ARGS];
    auto run = [&](const tad_derived::Node &node, void *out) -> int {
        for (size_t q = 0; q < node.src.size(); ++q) {
            ptrs[q] = source(node.src[q]);
            if (!ptrs[q]) return TAD_EINVAL;
        }
        return tad_eval_forward(node.plan, ptrs, out, ws + d->sub_offset, ws_bytes - d->sub_offset, stream);
    };
    for (const auto &seed : d->seeds) {
        const int rc = run(seed, ws + seed.out_offset);
        if (rc) return rc;
    }
    for (size_t t = 0; t < d->parts.size(); ++t) {
        void *out = t == 0 ? dx_dev : ws + d->tmp_offset;
        const int rc = run(d->parts[t], out);
        if (rc) return rc;
        if (t > 0) {
            const dim3 grid((unsigned)((d->count + 255) / 256));
            if (d->dtype == TAD_F64)
                TAD_LAUNCH("k_add_inplace", (k_add_inplace<double>), grid, dim3(256), 0, s, (double *)dx_dev,
                           (const double *)out, (long long)d->count);
            else
                TAD_LAUNCH("k_add_inplace", (k_add_inplace<float>), grid, dim3(256), 0, s, (float *)dx_dev,
                           (const float *)out, (long long)d->count);
            if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
        }
    }
    return TAD_OK;
}
