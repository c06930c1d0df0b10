// Device entry points of the C ABI: dispatch on the kernel family chosen at plan time.
#include <hip/hip_runtime.h>

#include <mutex>

#include "launch.h"

using namespace tad;

// Scratch memory of tad_eval_backward_static: one array per GPU, part of the loaded code object, held until the
// process ends.  In host code the array's name only stands for the symbol; its device address is looked up once per
// device with hipGetSymbolAddress and that pointer is what the kernels get.
static __device__ __align__(256) unsigned char scratch[TAD_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];

int static_scratch(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return TAD_EDEVICE;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return TAD_EDEVICE;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return TAD_OK;
}
}  // namespace

extern "C" {

int tad_eval_forward(const tad_plan *plan, const void *const *args_dev, void *f_dev, void *ws_dev,
                     size_t ws_bytes, void *stream) {
    if (!plan || !args_dev || !f_dev) return TAD_EINVAL;
    for (size_t p = 0; p < plan->args.size(); ++p)
        if (!args_dev[plan->root[p]]) return TAD_EINVAL;
    if (plan->ws_bytes && (!ws_dev || ws_bytes < plan->ws_bytes)) return TAD_ENOMEM;
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (plan->fwd_family) {
    case TAD_FAMILY_GENERIC: return generic_forward(*plan, args_dev, f_dev, ws_dev, s);
    case TAD_FAMILY_WORKED: return worked_forward(*plan, args_dev, f_dev, s);
    case TAD_FAMILY_WORKED_MFMA: return mfma_forward(*plan, args_dev, f_dev, ws_dev, s);
    case TAD_FAMILY_ROW_REDUCE:
    case TAD_FAMILY_DIAGONAL:
    case TAD_FAMILY_ANTIDIAGONAL: return pattern_forward(*plan, args_dev, f_dev, s);
    case TAD_FAMILY_STRIDED: return strided_forward(*plan, args_dev, f_dev, s);
    case TAD_FAMILY_CONTRACTION: return contract_forward(*plan, args_dev, f_dev, ws_dev, s);
    case TAD_FAMILY_PROGRAM: return program_forward(*plan, args_dev, f_dev, ws_dev, s);
    default: return TAD_EUNSUPPORTED;
    }
}

int tad_eval_backward(const tad_plan *plan, const void *const *args_dev, const void *f_dev,
                      const void *df_dev, void *const *dx_dev, void *ws_dev, size_t ws_bytes, void *stream) {
    if (!plan || !args_dev || !f_dev || !df_dev || !dx_dev) return TAD_EINVAL;
    for (size_t p = 0; p < plan->args.size(); ++p) {
        if (!args_dev[plan->root[p]]) return TAD_EINVAL;
        if (dx_dev[p] && (!plan->ap[p].derived || plan->root[p] != (int)p)) return TAD_EINVAL;  // not planned / alias
    }
    if (plan->ws_bytes && (!ws_dev || ws_bytes < plan->ws_bytes)) return TAD_ENOMEM;
    hipStream_t s = static_cast<hipStream_t>(stream);
    bool any_wanted = false;
    for (size_t p = 0; p < plan->args.size(); ++p) any_wanted |= dx_dev[p] != nullptr;
    if (!any_wanted) return TAD_OK;
    // a specialised family owns all gradients of its expression; anything left is generic
    int fam = TAD_FAMILY_GENERIC;
    for (size_t p = 0; p < plan->args.size(); ++p)
        if (plan->ap[p].derived && plan->ap[p].family != TAD_FAMILY_GENERIC) fam = plan->ap[p].family;
    switch (fam) {
    case TAD_FAMILY_GENERIC: return generic_backward(*plan, args_dev, f_dev, df_dev, dx_dev, ws_dev, s);
    case TAD_FAMILY_WORKED: return worked_backward(*plan, args_dev, f_dev, df_dev, dx_dev, ws_dev, s);
    case TAD_FAMILY_WORKED_MFMA: return mfma_backward(*plan, args_dev, f_dev, df_dev, dx_dev, ws_dev, s);
    case TAD_FAMILY_ROW_REDUCE:
    case TAD_FAMILY_DIAGONAL:
    case TAD_FAMILY_ANTIDIAGONAL: return pattern_backward(*plan, args_dev, df_dev, dx_dev, ws_dev, s);
    case TAD_FAMILY_STRIDED: return strided_backward(*plan, args_dev, f_dev, df_dev, dx_dev, ws_dev, s);
    case TAD_FAMILY_CONTRACTION: return contract_backward(*plan, args_dev, df_dev, dx_dev, ws_dev, s);
    case TAD_FAMILY_PROGRAM: return program_backward(*plan, args_dev, df_dev, dx_dev, ws_dev, s);
    default: return TAD_EUNSUPPORTED;
    }
}

int tad_eval_backward_static(const tad_plan *plan, const void *const *args_dev, const void *f_dev,
                             const void *df_dev, void *const *dx_dev, void *stream) {
    if (!plan) return TAD_EINVAL;
    if (plan->ws_bytes > (size_t)TAD_STATIC_SCRATCH_BYTES) return TAD_ENOMEM;
    void *ws = nullptr;
    int rc = static_scratch(&ws);
    if (rc != TAD_OK) return rc;
    // the kernels write every workspace entry before they read it, so the contents the previous call left behind
    // need no clearing
    return tad_eval_backward(plan, args_dev, f_dev, df_dev, dx_dev, ws, TAD_STATIC_SCRATCH_BYTES, stream);
}

}  // extern "C"
