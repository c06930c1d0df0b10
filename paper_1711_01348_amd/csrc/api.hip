// Device entry points of the C ABI: dispatch on the kernel family chosen at plan time.
#include <hip/hip_runtime.h>

#include "launch.h"

using namespace tad;

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

}  // extern "C"
