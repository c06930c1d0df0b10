// Declarations shared by the kernel translation units and the C ABI front end.
#pragma once
#include <hip/hip_runtime.h>

#include "plan.hpp"

namespace tad {

struct ArgPtrs {
    const void *p[kMaxArgs];
};

int generic_forward(const tad_plan &pl, const void *const *args, void *f, void *ws, hipStream_t s);
int generic_backward(const tad_plan &pl, const void *const *args, const void *f, const void *df,
                     void *const *dx, void *ws, hipStream_t s);

int worked_forward(const tad_plan &pl, const void *const *args, void *f, hipStream_t s);
int worked_backward(const tad_plan &pl, const void *const *args, const void *f, const void *df,
                    void *const *dx, void *ws, hipStream_t s);

int mfma_forward(const tad_plan &pl, const void *const *args, void *f, void *ws, hipStream_t s);
int mfma_backward(const tad_plan &pl, const void *const *args, const void *f, const void *df, void *const *dx,
                  void *ws, hipStream_t s);
int pattern_forward(const tad_plan &pl, const void *const *args, void *f, hipStream_t s);
int pattern_backward(const tad_plan &pl, const void *const *args, const void *df, void *const *dx, void *ws,
                     hipStream_t s);

int strided_forward(const tad_plan &pl, const void *const *args, void *f, hipStream_t s);
int strided_backward(const tad_plan &pl, const void *const *args, const void *f, const void *df,
                     void *const *dx, void *ws, hipStream_t s);

int contract_forward(const tad_plan &pl, const void *const *args, void *f, void *ws, hipStream_t s);
int contract_backward(const tad_plan &pl, const void *const *args, const void *df, void *const *dx, void *ws,
                      hipStream_t s);

int program_forward(const tad_plan &pl, const void *const *args, void *f, void *ws, hipStream_t s);
int program_backward(const tad_plan &pl, const void *const *args, const void *df, void *const *dx, void *ws,
                     hipStream_t s);

}  // namespace tad
