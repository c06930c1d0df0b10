// A gradient as the small graph of element-wise expressions that Sec. 5.3 describes: seed expressions for the
// factor the terms share, then one derived expression per occurrence of the tensor (and a second one where the outer
// function reads the operand), each with a plan of its own; the results of the parts are added.
#pragma once
#include <vector>

#include "plan.hpp"

// operand sources of an expression of the graph
constexpr int kSrcDf = -1;      // the incoming gradient df
constexpr int kSrcSeedG = -2;   // g = df * d outer / d sum
// -3 - p: h of operand p = df * d outer / d operand p; q >= 0: operand q of the original expression

struct tad_derived {
    struct Node {
        tad_plan *plan = nullptr;          // owned
        std::vector<int> src;              // per operand of `plan`: where its tensor comes from
        int seed = 0;                      // seeds: which one (kSrcSeedG or -3 - p); parts: 0
        size_t out_offset = 0;             // seeds: where the result lives in the workspace
    };
    std::vector<Node> seeds;               // evaluated first, over the function indices of the original expression
    std::vector<Node> parts;               // evaluated next; their results are added in this order
    tad_dtype dtype = TAD_F32;
    int arg = 0;                           // the tensor whose gradient this is
    int n_original = 0;                    // operands of the original expression
    std::vector<int> root;                 // original operand -> operand that holds its tensor
    int64_t count = 0;                     // elements of the gradient
    size_t tmp_offset = 0;                 // a second tensor of the gradient's size (results of the later parts)
    size_t sub_offset = 0;                 // workspace of the expressions' own kernels (shared: they run one after another)
    size_t ws_bytes = 0;
    ~tad_derived() {
        for (auto &n : seeds) tad_plan_free(n.plan);
        for (auto &n : parts) tad_plan_free(n.plan);
    }
};
