// Scalar bodies given as programs: parsing of the postfix form, symbolic differentiation by reverse
// accumulation on the expression graph (Sec. 2: the derivative of the output with respect to a node is the sum,
// over the nodes consuming it, of their derivative times the local partial derivative; one backward sweep yields
// the derivatives with respect to all inputs), and lowering to the three-address form the kernels interpret.
// Host only.
#pragma once
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <vector>

#include "../../include/tad.h"
#include "plan_dev.h"

namespace tad {

// expression graph in three-address form; node i only refers to nodes < i
struct Node {
    uint8_t op;     // ProgOp
    int a = -1, b = -1;   // input nodes
    int k = 0;      // operand index (P_ARG) or exponent (P_POWI)
    double c = 0;   // P_CONST
};

struct Graph {
    std::vector<Node> nodes;
    int add(uint8_t op, int a = -1, int b = -1, int k = 0, double c = 0) {
        nodes.push_back(Node{op, a, b, k, c});
        return (int)nodes.size() - 1;
    }
    int constant(double c) { return add(P_CONST, -1, -1, 0, c); }
};

// Postfix program -> graph.  Inner program: every operand may be read, the sum may not.  Outer program: the sum
// and those operands whose bit is set in `outer_operands` (their index ignores the summation indices, so they
// have one value per function index).  Returns the result node or a negative tad_status.
inline int parse_postfix(const tad_op *ops, int n, bool outer, int n_operands, Graph &g, uint32_t outer_operands = 0) {
    if (!ops || n < 1 || n > TAD_MAX_PROGRAM) return TAD_EINVAL;
    std::vector<int> st;
    int temp[TAD_MAX_TEMPS];   // node held by each temporary, -1: not stored yet
    for (int &t : temp) t = -1;
    for (int i = 0; i < n; ++i) {
        const tad_op &o = ops[i];
        auto pop = [&]() { int v = st.back(); st.pop_back(); return v; };
        switch (o.op) {
        case TAD_OP_CONST:
            if (!std::isfinite(o.value)) return TAD_EINVAL;
            st.push_back(g.constant(o.value));
            break;
        case TAD_OP_ARG:
            if (o.iarg < 0 || o.iarg >= n_operands) return TAD_EINVAL;
            if (outer && !((outer_operands >> o.iarg) & 1u)) return TAD_EINVAL;
            st.push_back(g.add(P_ARG, -1, -1, o.iarg));
            break;
        case TAD_OP_SUM:
            if (!outer) return TAD_EINVAL;
            st.push_back(g.add(P_SUM));
            break;
        case TAD_OP_ADD: case TAD_OP_SUB: case TAD_OP_MUL: case TAD_OP_DIV: {
            if (st.size() < 2) return TAD_EINVAL;
            const int b = pop(), a = pop();
            const uint8_t op = o.op == TAD_OP_ADD ? P_ADD : o.op == TAD_OP_SUB ? P_SUB : o.op == TAD_OP_MUL ? P_MUL : P_DIV;
            st.push_back(g.add(op, a, b));
            break;
        }
        case TAD_OP_NEG: case TAD_OP_EXP: case TAD_OP_LOG: case TAD_OP_SIN: case TAD_OP_COS: case TAD_OP_TANH:
        case TAD_OP_SQRT: {
            if (st.empty()) return TAD_EINVAL;
            const int a = pop();
            const uint8_t op = o.op == TAD_OP_NEG ? P_NEG : o.op == TAD_OP_EXP ? P_EXP : o.op == TAD_OP_LOG ? P_LOG
                             : o.op == TAD_OP_SIN ? P_SIN : o.op == TAD_OP_COS ? P_COS : o.op == TAD_OP_TANH ? P_TANH : P_SQRT;
            st.push_back(g.add(op, a));
            break;
        }
        case TAD_OP_POWI: {
            if (st.empty() || o.iarg < 1 || o.iarg > 16) return TAD_EINVAL;
            const int a = pop();
            st.push_back(g.add(P_POWI, a, -1, o.iarg));
            break;
        }
        case TAD_OP_STORE:   // in the graph a temporary is just a second reference to the node
            if (st.empty() || o.iarg < 0 || o.iarg >= TAD_MAX_TEMPS) return TAD_EINVAL;
            temp[o.iarg] = st.back();
            break;
        case TAD_OP_LOAD:
            if (o.iarg < 0 || o.iarg >= TAD_MAX_TEMPS || temp[o.iarg] < 0) return TAD_EINVAL;
            st.push_back(temp[o.iarg]);
            break;
        default: return TAD_EINVAL;
        }
    }
    if (st.size() != 1) return TAD_EINVAL;
    return st[0];
}

// The built-in bodies written as the postfix programs they stand for; false for a body that has none.
inline bool builtin_body_programs(int body, std::vector<tad_op> &inner, std::vector<tad_op> &outer) {
    auto op = [](int code, int iarg = 0) { tad_op o{}; o.op = code; o.iarg = iarg; return o; };
    const tad_op A0 = op(TAD_OP_ARG, 0), A1 = op(TAD_OP_ARG, 1), SUM = op(TAD_OP_SUM);
    switch (body) {
    case TAD_BODY_SQ: inner = {A0}; outer = {SUM, op(TAD_OP_POWI, 2)}; return true;
    case TAD_BODY_CUBE: inner = {A0}; outer = {SUM, op(TAD_OP_POWI, 3)}; return true;
    case TAD_BODY_SIN: inner = {A0}; outer = {SUM, op(TAD_OP_SIN)}; return true;
    case TAD_BODY_EXP: inner = {A0}; outer = {SUM, op(TAD_OP_EXP)}; return true;
    case TAD_BODY_MUL: inner = {A0, A1, op(TAD_OP_MUL)}; outer = {SUM}; return true;
    case TAD_BODY_TANH_DOT: inner = {A0, A1, op(TAD_OP_MUL)}; outer = {SUM, op(TAD_OP_TANH)}; return true;
    case TAD_BODY_WORKED:   // exp(-sum((a + b)^2 c + d^3))
        inner = {A0, A1, op(TAD_OP_ADD), op(TAD_OP_POWI, 2), op(TAD_OP_ARG, 2), op(TAD_OP_MUL),
                 op(TAD_OP_ARG, 3), op(TAD_OP_POWI, 3), op(TAD_OP_ADD)};
        outer = {SUM, op(TAD_OP_NEG), op(TAD_OP_EXP)};
        return true;
    default: return false;
    }
}

// Do two expression graphs compute the same function by the same operations?  Structural comparison from the result
// nodes down; sums and products match with their inputs in either order, x * x matches x^2.
inline bool same_expression(const Graph &ga, int a, const Graph &gb, int b) {
    const Node &x = ga.nodes[(size_t)a], &y = gb.nodes[(size_t)b];
    if (x.op != y.op) {
        // x * x against x^2
        const Node *m = x.op == P_MUL ? &x : y.op == P_MUL ? &y : nullptr, *p = x.op == P_POWI ? &x : y.op == P_POWI ? &y : nullptr;
        if (!m || !p || p->k != 2) return false;
        const Graph &gm = m == &x ? ga : gb, &gp = p == &x ? ga : gb;
        return same_expression(gm, m->a, gm, m->b) && same_expression(gm, m->a, gp, p->a);
    }
    switch (x.op) {
    case P_CONST: return x.c == y.c;
    case P_ARG: return x.k == y.k;
    case P_SUM: return true;
    case P_ADD: case P_MUL:
        return (same_expression(ga, x.a, gb, y.a) && same_expression(ga, x.b, gb, y.b)) ||
               (same_expression(ga, x.a, gb, y.b) && same_expression(ga, x.b, gb, y.a));
    case P_SUB: case P_DIV: return same_expression(ga, x.a, gb, y.a) && same_expression(ga, x.b, gb, y.b);
    case P_POWI: return x.k == y.k && same_expression(ga, x.a, gb, y.a);
    default: return same_expression(ga, x.a, gb, y.a);   // one-input functions
    }
}

// The built-in body whose inner and outer function a program body spells out (same operands in the same order), or -1.
// Such an expression is planned as that body, so that it reaches the kernels written for it.
inline int matching_builtin_body(const tad_expr &e) {
    if (e.body != TAD_BODY_PROGRAM) return -1;
    Graph gi, go;
    const uint32_t none = 0;
    const int ri = parse_postfix(e.inner, e.n_inner, false, e.n_operands, gi);
    const int ro = parse_postfix(e.outer, e.n_outer, true, e.n_operands, go, none);   // an outer function that reads operands fails here
    if (ri < 0 || ro < 0) return -1;
    static const int bodies[] = {TAD_BODY_SQ, TAD_BODY_CUBE, TAD_BODY_SIN, TAD_BODY_EXP, TAD_BODY_MUL, TAD_BODY_WORKED, TAD_BODY_TANH_DOT};
    static const int operands[] = {1, 1, 1, 1, 2, 4, 2};
    for (size_t t = 0; t < sizeof bodies / sizeof bodies[0]; ++t) {
        if (operands[t] != e.n_operands) continue;
        if (e.n_sum > 0 && (bodies[t] == TAD_BODY_SQ || bodies[t] == TAD_BODY_CUBE || bodies[t] == TAD_BODY_SIN)) continue;
        std::vector<tad_op> bi, bo;
        builtin_body_programs(bodies[t], bi, bo);
        Graph hi, ho;
        const int si = parse_postfix(bi.data(), (int)bi.size(), false, operands[t], hi);
        const int so = parse_postfix(bo.data(), (int)bo.size(), true, operands[t], ho, none);
        if (si >= 0 && so >= 0 && same_expression(gi, ri, hi, si) && same_expression(go, ro, ho, so)) return bodies[t];
    }
    return -1;
}

// Reverse accumulation from `result` back to the inputs.  The derivative expressions are appended to the same
// graph, so they share the forward nodes (Sec. 2: the derivative graph reuses the values of the function graph).
// input_grad[p] receives the node of d result / d operand p for p < n_operands and input_grad[n_operands] that of
// d result / d sum, or -1 where the derivative is identically zero.
inline void reverse_accumulate(Graph &g, int result, int n_operands, std::vector<int> &input_grad) {
    const int n_fwd = (int)g.nodes.size();
    std::vector<int> adj(n_fwd, -1);   // node holding d result / d node, -1 = zero
    auto accumulate = [&](int node, int term) { adj[node] = adj[node] < 0 ? term : g.add(P_ADD, adj[node], term); };
    input_grad.assign(n_operands + 1, -1);
    const int sum_slot = n_operands;
    adj[result] = g.constant(1.0);
    for (int i = n_fwd - 1; i >= 0; --i) {
        const int d = adj[i];
        if (d < 0) continue;
        const Node nd = g.nodes[i];   // copy: g.nodes grows below
        switch (nd.op) {
        case P_CONST: break;
        case P_ARG: input_grad[nd.k] = input_grad[nd.k] < 0 ? d : g.add(P_ADD, input_grad[nd.k], d); break;
        case P_SUM: input_grad[sum_slot] = input_grad[sum_slot] < 0 ? d : g.add(P_ADD, input_grad[sum_slot], d); break;
        case P_ADD: accumulate(nd.a, d); accumulate(nd.b, d); break;
        case P_SUB: accumulate(nd.a, d); accumulate(nd.b, g.add(P_NEG, d)); break;
        case P_MUL: accumulate(nd.a, g.add(P_MUL, d, nd.b)); accumulate(nd.b, g.add(P_MUL, d, nd.a)); break;
        case P_DIV: {   // a / b: d/da = 1 / b, d/db = -(a / b) / b
            accumulate(nd.a, g.add(P_DIV, d, nd.b));
            accumulate(nd.b, g.add(P_NEG, g.add(P_DIV, g.add(P_MUL, d, i), nd.b)));
            break;
        }
        case P_NEG: accumulate(nd.a, g.add(P_NEG, d)); break;
        case P_EXP: accumulate(nd.a, g.add(P_MUL, d, i)); break;
        case P_LOG: accumulate(nd.a, g.add(P_DIV, d, nd.a)); break;
        case P_SIN: accumulate(nd.a, g.add(P_MUL, d, g.add(P_COS, nd.a))); break;
        case P_COS: accumulate(nd.a, g.add(P_NEG, g.add(P_MUL, d, g.add(P_SIN, nd.a)))); break;
        case P_TANH: accumulate(nd.a, g.add(P_MUL, d, g.add(P_SUB, g.constant(1.0), g.add(P_MUL, i, i)))); break;
        case P_SQRT: accumulate(nd.a, g.add(P_DIV, d, g.add(P_MUL, g.constant(2.0), i))); break;
        case P_POWI: {
            int pw = nd.k == 1 ? -1 : nd.k == 2 ? nd.a : g.add(P_POWI, nd.a, -1, nd.k - 1);
            int t = nd.k == 1 ? d : g.add(P_MUL, d, g.add(P_MUL, g.constant((double)nd.k), pw));
            accumulate(nd.a, t);
            break;
        }
        }
    }
}

// Peephole simplification: alias[i] = an earlier node that computes the same value as node i (products with the
// constant 1, division by 1 and double negations are dropped).
inline std::vector<int> simplify(const Graph &g) {
    const int N = (int)g.nodes.size();
    std::vector<int> alias(N);
    auto is_one = [&](int i) { return g.nodes[i].op == P_CONST && g.nodes[i].c == 1.0; };
    for (int i = 0; i < N; ++i) {
        const Node &nd = g.nodes[i];
        alias[i] = i;
        const int a = nd.a >= 0 ? alias[nd.a] : -1, b = nd.b >= 0 ? alias[nd.b] : -1;
        if (nd.op == P_MUL && is_one(a)) alias[i] = b;
        else if (nd.op == P_MUL && is_one(b)) alias[i] = a;
        else if (nd.op == P_DIV && is_one(b)) alias[i] = a;
        else if (nd.op == P_NEG && g.nodes[a].op == P_NEG) alias[i] = alias[g.nodes[a].a];
    }
    return alias;
}

inline bool prog_is_leaf(uint8_t op) { return op == P_CONST || op == P_ARG || op == P_SUM; }
inline bool prog_is_binary(uint8_t op) { return op == P_ADD || op == P_SUB || op == P_MUL || op == P_DIV; }

// One operation on values (shared by the two host evaluators below).
inline double prog_apply(uint8_t op, double x, double y, int k) {
    switch (op) {
    case P_ADD: return x + y;
    case P_SUB: return x - y;
    case P_MUL: return x * y;
    case P_DIV: return x / y;
    case P_NEG: return -x;
    case P_EXP: return std::exp(x);
    case P_LOG: return std::log(x);
    case P_SIN: return std::sin(x);
    case P_COS: return std::cos(x);
    case P_TANH: return std::tanh(x);
    case P_SQRT: return std::sqrt(x);
    case P_POWI: { double r = x; for (int e = 1; e < k; ++e) r *= x; return r; }
    default: return 0.0;
    }
}

// Evaluation of a lowered program (the host twin of the kernels' interpreter), fp64: one temporary per operation.
inline double eval_host_temporaries(const DevProg &P, const double *v, double s) {
    if (P.result < 0) return 0.0;
    double t[kMaxProgOps] = {0};
    for (int i = 0; i < P.n; ++i) {
        switch (P.op[i]) {
        case P_CONST: t[i] = P.cst[P.a[i]]; break;
        case P_ARG: t[i] = v[P.a[i]]; break;
        case P_SUM: t[i] = s; break;
        default: t[i] = prog_apply(P.op[i], t[P.a[i]], t[P.b[i]], P.k[i]);
        }
    }
    return t[P.result];
}
// The same from the register form.
inline double eval_host_registers(const DevProg &P, const double *v, double s) {
    if (P.result < 0) return 0.0;
    double r[kProgRegs] = {0};
    auto fetch = [&](int code) {
        return code < kCodeArg ? r[code] : code < kCodeConst ? v[code - kCodeArg] : code < kCodeSum ? P.cst[code - kCodeConst] : s;
    };
    for (int i = 0; i < P.n_words; ++i) {
        const uint32_t w = P.word[i];
        const uint8_t op = (uint8_t)(w & 0xff);
        const int first = (int)((w >> 8) & 0xff), second = (int)((w >> 16) & 0xff), dst = (int)(w >> 24);
        r[dst] = op == P_POWI ? prog_apply(op, fetch(first), 0.0, second)
                              : prog_apply(op, fetch(first), prog_is_binary(op) ? fetch(second) : 0.0, 0);
    }
    return fetch(P.result_code);
}

// Register form: operands are folded into the operations that use them (no register, no operation of their
// own); the other temporaries get registers by live range, in program order: the inputs an operation reads for the
// last time are released before its destination is chosen (an operation reads before it writes), the lowest free
// register is taken.  The result is checked against the form with one temporary per operation at a few points; a
// program that needs more than kProgRegs registers, or fails the check, keeps n_regs < 0.
inline void allocate_registers(DevProg &P) {
    P.n_regs = -1;
    P.n_words = 0;
    P.result_code = 0;
    if (P.result < 0 || P.n <= 0) return;
    int last[kMaxProgOps], code[kMaxProgOps];
    for (int i = 0; i < P.n; ++i) last[i] = -1;
    for (int i = 0; i < P.n; ++i) {
        if (prog_is_leaf(P.op[i])) continue;
        last[P.a[i]] = i;
        if (prog_is_binary(P.op[i])) last[P.b[i]] = i;
    }
    last[P.result] = P.n;
    bool used[kProgRegs] = {false};
    int high = 0, words = 0;
    for (int i = 0; i < P.n; ++i) {
        const uint8_t op = P.op[i];
        if (prog_is_leaf(op)) {
            code[i] = op == P_ARG ? kCodeArg + P.a[i] : op == P_CONST ? kCodeConst + P.a[i] : kCodeSum;
            continue;
        }
        const bool binary = prog_is_binary(op);
        const int first = code[P.a[i]], second = binary ? code[P.b[i]] : op == P_POWI ? (int)(uint8_t)P.k[i] : 0;
        if (first < kCodeArg && last[P.a[i]] == i) used[first] = false;
        if (binary && second < kCodeArg && last[P.b[i]] == i) used[second] = false;
        int r = 0;
        while (r < kProgRegs && used[r]) ++r;
        if (r == kProgRegs) return;
        code[i] = r;
        if (last[i] >= 0) used[r] = true;      // a value nobody reads frees its register at once
        high = std::max(high, r + 1);
        P.word[words++] = (uint32_t)op | (uint32_t)first << 8 | (uint32_t)second << 16 | (uint32_t)r << 24;
    }
    P.n_words = words;
    P.result_code = code[P.result];
    // self-check at deterministic sample points (NaN results must agree as NaN)
    for (int t = 0; t < 4; ++t) {
        double v[TAD_MAX_ARGS];
        for (int q = 0; q < TAD_MAX_ARGS; ++q) v[q] = 0.37 + 0.21 * q + 0.13 * t;
        const double s = 0.45 + 0.3 * t;
        const double x = eval_host_temporaries(P, v, s), y = eval_host_registers(P, v, s);
        if (!(x == y || (x != x && y != y))) return;
    }
    P.n_regs = high;
}

// Lower the part of the graph that `result` depends on: simplified as above, equal constants share a slot, the
// nodes are renumbered densely.  False if it does not fit.
inline bool lower(const Graph &g, int result, DevProg &out) {
    out = DevProg{};
    if (result < 0) { out.n = 0; out.result = -1; return true; }
    const int N = (int)g.nodes.size();
    const std::vector<int> alias = simplify(g);
    result = alias[result];
    std::vector<char> live(N, 0);
    live[result] = 1;
    for (int i = N - 1; i >= 0; --i) {
        if (!live[i]) continue;
        if (g.nodes[i].a >= 0) live[alias[g.nodes[i].a]] = 1;
        if (g.nodes[i].b >= 0) live[alias[g.nodes[i].b]] = 1;
    }
    std::vector<int> slot(N, -1);
    int n = 0, nc = 0;
    for (int i = 0; i < N; ++i) {
        if (!live[i]) continue;
        if (n >= kMaxProgOps) return false;
        const Node &nd = g.nodes[i];
        out.op[n] = nd.op;
        out.k[n] = 0;
        out.a[n] = out.b[n] = 0;
        if (nd.op == P_CONST) {
            int c = 0;
            while (c < nc && out.cst[c] != nd.c) ++c;
            if (c == nc) {
                if (nc >= kMaxProgConst) return false;
                out.cst[nc++] = nd.c;
            }
            out.a[n] = (uint8_t)c;
        } else if (nd.op == P_ARG) {
            out.a[n] = (uint8_t)nd.k;
        } else if (nd.op != P_SUM) {
            out.a[n] = (uint8_t)slot[alias[nd.a]];
            if (nd.b >= 0) out.b[n] = (uint8_t)slot[alias[nd.b]];
            if (nd.op == P_POWI) out.k[n] = (int8_t)nd.k;
        }
        slot[i] = n++;
    }
    out.n = n;
    out.result = slot[result];
    allocate_registers(out);
    return true;
}

// Postfix form of the expression computing `node`, appended to `out`; same simplifications as lower().  A
// sub-expression with several consumers is written once, kept in a temporary (TAD_OP_STORE) and read back
// (TAD_OP_LOAD) while temporaries last; after that it is written out again.  False once the program grows
// beyond `cap` operations.
inline bool emit_postfix(const Graph &g, const std::vector<int> &alias, int node, std::vector<tad_op> &out, size_t cap) {
    static_assert((int)P_CONST == (int)TAD_OP_CONST && (int)P_ARG == (int)TAD_OP_ARG && (int)P_SUM == (int)TAD_OP_SUM && (int)P_ADD == (int)TAD_OP_ADD &&
                      (int)P_SUB == (int)TAD_OP_SUB && (int)P_MUL == (int)TAD_OP_MUL && (int)P_DIV == (int)TAD_OP_DIV && (int)P_NEG == (int)TAD_OP_NEG &&
                      (int)P_EXP == (int)TAD_OP_EXP && (int)P_LOG == (int)TAD_OP_LOG && (int)P_SIN == (int)TAD_OP_SIN && (int)P_COS == (int)TAD_OP_COS &&
                      (int)P_TANH == (int)TAD_OP_TANH && (int)P_SQRT == (int)TAD_OP_SQRT && (int)P_POWI == (int)TAD_OP_POWI,
                  "internal and public operation codes are numbered alike");
    const int N = (int)g.nodes.size();
    // consumers of every node inside the sub-graph of `node`
    std::vector<int> uses(N, 0);
    std::vector<char> seen(N, 0);
    std::vector<int> stack{alias[node]};
    seen[alias[node]] = 1;
    while (!stack.empty()) {
        const Node &nd = g.nodes[stack.back()];
        stack.pop_back();
        for (int in : {nd.a, nd.b}) {
            if (in < 0) continue;
            const int t = alias[in];
            ++uses[t];
            if (!seen[t]) { seen[t] = 1; stack.push_back(t); }
        }
    }
    std::vector<int> slot(N, -1);
    int next_slot = 0;
    bool ok = true;
    // recursion on the simplified graph
    struct Emit {
        const Graph &g; const std::vector<int> &alias; std::vector<int> &uses, &slot; int &next_slot;
        std::vector<tad_op> &out; size_t cap; bool &ok;
        void run(int n) {
            if (!ok) return;
            const int t = alias[n];
            const Node &nd = g.nodes[t];
            tad_op o{};
            if (slot[t] >= 0) {
                o.op = TAD_OP_LOAD;
                o.iarg = slot[t];
                out.push_back(o);
                ok = out.size() <= cap;
                return;
            }
            if (nd.a >= 0) run(nd.a);
            if (nd.b >= 0) run(nd.b);
            if (!ok) return;
            o.op = nd.op;
            o.iarg = (nd.op == P_ARG || nd.op == P_POWI) ? nd.k : 0;
            o.value = nd.op == P_CONST ? nd.c : 0.0;
            out.push_back(o);
            const bool leaf = nd.op == P_CONST || nd.op == P_ARG || nd.op == P_SUM;
            if (!leaf && uses[t] > 1 && next_slot < TAD_MAX_TEMPS) {
                tad_op st{};
                st.op = TAD_OP_STORE;
                st.iarg = slot[t] = next_slot++;
                out.push_back(st);
            }
            ok = out.size() <= cap;
        }
    } emit{g, alias, uses, slot, next_slot, out, cap, ok};
    emit.run(node);
    return ok;
}

inline bool reads_operands(const DevProg &P) {
    for (int i = 0; i < P.n; ++i)
        if (P.op[i] == P_ARG) return true;
    return false;
}
inline double eval_host(const DevProg &P, const double *v, double s) {
    return P.n_regs >= 0 ? eval_host_registers(P, v, s) : eval_host_temporaries(P, v, s);
}

// Everything a program-body plan carries.
struct ProgramBody {
    int n_operands = 0;
    DevProg inner, outer;            // values
    DevProg dinner[TAD_MAX_ARGS];    // d inner / d operand p
    DevProg douter;                  // d outer / d sum
    DevProg douter_arg[TAD_MAX_ARGS];   // d outer / d operand p (identically zero unless the outer program reads p)
    uint32_t outer_mask = 0;         // operands the outer program reads
};

// Parse, differentiate and lower both programs of an expression.  `outer_operands`: operands the outer program
// may read; `wanted`: operands whose gradient will be asked for (the derivatives with respect to the others are
// not lowered, so their length does not matter).  Returns a tad_status.
inline int build_program_body(const tad_expr &e, ProgramBody &pb, uint32_t outer_operands, uint32_t wanted) {
    if (e.n_operands < 1 || e.n_operands > TAD_MAX_ARGS) return TAD_EINVAL;
    pb.n_operands = e.n_operands;
    Graph gi;
    const int ri = parse_postfix(e.inner, e.n_inner, false, e.n_operands, gi);
    if (ri < 0) return ri;
    if (!lower(gi, ri, pb.inner)) return TAD_EUNSUPPORTED;
    std::vector<int> grads;
    reverse_accumulate(gi, ri, e.n_operands, grads);
    for (int p = 0; p < e.n_operands; ++p)
        if (!lower(gi, ((wanted >> p) & 1u) ? grads[p] : -1, pb.dinner[p])) return TAD_EUNSUPPORTED;
    Graph go;
    const int ro = parse_postfix(e.outer, e.n_outer, true, e.n_operands, go, outer_operands);
    if (ro < 0) return ro;
    if (!lower(go, ro, pb.outer)) return TAD_EUNSUPPORTED;
    pb.outer_mask = 0;
    for (int i = 0; i < e.n_outer; ++i)
        if (e.outer[i].op == TAD_OP_ARG) pb.outer_mask |= 1u << e.outer[i].iarg;
    reverse_accumulate(go, ro, e.n_operands, grads);
    if (!lower(go, wanted ? grads[e.n_operands] : -1, pb.douter)) return TAD_EUNSUPPORTED;
    for (int p = 0; p < e.n_operands; ++p)
        if (!lower(go, ((wanted >> p) & 1u) ? grads[p] : -1, pb.douter_arg[p])) return TAD_EUNSUPPORTED;
    return TAD_OK;
}

}  // namespace tad
