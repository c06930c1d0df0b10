// Fourier-Motzkin elimination for  A z >= B b  with a symbolic right-hand side
// (Sec. 4.2 of the paper): produces, for every variable z_k, the rows of
//
//     max(L^k b + Lhat^k z_{>k})  <=  z_k  <=  min(H^k b + Hhat^k z_{>k})
//
// and the feasibility rows F b <= 0.  Variables are eliminated in the order
// z_0, z_1, ...; z_0 therefore becomes the innermost loop.
//
// Instead of dividing a row by |A_ik| (which would need rationals) each row keeps
// its positive integer coefficient `scale` of z_k:   scale * z_k >= (or <=) rhs.
// A combined row is  |A_nk| * row_p + A_pk * row_n, divided by the gcd of its
// entries, which is the paper's sum of the two normalised rows up to a positive
// factor.  Rows that cannot be extreme (they combine more than t+1 original
// rows after t eliminations) are dropped, as are exact duplicates.
#pragma once
#include <algorithm>
#include <cstdint>
#include <vector>

#include "intmath.hpp"

namespace tad {

struct FMRow {
    int64_t scale = 0;            // > 0, coefficient of z_k
    std::vector<int64_t> coef_b;  // multiplies b
    std::vector<int64_t> coef_z;  // multiplies z (only entries > k are non-zero)
};

struct FMResult {
    std::vector<std::vector<FMRow>> lower, upper;  // per variable
    std::vector<std::vector<int64_t>> feasibility; // rows of F (coefficients of b):  F b <= 0
    // true for the rows of F that are original constraints without any variable; the other rows of F only
    // state "some lower bound <= some upper bound" and are implied by an empty loop range
    std::vector<bool> feasibility_original;
    bool bounded = true;                           // false if some z_k is bounded from one side only
};

inline FMResult fourier_motzkin(const IMat &A, int n_b, const IMat &Binit) {
    struct Row {
        std::vector<int64_t> a, b;
        uint64_t hist;
    };
    const int M = A.cols;
    std::vector<Row> rows;
    for (int i = 0; i < A.rows; ++i) {
        Row r;
        r.a.assign(A.a.begin() + (size_t)i * M, A.a.begin() + (size_t)(i + 1) * M);
        r.b.assign(Binit.a.begin() + (size_t)i * n_b, Binit.a.begin() + (size_t)(i + 1) * n_b);
        r.hist = 1ull << (i & 63);
        rows.push_back(std::move(r));
    }
    FMResult out;
    out.lower.resize(M);
    out.upper.resize(M);
    for (int k = 0; k < M; ++k) {
        std::vector<int> phi, mu, zeta;
        for (int i = 0; i < (int)rows.size(); ++i) {
            if (rows[i].a[k] > 0) phi.push_back(i);
            else if (rows[i].a[k] < 0) mu.push_back(i);
            else zeta.push_back(i);
        }
        for (int i : phi) {
            FMRow r;
            r.scale = rows[i].a[k];
            r.coef_b = rows[i].b;
            r.coef_z.assign(M, 0);
            for (int j = k + 1; j < M; ++j) r.coef_z[j] = cneg(rows[i].a[j]);
            out.lower[k].push_back(std::move(r));
        }
        for (int i : mu) {
            FMRow r;
            r.scale = cneg(rows[i].a[k]);
            r.coef_b.resize(n_b);
            for (int j = 0; j < n_b; ++j) r.coef_b[j] = cneg(rows[i].b[j]);
            r.coef_z.assign(M, 0);
            for (int j = k + 1; j < M; ++j) r.coef_z[j] = rows[i].a[j];
            out.upper[k].push_back(std::move(r));
        }
        if (phi.empty() || mu.empty()) out.bounded = false;
        std::vector<Row> next;
        for (int i : zeta) next.push_back(rows[i]);
        for (int p : phi)
            for (int n : mu) {
                Row r;
                r.hist = rows[p].hist | rows[n].hist;
                if (__builtin_popcountll(r.hist) > k + 2) continue;  // cannot be an extreme combination
                int64_t fp = cneg(rows[n].a[k]), fn = rows[p].a[k];
                r.a.resize(M);
                r.b.resize(n_b);
                int64_t g = 0;
                for (int j = 0; j < M; ++j) {
                    r.a[j] = cadd(cmul(fp, rows[p].a[j]), cmul(fn, rows[n].a[j]));
                    g = gcd64(g, r.a[j]);
                }
                for (int j = 0; j < n_b; ++j) {
                    r.b[j] = cadd(cmul(fp, rows[p].b[j]), cmul(fn, rows[n].b[j]));
                    g = gcd64(g, r.b[j]);
                }
                if (g > 1) {
                    for (auto &v : r.a) v /= g;
                    for (auto &v : r.b) v /= g;
                }
                bool dup = false;
                for (Row &q : next)
                    if (q.a == r.a && q.b == r.b) {
                        dup = true;
                        if (__builtin_popcountll(r.hist) < __builtin_popcountll(q.hist)) q.hist = r.hist;
                        break;
                    }
                if (!dup) next.push_back(std::move(r));
            }
        rows.swap(next);
    }
    for (const Row &r : rows) {
        bool zero = std::all_of(r.b.begin(), r.b.end(), [](int64_t v) { return v == 0; });
        if (!zero) {
            out.feasibility.push_back(r.b);
            out.feasibility_original.push_back(__builtin_popcountll(r.hist) == 1);
        }
    }
    return out;
}

}  // namespace tad
