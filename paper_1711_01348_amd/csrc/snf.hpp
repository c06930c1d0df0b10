// Smith normal form of a small integer matrix and the solution structure of
// A x = b over the integers (Sec. 4.1 of the paper).
//
//   S = U A V,  S = diag(alpha_1 .. alpha_R, 0 ..),  alpha_i > 0,  alpha_i | alpha_{i+1},
//   U (N x N) and V (M x M) unimodular.
//
// Where the paper leaves the pivot free ("there is some non-zero entry"), the
// pivot taken here is the entry of smallest magnitude in the trailing block,
// ties broken by smallest row then column, which makes U, V deterministic and
// keeps the cofactors small.  After the divisibility repair (adding column a+1
// to column a) the trailing block is diagonalised again from index a.
#pragma once
#include "intmath.hpp"

namespace tad {

struct Smith {
    IMat S, U, V;
    int R = 0;
};

namespace detail {

inline void swap_rows(IMat &m, int a, int b) {
    if (a == b) return;
    for (int j = 0; j < m.cols; ++j) std::swap(m(a, j), m(b, j));
}
inline void swap_cols(IMat &m, int a, int b) {
    if (a == b) return;
    for (int i = 0; i < m.rows; ++i) std::swap(m(i, a), m(i, b));
}
// (row_a, row_i) <- (s row_a + t row_i, -g row_a + al row_i)
inline void mix_rows(IMat &m, int a, int i, int64_t s, int64_t t, int64_t g, int64_t al) {
    for (int j = 0; j < m.cols; ++j) {
        int64_t x = m(a, j), y = m(i, j);
        m(a, j) = cadd(cmul(s, x), cmul(t, y));
        m(i, j) = cadd(cmul(cneg(g), x), cmul(al, y));
    }
}
inline void mix_cols(IMat &m, int a, int j, int64_t s, int64_t t, int64_t g, int64_t al) {
    for (int i = 0; i < m.rows; ++i) {
        int64_t x = m(i, a), y = m(i, j);
        m(i, a) = cadd(cmul(s, x), cmul(t, y));
        m(i, j) = cadd(cmul(cneg(g), x), cmul(al, y));
    }
}
// row_i <- row_i - f row_a
inline void sub_row(IMat &m, int i, int a, int64_t f) {
    for (int j = 0; j < m.cols; ++j) m(i, j) = csub(m(i, j), cmul(f, m(a, j)));
}
inline void sub_col(IMat &m, int j, int a, int64_t f) {
    for (int i = 0; i < m.rows; ++i) m(i, j) = csub(m(i, j), cmul(f, m(i, a)));
}

// Diagonalise the trailing block starting at (a, a); returns the rank.
inline int diagonalise(Smith &w, int a) {
    IMat &S = w.S, &U = w.U, &V = w.V;
    const int N = S.rows, M = S.cols;
    for (;;) {
        int pi = -1, pj = -1;
        int64_t best = 0;
        for (int i = a; i < N; ++i)
            for (int j = a; j < M; ++j) {
                int64_t v = cabs(S(i, j));
                if (v != 0 && (pi < 0 || v < best)) { best = v; pi = i; pj = j; }
            }
        if (pi < 0) break;
        swap_cols(S, a, pj); swap_cols(V, a, pj);
        swap_rows(S, a, pi); swap_rows(U, a, pi);
        bool changing = true;
        while (changing) {
            changing = false;
            for (int i = a + 1; i < N; ++i) {
                if (S(i, a) == 0) continue;
                changing = true;
                if (S(i, a) % S(a, a) != 0) {
                    // gcd step: beta = sigma S_aa + tau S_ia replaces the pivot, S_ia becomes 0
                    Bezout bz = egcd(S(a, a), S(i, a));
                    int64_t g = S(i, a) / bz.g, al = S(a, a) / bz.g;
                    mix_rows(S, a, i, bz.x, bz.y, g, al);
                    mix_rows(U, a, i, bz.x, bz.y, g, al);
                } else {
                    int64_t f = S(i, a) / S(a, a);
                    sub_row(S, i, a, f); sub_row(U, i, a, f);
                }
            }
            for (int j = a + 1; j < M; ++j) {
                if (S(a, j) == 0) continue;
                changing = true;
                if (S(a, j) % S(a, a) != 0) {
                    Bezout bz = egcd(S(a, a), S(a, j));
                    int64_t g = S(a, j) / bz.g, al = S(a, a) / bz.g;
                    mix_cols(S, a, j, bz.x, bz.y, g, al);
                    mix_cols(V, a, j, bz.x, bz.y, g, al);
                } else {
                    int64_t f = S(a, j) / S(a, a);
                    sub_col(S, j, a, f); sub_col(V, j, a, f);
                }
            }
        }
        ++a;
    }
    return a;
}

}  // namespace detail

inline Smith smith_normal_form(const IMat &A) {
    Smith w;
    w.S = A;
    w.U = IMat::identity(A.rows);
    w.V = IMat::identity(A.cols);
    w.R = detail::diagonalise(w, 0);
    bool again = true;
    while (again) {
        again = false;
        for (int a = 0; a < w.R; ++a) {
            if (w.S(a, a) < 0)
                for (int i = 0; i < w.S.rows || i < w.V.rows; ++i) {
                    if (i < w.S.rows) w.S(i, a) = cneg(w.S(i, a));
                    if (i < w.V.rows) w.V(i, a) = cneg(w.V(i, a));
                }
            if (a + 1 < w.R && w.S(a + 1, a + 1) % w.S(a, a) != 0) {
                for (int i = 0; i < w.S.rows; ++i) w.S(i, a) = cadd(w.S(i, a), w.S(i, a + 1));
                for (int i = 0; i < w.V.rows; ++i) w.V(i, a) = cadd(w.V(i, a), w.V(i, a + 1));
                w.R = detail::diagonalise(w, a);
                again = true;
                break;
            }
        }
    }
    return w;
}

}  // namespace tad
