// Exact integer helpers for the host-side index-plan derivation.
// All arithmetic is checked: an int64 overflow throws tad::overflow_error,
// which the C ABI turns into TAD_EOVERFLOW.
#pragma once
#include <cstdint>
#include <stdexcept>
#include <vector>

namespace tad {

struct overflow_error : std::runtime_error {
    overflow_error() : std::runtime_error("int64 overflow") {}
};

inline int64_t cadd(int64_t a, int64_t b) {
    int64_t r;
    if (__builtin_add_overflow(a, b, &r)) throw overflow_error();
    return r;
}
inline int64_t csub(int64_t a, int64_t b) {
    int64_t r;
    if (__builtin_sub_overflow(a, b, &r)) throw overflow_error();
    return r;
}
inline int64_t cmul(int64_t a, int64_t b) {
    int64_t r;
    if (__builtin_mul_overflow(a, b, &r)) throw overflow_error();
    return r;
}
inline int64_t cneg(int64_t a) { return csub(0, a); }
inline int64_t cabs(int64_t a) { return a < 0 ? cneg(a) : a; }

// floor(a / b) and ceil(a / b) for b > 0, exact for negative a (not C truncation).
inline int64_t floor_div(int64_t a, int64_t b) {
    int64_t q = a / b, r = a % b;
    return (r != 0 && r < 0) ? q - 1 : q;
}
inline int64_t ceil_div(int64_t a, int64_t b) {
    int64_t q = a / b, r = a % b;
    return (r != 0 && r > 0) ? q + 1 : q;
}

// Extended Euclidean algorithm (Sec. 4.1, "Extended Euclidean algorithm"):
// g = gcd(a, b) = a x + b y, g >= 0.  The remainder sequence runs on |a|, |b|;
// the cofactors are given the signs of the inputs afterwards.
struct Bezout {
    int64_t g, x, y;
};
inline Bezout egcd(int64_t a, int64_t b) {
    int64_t r0 = cabs(a), r1 = cabs(b);
    int64_t s0 = 1, s1 = 0, t0 = 0, t1 = 1;
    while (r1 != 0) {
        int64_t q = r0 / r1;
        int64_t r2 = r0 - q * r1;  // 0 <= r2 < r1: cannot overflow
        int64_t s2 = csub(s0, cmul(q, s1));
        int64_t t2 = csub(t0, cmul(q, t1));
        r0 = r1; r1 = r2;
        s0 = s1; s1 = s2;
        t0 = t1; t1 = t2;
    }
    return Bezout{r0, a < 0 ? cneg(s0) : s0, b < 0 ? cneg(t0) : t0};
}

inline int64_t gcd64(int64_t a, int64_t b) { return egcd(a, b).g; }

// Small dense integer matrix, row-major.
struct IMat {
    int rows = 0, cols = 0;
    std::vector<int64_t> a;
    IMat() = default;
    IMat(int r, int c) : rows(r), cols(c), a((size_t)r * c, 0) {}
    int64_t &operator()(int i, int j) { return a[(size_t)i * cols + j]; }
    int64_t operator()(int i, int j) const { return a[(size_t)i * cols + j]; }
    static IMat identity(int n) {
        IMat m(n, n);
        for (int i = 0; i < n; ++i) m(i, i) = 1;
        return m;
    }
};

inline IMat matmul(const IMat &x, const IMat &y) {
    IMat r(x.rows, y.cols);
    for (int i = 0; i < x.rows; ++i)
        for (int j = 0; j < y.cols; ++j) {
            int64_t s = 0;
            for (int k = 0; k < x.cols; ++k) s = cadd(s, cmul(x(i, k), y(k, j)));
            r(i, j) = s;
        }
    return r;
}

}  // namespace tad
