// Scalar bodies  f = outer( sum_k inner(values) )  and their partial derivatives, as device code.
// The derivative of the "sum-liberated" function (Sec. 5.2) with respect to argument p at one
// extended index is  douter * dinner(p):  douter is expressed through the forward value f where
// that is possible (exp, tanh), so the backward pass reuses f instead of recomputing the sum.
#pragma once
#include <hip/hip_runtime.h>

#include "../../include/tad.h"

namespace tad {

template <typename T> __device__ __forceinline__ T t_exp(T x);
template <> __device__ __forceinline__ float t_exp<float>(float x) { return expf(x); }
template <> __device__ __forceinline__ double t_exp<double>(double x) { return exp(x); }
template <typename T> __device__ __forceinline__ T t_tanh(T x);
template <> __device__ __forceinline__ float t_tanh<float>(float x) { return tanhf(x); }
template <> __device__ __forceinline__ double t_tanh<double>(double x) { return tanh(x); }
template <typename T> __device__ __forceinline__ T t_sin(T x);
template <> __device__ __forceinline__ float t_sin<float>(float x) { return sinf(x); }
template <> __device__ __forceinline__ double t_sin<double>(double x) { return sin(x); }
template <typename T> __device__ __forceinline__ T t_cos(T x);
template <> __device__ __forceinline__ float t_cos<float>(float x) { return cosf(x); }
template <> __device__ __forceinline__ double t_cos<double>(double x) { return cos(x); }

template <int BODY> struct BodyTraits;
template <> struct BodyTraits<TAD_BODY_SQ> { static constexpr int NA = 1; };
template <> struct BodyTraits<TAD_BODY_CUBE> { static constexpr int NA = 1; };
template <> struct BodyTraits<TAD_BODY_SIN> { static constexpr int NA = 1; };
template <> struct BodyTraits<TAD_BODY_EXP> { static constexpr int NA = 1; };
template <> struct BodyTraits<TAD_BODY_MUL> { static constexpr int NA = 2; };
template <> struct BodyTraits<TAD_BODY_WORKED> { static constexpr int NA = 4; };
template <> struct BodyTraits<TAD_BODY_TANH_DOT> { static constexpr int NA = 2; };

template <int BODY, typename T> __device__ __forceinline__ T body_inner(const T *v) {
    if constexpr (BODY == TAD_BODY_MUL || BODY == TAD_BODY_TANH_DOT) {
        return v[0] * v[1];
    } else if constexpr (BODY == TAD_BODY_WORKED) {
        T t = v[0] + v[1];
        return t * t * v[2] + v[3] * v[3] * v[3];
    } else {
        return v[0];
    }
}

template <int BODY, typename T> __device__ __forceinline__ T body_outer(T s) {
    if constexpr (BODY == TAD_BODY_SQ) return s * s;
    else if constexpr (BODY == TAD_BODY_CUBE) return s * s * s;
    else if constexpr (BODY == TAD_BODY_SIN) return t_sin<T>(s);
    else if constexpr (BODY == TAD_BODY_EXP) return t_exp<T>(s);
    else if constexpr (BODY == TAD_BODY_WORKED) return t_exp<T>(-s);
    else if constexpr (BODY == TAD_BODY_TANH_DOT) return t_tanh<T>(s);
    else return s;
}

// d outer / d s, from the forward value f (and, for the bodies without a sum, from s = v[0])
template <int BODY, typename T> __device__ __forceinline__ T body_douter(T f, const T *v) {
    if constexpr (BODY == TAD_BODY_SQ) return T(2) * v[0];
    else if constexpr (BODY == TAD_BODY_CUBE) return T(3) * v[0] * v[0];
    else if constexpr (BODY == TAD_BODY_SIN) return t_cos<T>(v[0]);
    else if constexpr (BODY == TAD_BODY_EXP) return f;
    else if constexpr (BODY == TAD_BODY_WORKED) return -f;
    else if constexpr (BODY == TAD_BODY_TANH_DOT) return T(1) - f * f;
    else return T(1);
}

// d inner / d v[p]
template <int BODY, typename T> __device__ __forceinline__ T body_dinner(int p, const T *v) {
    if constexpr (BODY == TAD_BODY_MUL || BODY == TAD_BODY_TANH_DOT) {
        return p == 0 ? v[1] : v[0];
    } else if constexpr (BODY == TAD_BODY_WORKED) {
        T t = v[0] + v[1];
        if (p <= 1) return T(2) * t * v[2];
        if (p == 2) return t * t;
        return T(3) * v[3] * v[3];
    } else {
        return T(1);
    }
}

}  // namespace tad
