// Products with the constant Winograd transform matrices, written so that every coefficient is a
// compile-time constant: zeros vanish and +-1 become an add or a subtract.
#ifndef IOLB_WINO_TRANSFORM_H
#define IOLB_WINO_TRANSFORM_H

#include <type_traits>
#include <utility>

#include "wino_mats.h"

namespace iolb {

// Compile-time loops: the body receives its index as an integral constant, so that a matrix coefficient
// read with it is a constant expression (a plain unrolled loop leaves the coefficient a run-time value,
// and every "is it zero / one" test becomes a branch).
template <class F, int... Is>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, Is...>)
{
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// which constant matrix of Mats<M> a product uses
struct UseA { template <int M> static constexpr float at(int i, int k) { return Mats<M>::A[i][k]; } };
struct UseB { template <int M> static constexpr float at(int i, int k) { return Mats<M>::B[i][k]; } };
struct UseL { template <int M> static constexpr float at(int i, int k) { return Mats<M>::L[i][k]; } };

// s += coef * v with the coefficient known at compile time: zeros vanish, +-1 are an add / subtract
template <int M, class Sel, int I, int K>
__device__ __forceinline__ void accumulate(float& s, bool& first, float v)
{
    constexpr float coef = Sel::template at<M>(I, K);
    if constexpr (coef != 0.f) {
        if (first) s = (coef == 1.f) ? v : (coef == -1.f) ? -v : coef * v;
        else       s = (coef == 1.f) ? s + v : (coef == -1.f) ? s - v : __builtin_fmaf(coef, v, s);
        first = false;
    }
}

// out[ROWS][COLS] = Mx[ROWS][IN] * in[IN][COLS], Mx = Sel's matrix of Mats<M>
template <int M, class Sel, int ROWS, int IN, int COLS>
__device__ __forceinline__ void left_mul(const float (&in)[IN][COLS], float (&out)[ROWS][COLS])
{
    static_for<ROWS>([&](auto i) {
        static_for<COLS>([&](auto j) {
            float s = 0.f;
            bool first = true;
            static_for<IN>([&](auto k) { accumulate<M, Sel, decltype(i)::value, decltype(k)::value>(s, first, in[k][j]); });
            out[i][j] = s;
        });
    });
}
// out[ROWS][COLS] = in[ROWS][IN] * Mx[COLS][IN]^T
template <int M, class Sel, int ROWS, int IN, int COLS>
__device__ __forceinline__ void right_mul_t(const float (&in)[ROWS][IN], float (&out)[ROWS][COLS])
{
    static_for<ROWS>([&](auto i) {
        static_for<COLS>([&](auto j) {
            float s = 0.f;
            bool first = true;
            static_for<IN>([&](auto k) { accumulate<M, Sel, decltype(j)::value, decltype(k)::value>(s, first, in[i][k]); });
            out[i][j] = s;
        });
    });
}

}  // namespace iolb

#endif
