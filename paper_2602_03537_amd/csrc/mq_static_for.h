// Compile-time loop: static_for<N>([&](auto i) { constexpr int I = i; ... });
#pragma once
#include <utility>

namespace mq {
template <int I> struct IntC {
    static constexpr int value = I;
    __host__ __device__ constexpr operator int() const { return I; }
};
template <class F, int... Is>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, Is...>) {
    (f(IntC<Is>{}), ...);
}
template <int N, class F> __device__ __forceinline__ void static_for(F &&f) {
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}
}  // namespace mq
