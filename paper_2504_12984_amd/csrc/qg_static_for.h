// Compile-time loop: static_for<N>([&](auto I) { ... decltype(I)::value ... });
#pragma once
#include <type_traits>
#include <utility>

namespace qg {
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  [&]<int... I>(std::integer_sequence<int, I...>) __attribute__((always_inline)) {
    (f(std::integral_constant<int, I>{}), ...);
  }(std::make_integer_sequence<int, N>{});
}
}  // namespace qg
