// Instantiates one slice of the dtype-specialised elementwise kernels and registers their
// launchers.  Included by ew_slice_*.hip with OCN_SLICE and OCN_NSLICES defined; the slices
// only exist so that the kernels compile in parallel.
#include <utility>

#include "ew_launch.hpp"

namespace ocn {
namespace {

template <int I> void register_binary() {
  constexpr int op = I / DT_COUNT, t = I % DT_COUNT;
  if constexpr (I % OCN_NSLICES == OCN_SLICE) {
    if constexpr (is_arith(op) || is_bitwise(op)) {
      if constexpr (binary_specialised(op, t, t, t)) g_binary_launchers[op][t][t][t] = &launch_ew<op, t, t, t, 2>;
    } else if constexpr (is_logical(op)) {
      if constexpr (t == DT_BOOL) g_binary_launchers[op][t][t][t] = &launch_ew<op, t, t, t, 2>;
    } else {
      if constexpr (binary_specialised(op, t, t, DT_BOOL))
        g_binary_launchers[op][t][t][DT_BOOL] = &launch_ew<op, t, t, DT_BOOL, 2>;
    }
  }
}

// mixed input types, converted on load
template <int I> void register_mixed() {
  constexpr int op = I / kNumMixedPairs;
  constexpr MixedPair m = kMixedPairs[I % kNumMixedPairs];
  if constexpr (I % OCN_NSLICES == OCN_SLICE && binary_specialised(op, m.sa, m.sb, m.so))
    g_binary_launchers[op][m.sa][m.sb][m.so] = &launch_ew<op, m.sa, m.sb, m.so, 2>;
}

template <int I> void register_unary() {
  constexpr int op = I / (DT_COUNT * DT_COUNT), sa = (I / DT_COUNT) % DT_COUNT, so = I % DT_COUNT;
  if constexpr (I % OCN_NSLICES == OCN_SLICE && unary_specialised(op, sa, so))
    g_unary_launchers[op][sa][so] = &launch_ew<op, sa, sa, so, 1>;
}

template <int... I> void register_all_binary(std::integer_sequence<int, I...>) { (register_binary<I>(), ...); }
template <int... I> void register_all_mixed(std::integer_sequence<int, I...>) { (register_mixed<I>(), ...); }
// two levels (per operation, then per type pair) keep each fold expression short
template <int OP, int... I> void register_unary_op(std::integer_sequence<int, I...>) {
  (register_unary<OP * DT_COUNT * DT_COUNT + I>(), ...);
}
template <int... OP> void register_all_unary(std::integer_sequence<int, OP...>) {
  (register_unary_op<OP>(std::make_integer_sequence<int, DT_COUNT * DT_COUNT>{}), ...);
}

}  // namespace

#define OCN_CAT2(a, b) a##b
#define OCN_CAT(a, b) OCN_CAT2(a, b)
void OCN_CAT(register_ew_slice_, OCN_SLICE)() {
  register_all_binary(std::make_integer_sequence<int, B_COUNT * DT_COUNT>{});
  register_all_mixed(std::make_integer_sequence<int, kNumMixedOps * kNumMixedPairs>{});
  register_all_unary(std::make_integer_sequence<int, U_COUNT>{});
}

}  // namespace ocn
