// Instantiates one slice of the reduction kernels and registers their launchers.  Included
// by red_slice_*.hip with OCN_SLICE and OCN_NSLICES defined.
#include <utility>

#include "red_launch.hpp"

namespace ocn {
namespace {

template <int I> void register_reduce() {
  constexpr int op = I / DT_COUNT, s = I % DT_COUNT;
  if constexpr (I % OCN_NSLICES == OCN_SLICE && red_supported(op, s))
    g_reduce_launchers[op][s] = &launch_red<s, op>;
}
template <int... I> void register_all_reduce(std::integer_sequence<int, I...>) { (register_reduce<I>(), ...); }

}  // namespace

#define OCN_CAT2(a, b) a##b
#define OCN_CAT(a, b) OCN_CAT2(a, b)
void OCN_CAT(register_red_slice_, OCN_SLICE)() {
  register_all_reduce(std::make_integer_sequence<int, R_COUNT * DT_COUNT>{});
}

}  // namespace ocn
