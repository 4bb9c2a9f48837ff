// Instantiates one slice of the fused elementwise+reduce kernels and registers their
// launchers.  Included by fred_slice_*.hip with OCN_SLICE and OCN_NSLICES defined.
#include <utility>

#include "fred_kernels.hpp"
#include "red_launch.hpp"

namespace ocn {
namespace {

template <class G, int OP> hipError_t launch_fred(const RedPlan &p, char *partial, hipStream_t stream) {
  const RedArgs args = make_red_args(p, partial);
  switch (p.kernel) {
    case OCN_KERNEL_RED_ROWS:
      if (p.lean) {
        hipLaunchKernelGGL((fred_rows_lean_kernel<G, OP>), dim3((unsigned)p.grid), dim3(kBlock), 0, stream,
                           make_red_lean_args(p, partial));
        break;
      }
      if (p.short_rows) {
        hipLaunchKernelGGL((fred_rows_short_kernel<G, OP>), dim3((unsigned)p.grid), dim3(kBlock), 0, stream, args);
        break;
      }
      hipLaunchKernelGGL((fred_rows_kernel<G, OP>), dim3((unsigned)p.grid), dim3(kBlock), 0, stream, args);
      break;
    case OCN_KERNEL_RED_COLS:
      {
        using A = typename FusedFold<G, OP>::A;
        const size_t lds = cols_lds_bytes<A>((int)p.block, p.vec > 1 ? G::V : 1);
        hipLaunchKernelGGL((fred_cols_kernel<G, OP>), dim3((unsigned)p.grid), dim3((unsigned)p.block), lds, stream, args);
      }
      break;
    default:
      hipLaunchKernelGGL((fred_generic_kernel<G, OP>), dim3((unsigned)p.grid), dim3(kBlock), 0, stream, args);
      break;
  }
  return hipGetLastError();
}

// index I enumerates (elementwise op, input dtype, reduce op)
template <int I> void register_fused() {
  constexpr int ew = I / (DT_COUNT * R_COUNT), t = (I / R_COUNT) % DT_COUNT, r = I % R_COUNT;
  constexpr int mid = is_compare(ew) ? (int)DT_BOOL : t;
  if constexpr (fused_specialised(ew, t, t, mid, r)) {
    // deal the instantiated signatures (not the sparse index space) round-robin to the slices
    constexpr int ord = ew * 7 + t + r;
    if constexpr (ord % OCN_NSLICES == OCN_SLICE)
      g_fused_launchers[ew][t][r] = &launch_fred<Sig<ew, t, t, mid, 2>, r>;
  }
}
template <int... I> void register_all_fused(std::integer_sequence<int, I...>) { (register_fused<I>(), ...); }

}  // namespace

#define OCN_CAT2(a, b) a##b
#define OCN_CAT(a, b) OCN_CAT2(a, b)
void OCN_CAT(register_fred_slice_, OCN_SLICE)() {
  register_all_fused(std::make_integer_sequence<int, B_COUNT * DT_COUNT * R_COUNT>{});
}

}  // namespace ocn
