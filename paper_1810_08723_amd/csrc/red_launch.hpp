// Host side of the reduction kernels.
#pragma once

#include <hip/hip_runtime.h>

#include "red_kernels.hpp"

namespace ocn {

using RedLauncher = hipError_t (*)(const RedPlan &, char *partial, hipStream_t);
extern RedLauncher g_reduce_launchers[R_COUNT][DT_COUNT];
// fused elementwise+reduce kernels: [elementwise op][input dtype (both inputs)][reduce op]
extern RedLauncher g_fused_launchers[B_COUNT][DT_COUNT][R_COUNT];

RedArgs make_red_args(const RedPlan &p, char *partial);
RedLeanArgs make_red_lean_args(const RedPlan &p, char *partial);

#if defined(__HIPCC__)
template <int S, int OP> hipError_t launch_red(const RedPlan &p, char *partial, hipStream_t stream) {
  const RedArgs args = make_red_args(p, partial);
  switch (p.kernel) {
    case OCN_KERNEL_RED_ROWS:
      if (p.lean) {
        hipLaunchKernelGGL((red_rows_lean_kernel<S, OP>), dim3((unsigned)p.grid), dim3(kBlock), 0, stream,
                           make_red_lean_args(p, partial));
        break;
      }
      if (p.short_rows) {
        hipLaunchKernelGGL((red_rows_short_kernel<S, OP>), dim3((unsigned)p.grid), dim3(kBlock), 0, stream, args);
        break;
      }
      hipLaunchKernelGGL((red_rows_kernel<S, OP>), dim3((unsigned)p.grid), dim3(kBlock), 0, stream, args);
      break;
    case OCN_KERNEL_RED_COLS:
      if (p.fold) {
        RedFoldArgs f;
        f.partial = p.a_ptr;
        f.out = p.out_ptr;
        f.kso = p.kstride_o[0];
        f.nout = (uint32_t)p.nout;
        f.split = (uint32_t)p.nredtot;
        f.out_dtype = p.out_dtype;
        f.swap_o = p.swap_o ? 1 : 0;
        hipLaunchKernelGGL((red_fold_kernel<S, OP>), dim3((unsigned)p.grid), dim3(kWave), 0, stream, f);
        break;
      }
      {
        using A = typename Reducer<S, OP>::A;
        constexpr int VF = 16 / (int)sizeof(storage_t<S>) > 0 ? 16 / (int)sizeof(storage_t<S>) : 1;
        const size_t lds = cols_lds_bytes<A>((int)p.block, p.vec > 1 ? VF : 1);
        hipLaunchKernelGGL((red_cols_kernel<S, OP>), dim3((unsigned)p.grid), dim3((unsigned)p.block), lds, stream, args);
      }
      break;
    default:
      hipLaunchKernelGGL((red_generic_kernel<S, OP>), dim3((unsigned)p.grid), dim3(kBlock), 0, stream, args);
      break;
  }
  return hipGetLastError();
}
#endif

}  // namespace ocn
