// Host side of the elementwise kernels: turns a plan into kernel arguments and launches.
#pragma once

#include <hip/hip_runtime.h>

#include "ew_kernels.hpp"

namespace ocn {

using EwLauncher = hipError_t (*)(const EwPlan &, hipStream_t);

// dispatch tables, filled once by the kernel translation units (see ew_register.cpp)
extern EwLauncher g_binary_launchers[B_COUNT][DT_COUNT][DT_COUNT][DT_COUNT];
extern EwLauncher g_unary_launchers[U_COUNT][DT_COUNT][DT_COUNT];

RowsArgs make_rows_args(const EwPlan &p);
// arguments of the kernel for the common row shapes; false if the plan is not one of them
bool make_rows_slim_args(const EwPlan &p, int block, RowsSlimArgs *args, int64_t *grid);
TiledArgs make_tiled_args(const EwPlan &p, int es_a);
FastTiledArgs make_fast_tiled_args(const EwPlan &p, int es_a);
InterpArgs make_interp_args(const EwPlan &p);
hipError_t launch_interp(const EwPlan &p, hipStream_t stream);
hipError_t launch_interleave(const EwPlan &p, hipStream_t stream);

#if defined(__HIPCC__)
template <int OP, int SA, int SB, int SO, int NIN>
hipError_t launch_ew(const EwPlan &p, hipStream_t stream) {
  using G = Sig<OP, SA, SB, SO, NIN>;
  if (p.kernel == OCN_KERNEL_EW_ROWS) {
    RowsSlimArgs slim;
    int64_t slim_grid;
    if (make_rows_slim_args(p, kSlimBlock, &slim, &slim_grid)) {
      hipLaunchKernelGGL((ew_rows_slim_kernel<G>), dim3((unsigned)slim_grid), dim3(kSlimBlock), 0, stream, slim);
    } else {
      const RowsArgs args = make_rows_args(p);
      hipLaunchKernelGGL((ew_rows_kernel<G>), dim3((unsigned)p.grid), dim3(kBlock), 0, stream, args);
    }
  } else if (p.fast_tiled) {
    const FastTiledArgs args = make_fast_tiled_args(p, (int)sizeof(typename G::SAt));
    hipLaunchKernelGGL((ew_tiled_fast_kernel<G>), dim3((unsigned)p.grid), dim3(kBlock), (size_t)p.lds_bytes, stream, args);
  } else {
    const TiledArgs args = make_tiled_args(p, (int)sizeof(typename G::SAt));
    hipLaunchKernelGGL((ew_tiled_kernel<G>), dim3((unsigned)p.grid), dim3(kBlock), (size_t)p.lds_bytes, stream, args);
  }
  return hipGetLastError();
}
#endif

}  // namespace ocn
