// Kernel-argument builder for the reduction kernels (dtype independent).
#include "red_launch.hpp"

#include <cstring>

namespace ocn {

RedLauncher g_reduce_launchers[R_COUNT][DT_COUNT];
RedLauncher g_fused_launchers[B_COUNT][DT_COUNT][R_COUNT];

RedArgs make_red_args(const RedPlan &p, char *partial) {
  RedArgs r;
  std::memset(&r, 0, sizeof r);
  r.a = p.a_ptr;
  r.out = p.out_ptr;
  r.partial = partial;
  r.nkept = p.nkept;
  r.nred = p.nred;
  r.out_dtype = p.out_dtype;
  r.vec = p.vec;
  r.group = p.group;
  for (int k = 0; k < p.nkept; ++k) {  // fastest first
    const int d = p.nkept - 1 - k;
    r.ksa[k] = p.kstride_a[d];
    r.kso[k] = p.kstride_o[d];
    r.kdiv[k] = make_fastdiv((uint32_t)p.ksize[d]);
    r.ksize[k] = p.ksize[d];
    r.ksb[k] = p.kstride_b[d];
  }
  for (int k = 0; k < p.nred; ++k) {
    const int d = p.nred - 1 - k;
    r.rsa[k] = p.rstride_a[d];
    r.rdiv[k] = make_fastdiv((uint32_t)p.rsize[d]);
    r.rsize[k] = p.rsize[d];
    r.rsb[k] = p.rstride_b[d];
  }
  r.b = p.b_ptr;
  r.a_bcast = p.a_fast_bcast;
  r.b_bcast = p.b_fast_bcast;
  r.nout = p.nout;
  r.nredtot = p.nredtot;
  r.split = p.split;
  r.chunk = p.chunk;
  r.nt_load = p.nt_load ? 1 : 0;
  r.swap_a = p.swap_a ? 1 : 0;
  r.swap_o = p.swap_o ? 1 : 0;
  if (p.kernel == OCN_KERNEL_RED_ROWS) {
    r.n0 = p.rsize[p.nred - 1];
    const int64_t vpr = (r.n0 + p.vec - 1) / p.vec;
    r.vpr_div = make_fastdiv((uint32_t)(p.nred > 1 ? vpr : 1));
    r.nvec = vpr * (p.nredtot / r.n0);
  } else if (p.kernel == OCN_KERNEL_RED_COLS) {
    r.nc = p.ksize[p.nkept - 1];
    r.cpw = p.cpw;
    const int64_t colblocks = (r.nc + (int64_t)p.cpw * p.vec - 1) / ((int64_t)p.cpw * p.vec);
    r.colblocks_div = make_fastdiv((uint32_t)colblocks);
  }
  return r;
}

RedLeanArgs make_red_lean_args(const RedPlan &p, char *partial) {
  RedLeanArgs r;
  std::memset(&r, 0, sizeof r);
  r.a = p.a_ptr;
  r.out = p.out_ptr;
  r.partial = partial;
  r.b = p.b_ptr;
  r.ksa = p.nkept ? p.kstride_a[0] : 0;
  r.ksb = p.nkept ? p.kstride_b[0] : 0;
  r.kso = p.nkept ? p.kstride_o[0] : 0;
  r.nout = (uint32_t)p.nout;
  r.split = (uint32_t)p.split;
  r.nvec = (uint32_t)(p.nredtot / p.vec);
  r.chunk = (uint32_t)p.chunk;
  r.out_dtype = p.out_dtype;
  r.group = p.group;
  r.nt_load = p.nt_load ? 1 : 0;
  r.swap_a = p.swap_a ? 1 : 0;
  r.swap_o = p.swap_o ? 1 : 0;
  return r;
}

}  // namespace ocn
