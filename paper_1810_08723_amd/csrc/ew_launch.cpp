// Kernel-argument builders for the elementwise kernels (dtype independent).
#include "ew_launch.hpp"

#include <cstring>

namespace ocn {

EwLauncher g_binary_launchers[B_COUNT][DT_COUNT][DT_COUNT][DT_COUNT];
EwLauncher g_unary_launchers[U_COUNT][DT_COUNT][DT_COUNT];

RowsArgs make_rows_args(const EwPlan &p) {
  RowsArgs r;
  std::memset(&r, 0, sizeof r);
  r.out = p.out.ptr;
  r.a = p.a.ptr;
  r.b = p.b.ptr;
  const int inner = p.ndim - 1;
  r.nouter = inner;
  for (int k = 0; k < inner; ++k) {  // fastest outer dim first
    const int d = inner - 1 - k;
    r.so[k] = p.out.stride[d];
    r.sa[k] = p.a.stride[d];
    r.sb[k] = p.b.stride[d];
    r.odiv[k] = make_fastdiv((uint32_t)p.size[d]);
  }
  r.inner = p.size[inner];
  const int64_t vpr = (r.inner + p.vec - 1) / p.vec;
  r.vpr_div = make_fastdiv((uint32_t)(inner > 0 ? vpr : 1));
  r.nvec = vpr * (p.numel / r.inner);
  r.a_bcast = p.a_inner_bcast;
  r.b_bcast = p.b_inner_bcast;
  return r;
}

TiledArgs make_tiled_args(const EwPlan &p, int es_a) {
  TiledArgs t;
  std::memset(&t, 0, sizeof t);
  t.out = p.out.ptr;
  t.a = p.a.ptr;
  t.b = p.b.ptr;
  t.ndim = p.ndim;
  t.nord = p.nord;
  t.tile_bits = p.tile_bits;
  for (int d = 0; d < p.ndim; ++d) {
    t.size[d] = p.size[d];
    t.so[d] = p.out.stride[d];
    t.sa[d] = p.a.stride[d];
    t.sb[d] = p.b.stride[d];
    t.tl[d] = p.tile_log2[d];
    t.ntdiv[d] = make_fastdiv((uint32_t)p.ntiles[d]);
  }
  t.stage_a = p.stage_a;
  t.stage_b = p.stage_b;
  t.pad_a = p.pad_shift_a;
  t.pad_b = p.pad_shift_b;
  const int64_t tile_elems = (int64_t)1 << p.tile_bits;
  t.lds_off_b = p.stage_a ? (uint32_t)(((tile_elems + (tile_elems >> p.pad_shift_a) + 1) * es_a + 15) / 16 * 16) : 0u;
  // bit position of each tiled dim in the output's enumeration order = its LDS slot shift
  int slot_shift[kMaxDims] = {0};
  int acc = 0;
  for (int k = 0; k < p.nord; ++k) {
    slot_shift[p.ord_o[k]] = acc;
    acc += p.tile_log2[p.ord_o[k]];
  }
  const int8_t *ords[3] = {p.ord_o, p.ord_a, p.ord_b};
  for (int x = 0; x < 3; ++x)
    for (int k = 0; k < p.nord; ++k) {
      const int d = ords[x][k];
      t.ord[x].dim[k] = (int8_t)d;
      t.ord[x].width[k] = (int8_t)p.tile_log2[d];
      t.ord[x].lds_shift[k] = (int8_t)slot_shift[d];
      t.ord[x].stride[0][k] = p.out.stride[d];
      t.ord[x].stride[1][k] = p.a.stride[d];
      t.ord[x].stride[2][k] = p.b.stride[d];
    }
  return t;
}

InterpArgs make_interp_args(const EwPlan &p) {
  InterpArgs a;
  std::memset(&a, 0, sizeof a);
  a.out = p.out.ptr;
  a.a = p.a.ptr;
  a.b = p.b.ptr;
  a.ndim = p.ndim;
  a.nin = p.nin;
  a.op = p.op;
  a.T = p.T;
  a.dt_a = p.a.dtype;
  a.dt_b = p.b.dtype;
  a.dt_o = p.out.dtype;
  for (int d = 0; d < p.ndim; ++d) {
    a.size[d] = p.size[d];
    a.so[d] = p.out.stride[d];
    a.sa[d] = p.a.stride[d];
    a.sb[d] = p.b.stride[d];
  }
  a.numel = p.numel;
  return a;
}

}  // namespace ocn
