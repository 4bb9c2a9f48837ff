// Kernel-argument builders for the elementwise kernels (dtype independent).
#include "ew_launch.hpp"

#include <algorithm>
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
  t.tile_bits = p.tile_bits;
  t.total_tiles = (uint32_t)p.total_tiles;
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
  const int64_t tile_elems = (int64_t)1 << p.tile_bits;
  t.lds_off_b = p.stage_a ? (uint32_t)((tile_elems * es_a + 15) / 16 * 16) : 0u;
  // bit position of each tiled dim in the output's enumeration order = its LDS slot shift
  int slot_shift[kMaxDims] = {0};
  int acc = 0;
  for (int k = 0; k < p.nord; ++k) {
    slot_shift[p.ord_o[k]] = acc;
    acc += p.tile_log2[p.ord_o[k]];
  }
  const int8_t *ords[3] = {p.ord_o, p.ord_a, p.ord_b};
  const int vecw[3] = {p.vecw_o, p.vecw_a, p.vecw_b};
  for (int x = 0; x < 3; ++x) {
    TileOrder &o = t.ord[x];
    o.nord = (int8_t)p.nord;
    o.vecw = (int8_t)vecw[x];
    for (int k = 0; k < p.nord; ++k) {
      const int d = ords[x][k];
      o.dim[k] = (int8_t)d;
      o.width[k] = (int8_t)p.tile_log2[d];
      o.lds_shift[k] = (int8_t)slot_shift[d];
      o.stride[0][k] = p.out.stride[d];
      o.stride[1][k] = p.a.stride[d];
      o.stride[2][k] = p.b.stride[d];
    }
    const int64_t nvec = tile_elems >> vecw[x];
    o.niter = (int32_t)((nvec + kBlock - 1) / kBlock);
    // contribution of the pass number (bits 8 and up of the vector index) to offsets and slot
    for (int j = 0; j < o.niter && j < kMaxTilePasses; ++j) {
      const LanePos hi = lane_pos(o, (uint32_t)j * kBlock);
      for (int y = 0; y < 3; ++y) o.hi_off[y][j] = hi.off[y];
      o.hi_slot[j] = hi.slot;
    }
  }
  // XOR swizzle of a staged operand's LDS slots: the vector index along the operand's own
  // fastest dim is folded into the low slot bits, at 16-byte granularity when the compute
  // phase reads whole vectors and at element granularity otherwise
  auto make_swizzle = [&](const TileOrder &o, int es) {
    TileSwizzle z{0, 0, 0};
    if (p.nord == 0) return z;
    const int w_f = o.width[0] - o.vecw;             // vector positions along the operand's dim
    const int w_0 = p.tile_log2[p.ord_o[0]];         // bits of the output's fastest dim
    int dst = 0, want = 5;
    if (p.vecw_o > 0) {
      while ((1 << dst) * es < 16) ++dst;            // keep 16-byte groups intact
      want = 3;
    }
    if (dst > w_0) dst = w_0;
    int bits = std::min(want, std::min(w_f, w_0 - dst));
    if (bits < 0) bits = 0;
    z.src = (uint32_t)(o.lds_shift[0] + o.vecw);
    z.mask = (1u << bits) - 1u;
    z.dst = (uint32_t)dst;
    return z;
  };
  if (p.stage_a) t.swz[0] = make_swizzle(t.ord[1], es_a);
  if (p.stage_b) t.swz[1] = make_swizzle(t.ord[2], dt_size(p.b.dtype));
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
