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
  r.nt_store = p.nt_store;
  r.swap = p.swap;
  r.nt_a = p.nt_a;
  r.nt_b = p.nt_b;
  return r;
}

bool make_rows_slim_args(const EwPlan &p, int block, RowsSlimArgs *args, int64_t *grid) {
  const int inner = p.ndim - 1;
  if (inner < 0 || inner > 1) return false;
  const int64_t n0 = p.size[inner];
  if (n0 % p.vec != 0) return false;
  const int64_t vpr = n0 / p.vec;
  const int64_t nvec = vpr * (inner == 1 ? p.size[0] : 1);
  const int64_t g = (nvec + (int64_t)block * p.unroll - 1) / ((int64_t)block * p.unroll);
  // 32-bit vector numbers (including those of the lanes past the end), one launch
  if (nvec >= ((int64_t)1 << 31) || g * block * p.unroll >= ((int64_t)1 << 32) || g > max_launch_blocks() || g < 1)
    return false;
  RowsSlimArgs r;
  std::memset(&r, 0, sizeof r);
  r.out = p.out.ptr;
  r.a = p.a.ptr;
  r.b = p.b.ptr;
  if (inner == 1) {
    r.so = p.out.stride[0];
    r.sa = p.a.stride[0];
    r.sb = p.b.stride[0];
  }
  r.nvec = (uint32_t)nvec;
  r.vpr_div = make_fastdiv((uint32_t)vpr);   // without an outer dim: row 0 for every vector
  r.flags = (p.a_inner_bcast ? kSlimABcast : 0u) | (p.b_inner_bcast ? kSlimBBcast : 0u) | (p.nt_a ? kSlimNtA : 0u) |
            (p.nt_b ? kSlimNtB : 0u) | (p.nt_store ? kSlimNtStore : 0u) | ((uint32_t)p.swap << kSlimSwapShift);
  *args = r;
  *grid = g;
  return true;
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
  t.nt_store = p.nt_store;
  t.swap = p.swap;
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
  // fastest dim is folded into the low slot bits, at the granularity of one LDS access of the
  // compute phase (the elements of a vector, at most 16 bytes), over as many bits as it takes
  // to spread the accesses of a wavefront over 128 bytes of banks
  auto make_swizzle = [&](const TileOrder &o, int es) {
    TileSwizzle z{0, 0, 0};
    if (p.nord == 0) return z;
    const int w_f = o.width[0] - o.vecw;             // vector positions along the operand's dim
    const int w_0 = p.tile_log2[p.ord_o[0]];         // bits of the output's fastest dim
    int dst = 0, want = 5;
    if (p.vecw_o > 0) {
      while (dst < p.vecw_o && (2 << dst) * es <= 16) ++dst;   // keep the groups read at once intact
      want = 0;
      while (((es << dst) << want) < 128) ++want;
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

FastTiledArgs make_fast_tiled_args(const EwPlan &p, int es_a) {
  const TiledArgs t = make_tiled_args(p, es_a);
  FastTiledArgs f;
  std::memset(&f, 0, sizeof f);
  f.out = t.out;
  f.a = t.a;
  f.b = t.b;
  f.stage_a = t.stage_a;
  f.stage_b = t.stage_b;
  f.nt_store = t.nt_store;
  f.swap = t.swap;
  // tile grid: only dims with more than one tile, fastest (last canonical dim) first.  Where
  // neighbouring tiles along one dim share input lines, that dim's tile index is split: its low
  // part (the group of tiles sharing a line) varies fastest of all, its high part stays in place.
  f.pair_log2 = p.pair_dim >= 0 ? p.pair_log2 : 0;
  auto add_dim = [&](int d, int64_t count, int64_t mult) {
    const int j = f.ntd++;
    f.ntdiv[j] = make_fastdiv((uint32_t)count);
    f.step[0][j] = t.so[d] * ((int64_t)mult << t.tl[d]);
    f.step[1][j] = t.sa[d] * ((int64_t)mult << t.tl[d]);
    f.step[2][j] = t.sb[d] * ((int64_t)mult << t.tl[d]);
  };
  const int64_t group = (int64_t)1 << f.pair_log2;
  if (f.pair_log2) add_dim(p.pair_dim, group, 1);
  for (int d = p.ndim - 1; d >= 0; --d) {
    const bool paired = f.pair_log2 && d == p.pair_dim;
    const int64_t count = paired ? p.ntiles[d] / group : p.ntiles[d];
    if (count <= 1) continue;
    add_dim(d, count, paired ? group : 1);
  }
  const int es[2] = {es_a, p.nin == 2 ? dt_size(p.b.dtype) : 1};
  // An input too large to be found in a cache again is read with streaming loads where every
  // run of it inside a tile - along its own fastest axis if it is staged, along the output's
  // if it is read in place - is a whole number of 128-byte lines starting on a line boundary
  // (a streaming load of part of a line runs at a fraction of the rate of an ordinary one).
  auto whole_lines = [&](const Operand &x, int esz, int run_dim) {
    if (x.stride[run_dim] != esz || (((int64_t)esz << p.tile_log2[run_dim]) % 128) != 0) return false;
    if (((intptr_t)x.ptr % 128) != 0) return false;
    int64_t distinct = esz;
    for (int d = 0; d < p.ndim; ++d) {
      if (x.stride[d] == 0) return false;
      if (d != run_dim && x.stride[d] % 128 != 0) return false;
      distinct *= p.size[d];
    }
    return distinct >= kStreamBytes;
  };
  if (p.nord > 0) {
    f.nt_a = whole_lines(p.a, es[0], p.stage_a ? p.ord_a[0] : p.ord_o[0]) ? 1 : 0;
    f.nt_b = p.nin == 2 && whole_lines(p.b, es[1], p.stage_b ? p.ord_b[0] : p.ord_o[0]) ? 1 : 0;
  }
  auto log2i = [](int64_t v) { int l = 0; while (((int64_t)1 << l) < v) ++l; return l; };
  const int64_t tile_elems = (int64_t)1 << p.tile_bits;
  // the larger staging area goes first, so that the smaller one starts at a multiple of its own
  // (power-of-two) size and the base can be OR-ed into XOR-built addresses
  const int64_t bytes_a = p.stage_a ? tile_elems * es[0] : 0, bytes_b = p.stage_b ? tile_elems * es[1] : 0;
  if (bytes_a >= bytes_b) { f.lds_base[0] = 0; f.lds_base[1] = (uint32_t)bytes_a; }
  else { f.lds_base[1] = 0; f.lds_base[0] = (uint32_t)bytes_b; }
  f.swz[0] = t.swz[0];
  f.swz[1] = t.swz[1];
  f.es_log2[0] = (uint32_t)log2i(es[0]);
  f.es_log2[1] = (uint32_t)log2i(es[1]);
  f.vc_log2 = (uint32_t)p.vecw_o;
  for (int x = 0; x < 3; ++x) {
    const TileOrder &o = t.ord[x];
    FastOrder &g = f.ord[x];
    g.niter = o.niter;
    uint32_t shift = 0;
    for (int k = 0; k < o.nord && shift < 8; ++k) {
      const uint32_t vw = k == 0 ? (uint32_t)o.vecw : 0u;
      const uint32_t w = (uint32_t)o.width[k] - vw;
      const uint32_t wl = std::min(w, 8u - shift);  // bits of this dim's index held by the lane number
      if (wl > 0) {
        const int i = g.nlane++;
        g.shift[i] = shift;
        g.mask[i] = (1u << wl) - 1u;
        g.up[i] = vw;
        g.slot_shift[i] = (uint32_t)o.lds_shift[k];
        for (int y = 0; y < 3; ++y) g.stride[y][i] = (uint32_t)o.stride[y][k];
      }
      shift += w;
    }
    for (int j = 0; j < o.niter && j < kMaxTilePasses; ++j)
      for (int y = 0; y < 3; ++y) g.hi_off[y][j] = (uint32_t)o.hi_off[y][j];
  }
  for (int y = 0; y < 2; ++y) {
    if (!(y == 0 ? p.stage_a : p.stage_b)) continue;
    const TileOrder &o = t.ord[y + 1];
    const TileSwizzle &z = t.swz[y];
    const uint32_t sh = f.es_log2[y];
    for (int j = 0; j < o.niter && j < kMaxTilePasses; ++j) f.st_hi[y][j] = swizzle(o.hi_slot[j], z) << sh;
    for (int i = 0; i < (1 << o.vecw) && i < 16; ++i) f.st_el[y][i] = swizzle((uint32_t)i << o.lds_shift[0], z) << sh;
    const TileOrder &oc = t.ord[0];
    for (int j = 0; j < oc.niter && j < kMaxTilePasses; ++j)
      f.rd_hi[y][j] = swizzle(((uint32_t)j * kBlock) << p.vecw_o, z) << sh;
    const int epc = std::min(std::max(1, 16 / es[y]), 1 << p.vecw_o);
    for (int c = 0; c * epc < (1 << p.vecw_o) && c < 16; ++c) f.rd_ch[y][c] = swizzle((uint32_t)(c * epc), z) << sh;
  }
  return f;
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
  a.swap = p.swap;
  a.vec = 1;
  // Four elements per lane where the innermost dim allows it: a multiple of four long,
  // contiguous in the output, contiguous or broadcast in the inputs, and every group of four
  // aligned as one access (at most 16 bytes).  The elementary functions stay at one.
  const bool elementary = p.nin == 1 && ((p.op >= U_SIN && p.op <= U_LOG) || (p.op >= U_ASIN && p.op <= U_TANH));
  if (p.ndim >= 1 && !elementary) {
    const int last = p.ndim - 1;
    auto fits = [&](const Operand &x, bool may_broadcast) {
      const int64_t es = dt_size(x.dtype), al = std::min<int64_t>(16, 4 * es);
      if (x.stride[last] == 0) return may_broadcast;
      if (x.stride[last] != es || (intptr_t)x.ptr % al) return false;
      for (int d = 0; d < last; ++d)
        if (x.stride[d] % al) return false;
      return true;
    };
    if (p.size[last] % 4 == 0 && fits(p.out, false) && fits(p.a, true) && (p.nin == 1 || fits(p.b, true))) {
      a.vec = 4;
      a.inner_a = p.a.stride[last] != 0;
      a.inner_b = p.nin == 2 && p.b.stride[last] != 0;
      a.size[last] /= 4;
      a.so[last] *= 4;
      a.sa[last] *= 4;
      a.sb[last] *= 4;
      a.numel /= 4;
    }
  }
  a.idx32 = a.numel < ((int64_t)1 << 31);
  if (a.idx32)
    for (int d = 0; d < p.ndim; ++d) a.div[d] = make_fastdiv((uint32_t)a.size[d]);
  return a;
}

}  // namespace ocn
