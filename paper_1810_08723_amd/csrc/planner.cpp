// Host planner: see planner.hpp.  Plain C++, no HIP.
#include "planner.hpp"

#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <cstring>

#include "sigs.hpp"

namespace ocn {

// ---------------------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------------------

namespace {
std::atomic<int64_t> g_max_launch_blocks{((int64_t)1 << 24) - 1};
}
int64_t max_launch_blocks() { return g_max_launch_blocks.load(std::memory_order_relaxed); }
void set_max_launch_blocks(int64_t blocks) {
  const int64_t hard = ((int64_t)1 << 24) - 1;
  g_max_launch_blocks.store(blocks <= 0 || blocks > hard ? hard : blocks, std::memory_order_relaxed);
}

FastDiv make_fastdiv(uint32_t d) {
  // q = (mulhi(n, m) + n) >> s with s = ceil(log2 d), m = floor(2^32 (2^s - d) / d) + 1;
  // exact for every n < 2^31
  FastDiv f;
  f.d = d ? d : 1;
  uint32_t s = 0;
  while (((uint64_t)1 << s) < f.d) ++s;
  f.s = s;
  f.m = (uint32_t)(((((uint64_t)1 << s) - f.d) << 32) / f.d + 1);
  return f;
}

static bool valid_dtype(int dt) { return dt >= 0 && dt < DT_COUNT; }
static int scalar_size(int dt) { return dt_size(dt_real_of(dt)); }

static int check_tensor(const ocn_tensor *t) {
  if (!t) return OCN_ERR_NULLPTR;
  if (!valid_dtype(t->dtype)) return OCN_ERR_DTYPE;
  if (t->ndim < 0 || t->ndim > kMaxDims) return OCN_ERR_NDIM;
  bool empty = false;
  for (int d = 0; d < t->ndim; ++d) {
    if (t->size[d] < 0) return OCN_ERR_SHAPE;
    if (t->size[d] == 0) empty = true;
  }
  if (!empty && !t->base) return OCN_ERR_NULLPTR;
  return OCN_OK;
}

static int check_alignment(const ocn_tensor *t) {
  const int64_t sc = scalar_size(t->dtype);
  if (((intptr_t)t->base + t->offset) % sc != 0) return OCN_ERR_ALIGN;
  for (int d = 0; d < t->ndim; ++d)
    if (t->size[d] > 1 && t->stride[d] % sc != 0) return OCN_ERR_ALIGN;
  return OCN_OK;
}

// [lo, hi) of the bytes a view touches, relative to address zero
static void byte_range(const ocn_tensor *t, intptr_t *lo, intptr_t *hi) {
  intptr_t l = (intptr_t)t->base + t->offset, h = l;
  for (int d = 0; d < t->ndim; ++d) {
    if (t->size[d] <= 1) continue;
    int64_t span = (t->size[d] - 1) * t->stride[d];
    if (span < 0) l += span; else h += span;
  }
  *lo = l;
  *hi = h + dt_size(t->dtype);
}

// Conservative proof that no byte of the view is addressed twice: with dimensions sorted by
// |stride|, each stride must step over everything the faster dimensions span.
static bool provably_non_overlapping(const ocn_tensor *t) {
  int64_t st[kMaxDims], sz[kMaxDims];
  int n = 0;
  for (int d = 0; d < t->ndim; ++d) {
    if (t->size[d] <= 1) continue;
    st[n] = std::llabs(t->stride[d]);
    sz[n] = t->size[d];
    ++n;
  }
  for (int i = 1; i < n; ++i)  // insertion sort by stride, ascending
    for (int j = i; j > 0 && st[j] < st[j - 1]; --j) {
      std::swap(st[j], st[j - 1]);
      std::swap(sz[j], sz[j - 1]);
    }
  int64_t extent = dt_size(t->dtype);  // bytes spanned so far
  for (int i = 0; i < n; ++i) {
    if (st[i] < extent) return false;
    extent = (sz[i] - 1) * st[i] + extent;
  }
  return true;
}

// ---------------------------------------------------------------------------------------
// implicit casting (section 3.2.1): the smallest type that can keep both
// ---------------------------------------------------------------------------------------

static int int_bits_of(int dt) { return dt_size(dt) * 8; }

static int float_for_bits(int need_bits, int at_least) {
  // smallest real floating type with >= need_bits of exact integer range and >= at_least
  int r = at_least;
  if (need_bits > 11 && r < DT_F32) r = DT_F32;
  if (need_bits > 24 && r < DT_F64) r = DT_F64;
  return r;
}

static int promote_real(int a, int b) {
  const int ka = dt_kind(a), kb = dt_kind(b);
  if (ka == K_BOOL) return b;
  if (kb == K_BOOL) return a;
  if (ka == K_REAL && kb == K_REAL) return std::max(a, b);
  if (ka == K_REAL || kb == K_REAL) {
    const int f = ka == K_REAL ? a : b, i = ka == K_REAL ? b : a;
    // magnitude bits an integer type needs to be held exactly by a float significand
    const int need = dt_kind(i) == K_SINT ? int_bits_of(i) - 1 : int_bits_of(i);
    if (need > 53) return DT_F64;  // the paper's stated exception for 64-bit integers
    return float_for_bits(need, f);
  }
  if (ka == kb) return int_bits_of(a) >= int_bits_of(b) ? a : b;
  // signed with unsigned: a signed type strictly wider than the unsigned one
  const int s = ka == K_SINT ? a : b, u = ka == K_SINT ? b : a;
  const int ub = int_bits_of(u), sb = int_bits_of(s);
  if (sb > ub) return s;
  switch (ub) {
    case 8: return DT_I16;
    case 16: return DT_I32;
    case 32: return DT_I64;
    default: return DT_F64;  // nothing keeps uint64 and a signed integer
  }
}

int promote(int a, int b) {
  if (!valid_dtype(a) || !valid_dtype(b)) return OCN_ERR_DTYPE;
  if (dt_kind(a) == K_CPLX || dt_kind(b) == K_CPLX) {
    const int r = promote_real(dt_real_of(a), dt_real_of(b));
    return r == DT_F16 ? DT_C16 : r == DT_F32 ? DT_C32 : DT_C64;
  }
  return promote_real(a, b);
}

// ---------------------------------------------------------------------------------------
// elementwise planning
// ---------------------------------------------------------------------------------------

namespace {

struct Dim {
  int64_t size;
  int64_t so, sa, sb;
};

int64_t iabs64(int64_t x) { return x < 0 ? -x : x; }

int ilog2_ceil(int64_t x) {
  int l = 0;
  while (((int64_t)1 << l) < x) ++l;
  return l;
}

// is the input the identical view as the output (same address, element size and strides)?
bool same_view(const ocn_tensor *in, const ocn_tensor *out) {
  if ((intptr_t)in->base + in->offset != (intptr_t)out->base + out->offset) return false;
  if (dt_size(in->dtype) != dt_size(out->dtype)) return false;
  if (in->ndim != out->ndim) return false;
  for (int d = 0; d < out->ndim; ++d) {
    if (in->size[d] != out->size[d]) return false;
    if (out->size[d] > 1 && in->stride[d] != out->stride[d]) return false;
  }
  return true;
}

int check_alias(const ocn_tensor *in, const ocn_tensor *out) {
  if (same_view(in, out)) return OCN_OK;
  intptr_t ilo, ihi, olo, ohi;
  byte_range(in, &ilo, &ihi);
  byte_range(out, &olo, &ohi);
  if (ilo < ohi && olo < ihi) return OCN_ERR_ALIAS;
  return OCN_OK;
}

int check_broadcast(const ocn_tensor *in, const ocn_tensor *out) {
  if (in->ndim > out->ndim) return OCN_ERR_SHAPE;
  const int lead = out->ndim - in->ndim;
  for (int d = 0; d < in->ndim; ++d)
    if (in->size[d] != out->size[lead + d] && in->size[d] != 1) return OCN_ERR_SHAPE;
  return OCN_OK;
}

// stride of input along out's dimension d (zero where the input is broadcast)
int64_t bstride(const ocn_tensor *in, const ocn_tensor *out, int d) {
  const int lead = out->ndim - in->ndim;
  if (d < lead) return 0;
  return in->size[d - lead] == 1 ? 0 : in->stride[d - lead];
}

// the dimension with the smallest non-zero |stride| (ties: the later one); -1 if none
template <class Get> int fastest_dim(int n, Get stride_of) {
  int best = -1;
  int64_t bs = 0;
  for (int d = 0; d < n; ++d) {
    int64_t s = iabs64(stride_of(d));
    if (s == 0) continue;
    if (best < 0 || s <= bs) { best = d; bs = s; }
  }
  return best;
}

// order the tiled dims of one operand by that operand's |stride|, fastest first; zero
// strides (broadcast) go last since they do not affect coalescing
void tile_order(const EwPlan &p, const int64_t *stride, int8_t *ord) {
  int n = 0;
  for (int d = p.ndim - 1; d >= 0; --d)
    if (p.tile_log2[d] > 0) ord[n++] = (int8_t)d;
  auto key = [&](int d) {
    int64_t s = iabs64(stride[d]);
    return s == 0 ? INT64_MAX : s;
  };
  for (int i = 1; i < n; ++i)
    for (int j = i; j > 0 && key(ord[j]) < key(ord[j - 1]); --j) std::swap(ord[j], ord[j - 1]);
}

// LDS per workgroup, so that several share a CU's 160 KB.  A tile grows to the run lengths its
// operands want and no further: small tiles, i.e. many resident workgroups, measured faster
// than large ones on MI355X once every run is a full cache line.
constexpr int64_t kMaxLdsBytes = 32 * 1024;

void choose_tiles(EwPlan &p, bool general_form) {
  // Operands that want coalescing along their own fastest axis: the output and every staged
  // input.  Tile bits are handed out one at a time, each to the fastest unsaturated dimension
  // of one operand.  First every staged input is grown to a contiguous run of a full 128-byte
  // cache line (a shorter read run still fetches the whole line, and the other half is fetched
  // again by a neighbouring tile); the output to a full line as well when it is written with
  // streaming stores (partial-line streaming writes run at half rate), else to 64 bytes
  // (partial-line writes into the cache cost no extra traffic).  After that the tile only
  // grows, round-robin, until every enumeration order has a whole vector for each of the 256
  // lanes (which the lean kernel form needs); for the general form it grows on while the
  // staging areas stay within 16 KiB.
  const int es[3] = {dt_size(p.out.dtype), dt_size(p.a.dtype), p.nin == 2 ? dt_size(p.b.dtype) : 1};
  const int staged_bytes = (p.stage_a ? es[1] : 0) + (p.stage_b ? es[2] : 0);
  int budget = 12;
  while (budget > 8 && ((int64_t)staged_bytes << budget) > kMaxLdsBytes) --budget;
  const int es_max = std::max({es[0], es[1], p.nin == 2 ? es[2] : es[1]});
  const int vmax = std::max({rows_vec(es[0], es_max), p.stage_a ? 16 / es[1] : 1, p.stage_b ? 16 / es[2] : 1});
  int vbits = 0;
  while ((1 << vbits) < vmax) ++vbits;
  int preferred = std::min(budget, 8 + vbits);
  if (general_form) {  // larger tiles, within 16 KiB of LDS
    preferred = budget;
    while (preferred > 8 && ((int64_t)staged_bytes << preferred) > 16 * 1024) --preferred;
  }
  const int64_t *strides[3] = {p.out.stride, p.a.stride, p.b.stride};
  const bool wants[3] = {true, p.stage_a, p.stage_b};
  int used = 0;
  auto saturated = [&](int d) { return ((int64_t)1 << p.tile_log2[d]) >= p.size[d]; };
  // give operand o one more bit along its fastest unsaturated dim; false if it has none
  auto grow = [&](int o) {
    int best = -1;
    int64_t bs = 0;
    for (int d = 0; d < p.ndim; ++d) {
      if (saturated(d)) continue;
      const int64_t s = iabs64(strides[o][d]);
      if (s == 0) continue;
      if (best < 0 || s < bs || (s == bs && d > best)) { best = d; bs = s; }
    }
    if (best < 0) return false;
    ++p.tile_log2[best];
    ++used;
    return true;
  };
  // bytes of operand o that the tile covers contiguously, starting from its fastest dim
  auto run_bytes = [&](int o) {
    int64_t run = es[o];
    bool any = true;
    while (any) {
      any = false;
      for (int d = 0; d < p.ndim; ++d)
        if (p.tile_log2[d] > 0 && iabs64(strides[o][d]) == run) {
          const int64_t ext = std::min<int64_t>((int64_t)1 << p.tile_log2[d], p.size[d]);
          run *= ext;
          any = ext > 1 && ext == p.size[d] ? true : false;  // only a fully covered dim chains on
          if (!any) return run;
          break;
        }
    }
    return run;
  };
  const int64_t target[3] = {p.nt_store ? 128 : 64, 128, 128};
  bool progress = true;
  while (used < budget && progress) {
    progress = false;
    for (int o = 0; o < 3 && used < budget; ++o)
      if (wants[o] && run_bytes(o) < target[o] && grow(o)) progress = true;
  }
  progress = true;
  while (used < preferred && progress) {
    progress = false;
    for (int o = 0; o < 3 && used < preferred; ++o)
      if (wants[o] && grow(o)) progress = true;
  }
  p.tile_bits = used;
}

}  // namespace

int plan_elementwise(int nin, int op, const ocn_tensor *a, const ocn_tensor *b,
                     const ocn_tensor *out, uint32_t flags, EwPlan *plan) {
  EwPlan p;
  p.nin = nin;
  p.op = op;
  int rc;
  if ((rc = check_tensor(a)) != OCN_OK) return rc;
  if (nin == 2 && (rc = check_tensor(b)) != OCN_OK) return rc;
  if ((rc = check_tensor(out)) != OCN_OK) return rc;
  if (nin == 2 ? (op < 0 || op >= B_COUNT) : (op < 0 || op >= U_COUNT)) return OCN_ERR_OP;
  if (a->device != out->device || (nin == 2 && b->device != out->device)) return OCN_ERR_DEVICE;
  if ((rc = check_broadcast(a, out)) != OCN_OK) return rc;
  if (nin == 2 && (rc = check_broadcast(b, out)) != OCN_OK) return rc;

  // operands stored in the other byte order (section 3.1.3); one-byte scalars have no order
  p.swap = (a->byteswapped && scalar_size(a->dtype) > 1 ? 1 : 0) |
           (nin == 2 && b->byteswapped && scalar_size(b->dtype) > 1 ? 2 : 0) |
           (out->byteswapped && scalar_size(out->dtype) > 1 ? 4 : 0);

  // compute type and strict-mode checks (section 3.2.1)
  const int sa = a->dtype, sb = nin == 2 ? b->dtype : a->dtype, so = out->dtype;
  if (nin == 2) {
    if ((flags & OCN_STRICT_TYPES) && sa != sb) return OCN_ERR_DTYPE;
    if ((flags & OCN_STRICT_TYPES) && !is_compare(op) && !is_logical(op) && sa != so) return OCN_ERR_DTYPE;
    const int promoted = promote(sa, sb);
    p.T = binary_compute_dtype(op, sa, sb, so, promoted, promote(promoted, so));
    if (!binary_supported(op, p.T)) return OCN_ERR_DTYPE;
    p.specialised = binary_specialised(op, sa, sb, so);
  } else {
    const bool modulus = op == U_ABS && dt_kind(sa) == K_CPLX;   // complex -> real of the same precision
    if ((flags & OCN_STRICT_TYPES) && op != U_LNOT && sa != so && !(modulus && so == dt_real_of(sa)))
      return OCN_ERR_DTYPE;
    p.T = unary_compute_dtype(op, sa, so);
    if (!unary_supported(op, p.T)) return OCN_ERR_DTYPE;
    p.specialised = unary_specialised(op, sa, so);
  }

  int64_t numel = 1;
  for (int d = 0; d < out->ndim; ++d) numel *= out->size[d];
  p.numel = numel;
  if (numel == 0) {  // nothing to do
    *plan = p;
    return OCN_OK;
  }
  if ((rc = check_alignment(a)) != OCN_OK) return rc;
  if (nin == 2 && (rc = check_alignment(b)) != OCN_OK) return rc;
  if ((rc = check_alignment(out)) != OCN_OK) return rc;
  if (!provably_non_overlapping(out)) return OCN_ERR_OVERLAP_OUT;
  if ((rc = check_alias(a, out)) != OCN_OK) return rc;
  if (nin == 2 && (rc = check_alias(b, out)) != OCN_OK) return rc;

  // ---- canonical dimension list ---------------------------------------------------------
  Dim dims[kMaxDims];
  int n = 0;
  int64_t off_o = out->offset, off_a = a->offset, off_b = nin == 2 ? b->offset : 0;
  for (int d = 0; d < out->ndim; ++d) {
    if (out->size[d] == 1) continue;  // drop
    Dim x{out->size[d], out->stride[d], bstride(a, out, d), nin == 2 ? bstride(b, out, d) : 0};
    if (x.so < 0) {  // flip so that the output walks forward
      off_o += (x.size - 1) * x.so;
      off_a += (x.size - 1) * x.sa;
      off_b += (x.size - 1) * x.sb;
      x.so = -x.so; x.sa = -x.sa; x.sb = -x.sb;
    }
    dims[n++] = x;
  }
  // sort by output stride, slowest first (insertion sort: n <= 8, and stable)
  for (int i = 1; i < n; ++i)
    for (int j = i; j > 0 && dims[j].so > dims[j - 1].so; --j) std::swap(dims[j], dims[j - 1]);
  // merge neighbours that every operand walks as one longer dimension
  int m = 0;
  for (int i = 0; i < n; ++i) {
    if (m > 0) {
      Dim &u = dims[m - 1];
      const Dim &v = dims[i];
      if (u.so == v.so * v.size && u.sa == v.sa * v.size && u.sb == v.sb * v.size) {
        u.size *= v.size;
        u.so = v.so; u.sa = v.sa; u.sb = v.sb;
        continue;
      }
    }
    dims[m++] = dims[i];
  }
  n = m;
  if (n == 0) {  // a single element
    dims[0] = Dim{1, (int64_t)dt_size(so), 0, 0};
    n = 1;
  }
  p.ndim = n;
  for (int d = 0; d < n; ++d) {
    p.size[d] = dims[d].size;
    p.out.stride[d] = dims[d].so;
    p.a.stride[d] = dims[d].sa;
    p.b.stride[d] = dims[d].sb;
  }
  p.off_out = off_o; p.off_a = off_a; p.off_b = off_b;
  p.out.ptr = (char *)out->base + off_o; p.out.dtype = so;
  p.a.ptr = (char *)a->base + off_a; p.a.dtype = sa;
  p.b.ptr = nin == 2 ? (char *)b->base + off_b : nullptr; p.b.dtype = sb;

  // ---- kernel selection ------------------------------------------------------------------
  const int es_o = dt_size(so), es_a = dt_size(sa), es_b = dt_size(sb);
  // An output of 32 MiB or more will not be found in the caches by whoever reads it next
  // (4 MB of L2 per XCD, 256 MB of Infinity Cache shared with the inputs): write it with
  // streaming stores, so that its dirty lines do not burden the next kernel.
  p.nt_store = numel * es_o >= kStreamBytes;
  const int inner = n - 1;
  const int es_max = std::max({es_o, es_a, nin == 2 ? es_b : es_a});
  const int es_min = std::min({es_o, es_a, nin == 2 ? es_b : es_a});
  const int VT = rows_vec(es_o, es_max);                    // the tiled kernel's compute vector (Sig::V)
  const int V = rows_stream_vec(es_o, es_min, es_max);      // the rows kernel's vector (Sig::VR)
  auto inner_ok = [&](int64_t stride, int es) { return stride == es || stride == 0; };
  bool rows = p.specialised && p.out.stride[inner] == es_o && inner_ok(p.a.stride[inner], es_a) &&
              (nin == 1 || inner_ok(p.b.stride[inner], es_b));
  if (rows) {
    // every row start of every non-broadcast operand must be aligned to its vector
    auto aligned = [&](const Operand &x, int es) {
      if (x.stride[inner] == 0) return true;
      const int64_t vb = (int64_t)V * es;
      if ((intptr_t)x.ptr % vb != 0) return false;
      for (int d = 0; d < inner; ++d)
        if (x.stride[d] % vb != 0) return false;
      return true;
    };
    rows = aligned(p.out, es_o) && aligned(p.a, es_a) && (nin == 1 || aligned(p.b, es_b));
    // 32-bit vector and row indices (a flat 1-D tensor needs no division and may be larger)
    const int64_t vpr = (p.size[inner] + V - 1) / V;
    const int64_t nrows = numel / p.size[inner];
    if (n > 1 && (vpr * nrows >= ((int64_t)1 << 31))) rows = false;
    // more workgroups than one launch may have: the generic kernel, which loops, takes it
    if ((vpr * nrows + (int64_t)kBlock * rows_stream_unroll(V, es_min) - 1) /
            ((int64_t)kBlock * rows_stream_unroll(V, es_min)) > max_launch_blocks()) {
      rows = false;
      p.specialised = false;
    }
    if (rows) {
      p.kernel = OCN_KERNEL_EW_ROWS;
      p.vec = V;
      p.unroll = rows_stream_unroll(V, es_min);
      p.a_inner_bcast = p.a.stride[inner] == 0;
      p.b_inner_bcast = nin == 2 && p.b.stride[inner] == 0;
      // Inputs too large to be found in a cache again are read with streaming loads: those
      // that move one piece per lane and are not broadcast along any dim (a broadcast operand
      // is re-read from the caches by every row).
      auto streamed = [&](const Operand &x, int es) {
        if (V * es > 16) return false;
        int64_t distinct = es;
        for (int d = 0; d < n; ++d) {
          if (x.stride[d] == 0) return false;
          distinct *= p.size[d];
        }
        return distinct >= kStreamBytes;
      };
      p.nt_a = streamed(p.a, es_a);
      p.nt_b = nin == 2 && streamed(p.b, es_b);
      const int64_t nvec = vpr * nrows;
      p.grid = (nvec + (int64_t)kBlock * p.unroll - 1) / ((int64_t)kBlock * p.unroll);
      p.lds_bytes = 0;
      *plan = p;
      return OCN_OK;
    }
  }

  // A plain copy from planes into an output whose fastest axis is 2..8 elements long, the
  // next output axis being the input's fastest (channel-first to channel-last): lanes take
  // 16-byte vectors along that long axis and deal them out in registers.
  if (nin == 1 && op == U_IDENT && sa == so && es_o <= 8 && n >= 2 && (p.swap == 0 || p.swap == 5)) {
    const int64_t c = p.size[n - 1], mlen = p.size[n - 2], vv = 16 / es_o;
    bool ok = c >= 2 && c <= 8 && p.out.stride[n - 1] == es_o && p.out.stride[n - 2] == c * es_o &&
              p.a.stride[n - 2] == es_o && p.a.stride[n - 1] % 16 == 0 && mlen % vv == 0 &&
              (intptr_t)p.out.ptr % 16 == 0 && (intptr_t)p.a.ptr % 16 == 0;
    for (int d = 0; d < n - 2 && ok; ++d) ok = p.out.stride[d] % 16 == 0 && p.a.stride[d] % 16 == 0;
    const int64_t nvec = numel / (c * vv);
    const int64_t grid = (nvec + kBlock - 1) / kBlock;
    if (ok && nvec < ((int64_t)1 << 31) && grid <= max_launch_blocks()) {
      p.kernel = OCN_KERNEL_EW_INTERLEAVE;
      p.vec = (int)vv;
      p.grid = grid;
      p.nt_a = numel * es_o >= kStreamBytes;
      p.lds_bytes = (int64_t)kBlock * c * 16;
      *plan = p;
      return OCN_OK;
    }
  }

  if (!p.specialised) {
    // generic-dtype kernel: one element per lane, conversions through runtime switches
    p.kernel = OCN_KERNEL_EW_GENERIC;
    p.vec = 1;
    p.grid = std::min<int64_t>((numel + kBlock - 1) / kBlock, max_launch_blocks());   // the kernel loops beyond that
    *plan = p;
    return OCN_OK;
  }

  // tiled / generic: stage an input through LDS when its fastest axis is not the output's
  const int fo = inner;  // the output's fastest dim after sorting
  const int fa = fastest_dim(n, [&](int d) { return p.a.stride[d]; });
  const int fb = nin == 2 ? fastest_dim(n, [&](int d) { return p.b.stride[d]; }) : -1;
  p.stage_a = fa >= 0 && fa != fo;
  p.stage_b = fb >= 0 && fb != fo;
  // First the small tiles that suit the unclipped all-vector form of the tiled kernel.  A plan
  // that cannot take that form is laid out again for the general form, which wants larger
  // tiles (its per-tile overhead is higher), and without staging for inputs whose own fastest
  // axis is shorter than 32 bytes: coalescing along such an axis gains less than the general
  // form's staging costs (measured on channel-last to channel-first copies with 3 channels).
  bool stage_a0 = p.stage_a, stage_b0 = p.stage_b;
  for (int attempt = 0; attempt < 2; ++attempt) {
    if (attempt == 1) {
      if (stage_a0 && p.size[fa] * es_a < 32) stage_a0 = false;
      if (stage_b0 && p.size[fb] * es_b < 32) stage_b0 = false;
    }
    p.stage_a = stage_a0;
    p.stage_b = stage_b0;
    for (int d = 0; d < kMaxDims; ++d) p.tile_log2[d] = 0;
    p.fast_tiled = false;
    choose_tiles(p, attempt == 1);
    tile_order(p, p.out.stride, p.ord_o);
    tile_order(p, p.a.stride, p.ord_a);
    tile_order(p, p.b.stride, p.ord_b);
    p.nord = 0;
    for (int d = 0; d < n; ++d)
      if (p.tile_log2[d] > 0) ++p.nord;
    // an input whose fastest tiled dim is the output's needs no staging after all
    if (p.nord == 0 || p.ord_a[0] == p.ord_o[0]) p.stage_a = false;
    if (p.nord == 0 || p.ord_b[0] == p.ord_o[0]) p.stage_b = false;

    // ---- vector widths of the three enumeration orders -----------------------------------
    // aligned: base pointer and every stride except the one along `skip` are multiples of vb
    auto aligned = [&](const Operand &x, int64_t vb, int skip) {
      if ((intptr_t)x.ptr % vb != 0) return false;
      for (int d = 0; d < n; ++d)
        if (d != skip && x.stride[d] % vb != 0) return false;
      return true;
    };
    auto log2i = [](int v) { int l = 0; while ((1 << l) < v) ++l; return l; };
    p.vecw_o = p.vecw_a = p.vecw_b = 0;
    if (p.nord > 0) {
      const int d0 = p.ord_o[0];
      // compute phase: V consecutive elements along the output's fastest dim per lane
      bool ok = p.out.stride[d0] == es_o && p.tile_log2[d0] >= log2i(VT) && VT > 1 &&
                aligned(p.out, (int64_t)VT * es_o, d0);
      auto direct_ok = [&](const Operand &x, int es, bool staged) {
        if (staged) return true;
        if (x.stride[d0] != es) return true;  // broadcast or strided: element loads, no constraint
        return aligned(x, (int64_t)VT * es, d0);
      };
      ok = ok && direct_ok(p.a, es_a, p.stage_a) && (nin == 1 || direct_ok(p.b, es_b, p.stage_b));
      if (ok) p.vecw_o = log2i(VT);
      auto stage_vec = [&](const Operand &x, int es, const int8_t *ord) {
        const int v = 16 / es;
        if (v <= 1) return 0;
        const int f = ord[0];
        if (x.stride[f] != es || p.tile_log2[f] < log2i(v) || !aligned(x, 16, f)) return 0;
        return log2i(v);
      };
      if (p.stage_a) p.vecw_a = stage_vec(p.a, es_a, p.ord_a);
      if (p.stage_b) p.vecw_b = stage_vec(p.b, es_b, p.ord_b);
    }
    const int64_t tile_elems = (int64_t)1 << p.tile_bits;
    p.lds_bytes = 0;
    if (p.stage_a) p.lds_bytes += (tile_elems * es_a + 15) / 16 * 16;
    if (p.stage_b) p.lds_bytes += (tile_elems * es_b + 15) / 16 * 16;
    p.total_tiles = 1;
    for (int d = 0; d < n; ++d) {
      p.ntiles[d] = (p.size[d] + ((int64_t)1 << p.tile_log2[d]) - 1) >> p.tile_log2[d];
      p.total_tiles *= p.ntiles[d];
    }
    // One tile per workgroup.  (Persistent workgroups looping over tiles, and handing each XCD
    // a contiguous range of tiles, were both measured slower on MI355X.)
    p.grid = p.total_tiles;
    p.kernel = (p.stage_a || p.stage_b) ? OCN_KERNEL_EW_TILED : OCN_KERNEL_EW_GENERIC;
    // The unclipped all-vector form of the tiled kernel: no tile is clipped, every enumeration
    // order moves whole vectors over at least one full pass, inputs that are not staged are
    // contiguous along the output's fastest dim, and inside a tile every stride is non-negative
    // with offsets that fit 31 bits.
    if (p.kernel == OCN_KERNEL_EW_TILED && p.vecw_o > 0) {
      bool ok = true;
      const int d0 = p.ord_o[0];
      if (p.stage_a ? p.vecw_a == 0 : p.a.stride[d0] != es_a) ok = false;
      if (nin == 2 && (p.stage_b ? p.vecw_b == 0 : p.b.stride[d0] != es_b)) ok = false;
      const int vmax = std::max(p.vecw_o, std::max(p.stage_a ? p.vecw_a : 0, p.stage_b ? p.vecw_b : 0));
      if (p.tile_bits - vmax < 8) ok = false;  // fewer vectors than lanes in some order
      int64_t span_o = 0, span_a = 0, span_b = 0;
      for (int d = 0; d < n && ok; ++d) {
        const int64_t ext = (int64_t)1 << p.tile_log2[d];
        if (p.size[d] % ext != 0) ok = false;
        if (ext > 1 && (p.a.stride[d] < 0 || p.b.stride[d] < 0)) ok = false;
        span_o += (ext - 1) * p.out.stride[d];
        span_a += (ext - 1) * iabs64(p.a.stride[d]);
        span_b += (ext - 1) * iabs64(p.b.stride[d]);
      }
      const int64_t lim = ((int64_t)1 << 31) - 64;
      p.fast_tiled = ok && span_o < lim && span_a < lim && span_b < lim;
    }
    if (p.fast_tiled) {
      // An input whose contiguous run inside a tile is a fraction of a 128-byte line shares its
      // lines with the neighbouring tiles along the dim that continues the run.  Such tiles are
      // handed to workgroups that land on the same XCD one after the other (see the kernel), so
      // that the line is fetched into that L2 once instead of once per tile.
      p.pair_dim = -1;
      p.pair_log2 = 0;
      const Operand *ins[2] = {&p.a, &p.b};
      const int es_in[2] = {es_a, es_b};
      for (int x = 0; x < nin && p.pair_dim < 0; ++x) {
        int64_t run = es_in[x];
        int cont = -1;
        for (bool more = true; more;) {
          more = false;
          for (int d = 0; d < n; ++d) {
            if (iabs64(ins[x]->stride[d]) != run || p.size[d] == 1) continue;
            const int64_t ext = (int64_t)1 << p.tile_log2[d];
            if (ext >= p.size[d]) {  // fully covered: the run goes on along another dim
              run *= p.size[d];
              more = true;
            } else {                 // the neighbouring tiles along d continue the run
              run *= ext;
              cont = d;
            }
            break;
          }
        }
        if (cont < 0 || run >= 128 || 128 % run != 0 || ins[x]->stride[cont] < 0) continue;
        const int lg = run == 64 ? 1 : run == 32 ? 2 : 0;
        if (lg == 0 || p.ntiles[cont] % (1 << lg) != 0 || p.total_tiles % (8 << lg) != 0) continue;
        p.pair_dim = cont;
        p.pair_log2 = lg;
      }
      break;
    }
  }  // attempts
  p.vec = 1 << p.vecw_o;
  if (p.total_tiles >= ((int64_t)1 << 31)) {  // tile coordinates are 32-bit: use the 64-bit generic kernel
    p.specialised = false;
    p.kernel = OCN_KERNEL_EW_GENERIC;
    p.vec = 1;
    p.stage_a = p.stage_b = false;
    p.lds_bytes = 0;
    p.grid = (numel + kBlock - 1) / kBlock;
  }
  *plan = p;
  return OCN_OK;
}

// ---------------------------------------------------------------------------------------
// reduction planning
// ---------------------------------------------------------------------------------------

bool reduce_supported(int op, int dt) {
  if (op < 0 || op >= R_COUNT || !valid_dtype(dt)) return false;
  const int k = dt_kind(dt);
  switch (op) {
    case R_SUM: case R_ANY: case R_ALL: return true;
    default: return k != K_CPLX;
  }
}

int reduce_acc_dtype(int op, int dt) {
  const int k = dt_kind(dt);
  switch (op) {
    case R_SUM: case R_PROD:
      if (k == K_BOOL || k == K_SINT) return DT_I64;
      if (k == K_UINT) return DT_U64;
      if (dt == DT_F16) return DT_F32;
      if (dt == DT_F32 || dt == DT_F64) return DT_F64;
      return dt == DT_C16 ? DT_C32 : DT_C64;
    case R_MIN: case R_MAX: return dt;
    default: return DT_BOOL;
  }
}

namespace {

struct RDim { int64_t size, sa, so, sb; };

// sorts by decreasing key, then merges neighbours that every operand walks as one longer dim
template <class Key> int sort_merge_by(RDim *d, int n, Key key) {
  for (int i = 1; i < n; ++i)
    for (int j = i; j > 0 && key(d[j]) > key(d[j - 1]); --j) std::swap(d[j], d[j - 1]);
  int m = 0;
  for (int i = 0; i < n; ++i) {
    if (m > 0) {
      RDim &u = d[m - 1];
      const RDim &v = d[i];
      if (u.sa == v.sa * v.size && u.so == v.so * v.size && u.sb == v.sb * v.size) {
        u.size *= v.size; u.sa = v.sa; u.so = v.so; u.sb = v.sb;
        continue;
      }
    }
    d[m++] = d[i];
  }
  return m;
}

int sort_merge(RDim *d, int n, bool by_out) {
  return sort_merge_by(d, n, [&](const RDim &x) { return by_out ? x.so : iabs64(x.sa); });
}

#ifndef OCN_RED_TARGET_WAVES
#define OCN_RED_TARGET_WAVES (256 * 16)
#endif
constexpr int64_t kTargetWaves = OCN_RED_TARGET_WAVES;  // enough wavefronts to occupy every CU
// A row reduction that runs in the lean form of the kernel and has to be split over workgroups
// is split into half as many wavefronts, eight per CU: with four 16-byte loads per lane in
// flight that measured fastest (int8 full sum of 2^28: 41.9 us, against 45.2, 44.7 and 43.6 with
// 6, 12 and 16 per CU; the count of a > b over 2^26 pairs: 81.7 against 83.2 with 16).  The
// general kernel's element loads want the sixteen (full sum of a stride-2 view: 96 against 104 us).
constexpr int64_t kLeanSplitWaves = 256 * 8;

void choose_reduce_launch(RedPlan &p) {
  const int es = dt_size(p.a_dtype);
  const int acc_es = dt_size(p.acc_dtype);
  // fastest dims
  const int64_t r_fast = p.nred ? iabs64(p.rstride_a[p.nred - 1]) : 0;
  int64_t k_fast = 0;  // smallest non-zero kept stride of the input
  int k_fast_dim = -1;
  for (int d = 0; d < p.nkept; ++d) {
    int64_t s = iabs64(p.kstride_a[d]);
    if (s && (k_fast_dim < 0 || s <= k_fast)) { k_fast = s; k_fast_dim = d; }
  }
  const int vfull = std::max(1, 16 / es);
  auto all_aligned = [&](int64_t vb, int skip_kept, int skip_red) {
    if ((intptr_t)p.a_ptr % vb) return false;
    for (int d = 0; d < p.nkept; ++d)
      if (d != skip_kept && p.kstride_a[d] % vb) return false;
    for (int d = 0; d < p.nred; ++d)
      if (d != skip_red && p.rstride_a[d] % vb) return false;
    return true;
  };
  bool idx32 = p.nout < ((int64_t)1 << 31) && p.nredtot < ((int64_t)1 << 31);
  for (int d = 0; d < p.nkept; ++d) idx32 = idx32 && p.ksize[d] < ((int64_t)1 << 31);
  for (int d = 0; d < p.nred; ++d) idx32 = idx32 && p.rsize[d] < ((int64_t)1 << 31);
  // a flat contiguous full reduction may be longer than 2^31 elements
  const bool flat_full = p.nkept == 0 && p.nred == 1;

  const bool rows_contig = p.nred >= 1 && r_fast == es && (k_fast_dim < 0 || k_fast > r_fast);
  const bool cols_ok = k_fast_dim >= 0 && k_fast == es && p.kstride_a[k_fast_dim] == es &&
                       (p.nred == 0 || r_fast == 0 || r_fast > k_fast) && p.nredtot >= 1 && idx32 &&
                       k_fast_dim == p.nkept - 1 && p.nred >= 1;
  if (p.nred >= 1 && (idx32 || flat_full) && (rows_contig || !cols_ok)) {
    // ---- rows: lanes share an output ---------------------------------------------------
    // With the reduced axis the input's fastest, lanes load whole vectors; any other layout
    // goes element by element with the innermost reduced stride.
    p.kernel = OCN_KERNEL_RED_ROWS;
    p.vec = rows_contig && all_aligned((int64_t)vfull * es, -1, p.nred - 1) ? vfull : 1;
    const int64_t n0 = p.rsize[p.nred - 1];
    const int64_t vpr = (n0 + p.vec - 1) / p.vec;         // vectors per innermost run
    const int64_t nvec = vpr * (p.nredtot / n0);          // vectors per output
    int64_t cover = 1;                                    // lanes one output can keep busy
    while (cover < nvec && cover < kBlock) cover <<= 1;
    if (rows_contig || k_fast_dim < 0 || r_fast < k_fast) {
      // neighbouring lanes read neighbouring addends
      // a whole workgroup only when each of its lanes gets at least four vectors (the depth of
      // the unrolled loop): rows of 10 to 14 KiB measured 10-20 % slower on 256 lanes than on 64
      p.group = nvec < 4 * kBlock ? (int)std::min<int64_t>(cover, kWave) : kBlock;
    } else {
      // a kept axis is faster: neighbouring lanes take neighbouring outputs, and share one
      // only as far as it takes to fill the device
      int64_t need = 1;
      while (need * p.nout < kTargetWaves * kWave && need < cover) need <<= 1;
      p.group = need > kWave ? kBlock : (int)need;
    }
    const int64_t groups_per_block = kBlock / p.group;
    const int64_t waves = (p.nout * p.group + kWave - 1) / kWave;
    p.split = 1;
    // the common 2-D shape: one reduced dim of whole vectors, at most one kept dim, a wavefront or
    // a workgroup per output (or per split of it), everything below 2^31
    const bool lean_shape = p.nred == 1 && p.nkept <= 1 && p.vec > 1 && es < 16 && n0 % p.vec == 0 &&
                            p.group >= kWave && nvec < ((int64_t)1 << 31);
    if (p.group >= kWave && waves < kTargetWaves) {
      // split long reductions so the device fills; keep >= 16 vectors per lane per split
      const int64_t want = ((lean_shape ? kLeanSplitWaves : kTargetWaves) + waves - 1) / waves;
      const int64_t most = std::max<int64_t>(1, nvec / ((int64_t)p.group * 16));
      p.split = std::max<int64_t>(1, std::min(want, most));
    }
    p.chunk = (nvec + p.split - 1) / p.split;
    p.split = (nvec + p.chunk - 1) / p.chunk;
    p.grid = (p.nout * p.split + groups_per_block - 1) / groups_per_block;
    p.short_rows = p.group <= kWave && nvec <= p.group && p.nred == 1 && p.split == 1 &&
                   p.nout * p.group < ((int64_t)1 << 32) && n0 < ((int64_t)1 << 31);
    p.lean = !p.short_rows && lean_shape && p.nout * p.split < ((int64_t)1 << 31) && p.chunk < ((int64_t)1 << 31);
  } else if (cols_ok) {
    // ---- cols: a kept axis is the input's fastest; lanes own output columns -------------
    // (requires that axis to be the last canonical kept dim, i.e. also the output's fastest)
    p.kernel = OCN_KERNEL_RED_COLS;
    p.vec = all_aligned((int64_t)vfull * es, p.nkept - 1, -1) ? vfull : 1;
    const int64_t nc = p.ksize[p.nkept - 1];
    // few columns: a wavefront covers 64 / cpw rows at a time
    const int64_t col_lanes = (nc + p.vec - 1) / p.vec;
    p.cpw = kWave;
    while (p.cpw > 1 && p.cpw / 2 >= col_lanes) p.cpw /= 2;
    const int rpw = kWave / p.cpw;
    const int64_t colblocks = (nc + (int64_t)p.cpw * p.vec - 1) / ((int64_t)p.cpw * p.vec);
    const int64_t others = p.nout / nc;
    const int64_t blocks0 = colblocks * others;
    // Rows are dealt to the wavefronts of a workgroup, which combine through LDS, and to
    // `split` workgroups, which combine through the workspace.  Sixteen wavefronts per
    // workgroup keep the partial results (and the second pass) four times smaller.
    int nw = 4;
    p.split = 1;
    if (blocks0 * nw < kTargetWaves) {
      if (p.nredtot >= 16 * 64 * rpw && blocks0 * 16 * 2 <= kTargetWaves) nw = 16;
      const int64_t want = (kTargetWaves + blocks0 * nw - 1) / (blocks0 * nw);
      const int64_t most = std::max<int64_t>(1, p.nredtot / ((int64_t)nw * rpw * 16));  // >= 16 rows per lane
      p.split = std::max<int64_t>(1, std::min(want, most));
    }
    p.block = nw * kWave;
    p.chunk = (p.nredtot + p.split - 1) / p.split;
    p.split = (p.nredtot + p.chunk - 1) / p.chunk;
    p.grid = blocks0 * p.split;
  } else {
    p.kernel = OCN_KERNEL_RED_GENERIC;
    p.vec = 1;
    p.split = 1;
    p.chunk = p.nredtot;
    p.grid = std::min<int64_t>((p.nout + kBlock - 1) / kBlock, max_launch_blocks());   // the kernel loops beyond that
  }
  if (p.grid > max_launch_blocks()) {
    // more workgroups than one launch may have: the generic kernel, which loops over its outputs
    p.kernel = OCN_KERNEL_RED_GENERIC;
    p.vec = 1;
    p.split = 1;
    p.short_rows = p.lean = false;
    p.block = kBlock;
    p.chunk = p.nredtot;
    p.grid = std::min<int64_t>((p.nout + kBlock - 1) / kBlock, max_launch_blocks());
  }
  p.passes = p.split > 1 ? 2 : 1;
  p.workspace_bytes = p.split > 1 ? (size_t)(p.nout * p.split * acc_es) : 0;
  // an input that cannot stay in the caches anyway is read with streaming loads (whole
  // 16-byte vectors only: neighbouring lanes then cover whole lines)
  p.nt_load = p.vec > 1 && p.kernel != OCN_KERNEL_RED_GENERIC && p.nout * p.nredtot * es >= kStreamBytes;
}

}  // namespace

int plan_reduce(int op, const ocn_tensor *a, const int32_t *axes, int32_t naxes,
                const ocn_tensor *out, RedPlan *plan) {
  RedPlan p;
  p.op = op;
  int rc;
  if ((rc = check_tensor(a)) != OCN_OK) return rc;
  if ((rc = check_tensor(out)) != OCN_OK) return rc;
  if (op < 0 || op >= R_COUNT) return OCN_ERR_OP;
  if (a->device != out->device) return OCN_ERR_DEVICE;
  if (naxes < 0 || naxes > a->ndim) return OCN_ERR_SHAPE;
  if (naxes > 0 && !axes) return OCN_ERR_NULLPTR;
  bool reduced[kMaxDims] = {false};
  for (int i = 0; i < naxes; ++i) {
    if (axes[i] < 0 || axes[i] >= a->ndim || reduced[axes[i]]) return OCN_ERR_SHAPE;
    reduced[axes[i]] = true;
  }
  if (out->ndim != a->ndim - naxes) return OCN_ERR_SHAPE;
  RDim kd[kMaxDims], rd[kMaxDims];
  int nk = 0, nr = 0, j = 0;
  int64_t nout = 1, nred = 1;
  for (int d = 0; d < a->ndim; ++d) {
    if (reduced[d]) {
      nred *= a->size[d];
      rd[nr++] = RDim{a->size[d], a->stride[d], 0};
    } else {
      if (out->size[j] != a->size[d]) return OCN_ERR_SHAPE;
      nout *= a->size[d];
      kd[nk++] = RDim{a->size[d], a->stride[d], out->stride[j]};
      ++j;
    }
  }
  if (!reduce_supported(op, a->dtype)) return OCN_ERR_DTYPE;
  p.nout = nout;
  p.nredtot = nred;
  p.a_dtype = a->dtype;
  p.out_dtype = out->dtype;
  p.acc_dtype = reduce_acc_dtype(op, a->dtype);
  p.swap_a = a->byteswapped && scalar_size(a->dtype) > 1;     // stored in the other byte order (section 3.1.3)
  p.swap_o = out->byteswapped && scalar_size(out->dtype) > 1;
  if (nout == 0) { *plan = p; return OCN_OK; }
  if ((op == R_MIN || op == R_MAX) && nred == 0) return OCN_ERR_EMPTY;
  if (nred > 0 && (rc = check_alignment(a)) != OCN_OK) return rc;
  if ((rc = check_alignment(out)) != OCN_OK) return rc;
  if (!provably_non_overlapping(out)) return OCN_ERR_OVERLAP_OUT;
  if (nred > 0) {
    intptr_t ilo, ihi, olo, ohi;
    byte_range(a, &ilo, &ihi);
    byte_range(out, &olo, &ohi);
    if (ilo < ohi && olo < ihi) return OCN_ERR_ALIAS;
  }

  int64_t off_a = a->offset, off_o = out->offset;
  // kept dims: drop size 1, flip to forward output strides, sort by output stride, merge
  int n = 0;
  for (int d = 0; d < nk; ++d) {
    if (kd[d].size == 1) continue;
    RDim x = kd[d];
    if (x.so < 0) {
      off_o += (x.size - 1) * x.so;
      off_a += (x.size - 1) * x.sa;
      x.so = -x.so; x.sa = -x.sa;
    }
    kd[n++] = x;
  }
  nk = sort_merge(kd, n, true);
  // The column kernel walks the fastest kept dim forward through the input.  If making the
  // output stride positive left the input stride there at minus one element, turn that dim
  // around again: the kernels accept a negative output stride.
  if (nk > 0 && kd[nk - 1].sa == -(int64_t)dt_size(a->dtype)) {
    RDim &x = kd[nk - 1];
    off_o += (x.size - 1) * x.so;
    off_a += (x.size - 1) * x.sa;
    x.so = -x.so;
    x.sa = -x.sa;
  }
  // reduced dims: drop size 1, flip to forward input strides (the set of addends is the
  // same), sort by input stride, merge
  n = 0;
  for (int d = 0; d < nr; ++d) {
    if (rd[d].size == 1) continue;
    RDim x = rd[d];
    if (x.sa < 0) {
      off_a += (x.size - 1) * x.sa;
      x.sa = -x.sa;
    }
    rd[n++] = x;
  }
  nr = nred == 0 ? 0 : sort_merge(rd, n, false);
  p.nkept = nk;
  p.nred = nr;
  for (int d = 0; d < nk; ++d) { p.ksize[d] = kd[d].size; p.kstride_a[d] = kd[d].sa; p.kstride_o[d] = kd[d].so; }
  for (int d = 0; d < nr; ++d) { p.rsize[d] = rd[d].size; p.rstride_a[d] = rd[d].sa; }
  p.off_a = off_a;
  p.off_out = off_o;
  p.a_ptr = (char *)a->base + off_a;
  p.out_ptr = (char *)out->base + off_o;
  choose_reduce_launch(p);
  *plan = p;
  return OCN_OK;
}

namespace {

// Launch shape of a fused elementwise+reduce kernel.  Same three layouts as the plain
// reduction; an input may be broadcast (stride 0) along the vectorised dim as long as the
// other one is contiguous there.
void choose_fused_launch(RedPlan &p) {
  const int es_a = dt_size(p.a_dtype), es_b = dt_size(p.b_dtype), es_m = dt_size(p.mid_dtype);
  const int acc_es = dt_size(p.acc_dtype);
  auto fast_ok = [&](int64_t sa, int64_t sb) {
    return (sa == es_a || sa == 0) && (sb == es_b || sb == 0) && !(sa == 0 && sb == 0);
  };
  // stride in elements along a dim, of the input that moves slower there (0: both broadcast):
  // a dim counts as fast only if no input jumps along it
  auto elems = [&](int64_t sa, int64_t sb) {
    return std::max(iabs64(sa) / es_a, iabs64(sb) / es_b);
  };
  int64_t r_fast = 0, k_fast = 0;
  int k_fast_dim = -1;
  if (p.nred) r_fast = elems(p.rstride_a[p.nred - 1], p.rstride_b[p.nred - 1]);
  for (int d = 0; d < p.nkept; ++d) {
    const int64_t e = elems(p.kstride_a[d], p.kstride_b[d]);
    if (e && (k_fast_dim < 0 || e <= k_fast)) { k_fast = e; k_fast_dim = d; }
  }
  const int vfull = rows_vec(es_m, std::max({es_a, es_b, es_m}));  // as Sig::V with the intermediate type as output
  // every stride except the one along the vectorised dim, and the base, are multiples of the
  // vector size of each input that is not broadcast there
  auto all_aligned = [&](int skip_kept, int skip_red, bool a_bcast, bool b_bcast) {
    const int64_t va = a_bcast ? es_a : (int64_t)vfull * es_a, vb = b_bcast ? es_b : (int64_t)vfull * es_b;
    if ((intptr_t)p.a_ptr % va || (intptr_t)p.b_ptr % vb) return false;
    for (int d = 0; d < p.nkept; ++d)
      if (d != skip_kept && (p.kstride_a[d] % va || p.kstride_b[d] % vb)) return false;
    for (int d = 0; d < p.nred; ++d)
      if (d != skip_red && (p.rstride_a[d] % va || p.rstride_b[d] % vb)) return false;
    return true;
  };
  bool idx32 = p.nout < ((int64_t)1 << 31) && p.nredtot < ((int64_t)1 << 31);
  for (int d = 0; d < p.nkept; ++d) idx32 = idx32 && p.ksize[d] < ((int64_t)1 << 31);
  for (int d = 0; d < p.nred; ++d) idx32 = idx32 && p.rsize[d] < ((int64_t)1 << 31);
  const bool flat_full = p.nkept == 0 && p.nred == 1;

  p.split = 1;
  if (p.nred >= 1 && fast_ok(p.rstride_a[p.nred - 1], p.rstride_b[p.nred - 1]) &&
      (k_fast_dim < 0 || k_fast > r_fast) && (idx32 || flat_full)) {
    p.kernel = OCN_KERNEL_RED_ROWS;
    p.a_fast_bcast = p.rstride_a[p.nred - 1] == 0;
    p.b_fast_bcast = p.rstride_b[p.nred - 1] == 0;
    p.vec = all_aligned(-1, p.nred - 1, p.a_fast_bcast, p.b_fast_bcast) ? vfull : 1;
    const int64_t n0 = p.rsize[p.nred - 1];
    const int64_t vpr = (n0 + p.vec - 1) / p.vec;
    const int64_t nvec = vpr * (p.nredtot / n0);
    int64_t cover = 1;                                    // lanes one output can keep busy
    while (cover < nvec && cover < kWave) cover <<= 1;
    p.group = (nvec * p.vec * (es_a + es_b) <= 16 * 1024) ? (int)cover : kBlock;
    const int64_t groups_per_block = kBlock / p.group;
    const int64_t waves = (p.nout * p.group + kWave - 1) / kWave;
    if (p.group >= kWave && waves < kTargetWaves) {
      const int64_t want = (kTargetWaves + waves - 1) / waves;
      const int64_t most = std::max<int64_t>(1, nvec / ((int64_t)p.group * 8));
      p.split = std::max<int64_t>(1, std::min(want, most));
    }
    p.chunk = (nvec + p.split - 1) / p.split;
    p.split = (nvec + p.chunk - 1) / p.chunk;
    p.grid = (p.nout * p.split + groups_per_block - 1) / groups_per_block;
    p.short_rows = p.group <= kWave && nvec <= p.group && p.nred == 1 && p.split == 1 &&
                   p.nout * p.group < ((int64_t)1 << 32) && n0 < ((int64_t)1 << 31);
    // The common 2-D shape takes the lean form of the kernel: one reduced dim along which both
    // inputs are contiguous and made of whole, aligned 16-byte vectors, at most one kept dim,
    // at least a wavefront per output, everything below 2^31.  Its vectors are 16 bytes of
    // each input whatever the intermediate type is.
    const int lv = es_a == es_b && es_a <= 16 ? 16 / es_a : 0;   // elements per vector
    if (!p.short_rows && lv >= 1 && p.nred == 1 && p.nkept <= 1 && !p.a_fast_bcast && !p.b_fast_bcast &&
        n0 % lv == 0 && n0 / lv >= kWave && n0 / lv < ((int64_t)1 << 31) && p.nout < ((int64_t)1 << 31) &&
        (intptr_t)p.a_ptr % 16 == 0 && (intptr_t)p.b_ptr % 16 == 0 &&
        (p.nkept == 0 || (p.kstride_a[0] % 16 == 0 && p.kstride_b[0] % 16 == 0))) {
      const int64_t nv = n0 / lv;
      const int group = nv * 32 <= 16 * 1024 ? kWave : kBlock;    // as above: rows of up to 16 KiB take a wavefront
      const int64_t lwaves = (p.nout * group + kWave - 1) / kWave;
      int64_t split = 1;
      if (lwaves < kTargetWaves) {
        const int64_t want = (kLeanSplitWaves + lwaves - 1) / lwaves;
        const int64_t most = std::max<int64_t>(1, nv / ((int64_t)group * 8));
        split = std::max<int64_t>(1, std::min(want, most));
      }
      const int64_t chunk = (nv + split - 1) / split;
      split = (nv + chunk - 1) / chunk;
      if (p.nout * split < ((int64_t)1 << 31)) {
        p.lean = true;
        p.vec = lv;
        p.group = group;
        p.split = split;
        p.chunk = chunk;
        p.grid = (p.nout * split + kBlock / group - 1) / (kBlock / group);
        // inputs far larger than the caches are streamed; one that is broadcast along the kept
        // dim is re-read by every output and stays cacheable, and then so does the other (one flag)
        const bool a_rows = p.nkept == 0 || p.kstride_a[0] != 0, b_rows = p.nkept == 0 || p.kstride_b[0] != 0;
        p.nt_load = a_rows && b_rows && p.nout * n0 * es_a >= kStreamBytes;
      }
    }
  } else if (k_fast_dim >= 0 && k_fast_dim == p.nkept - 1 && p.nred >= 1 && idx32 &&
             fast_ok(p.kstride_a[k_fast_dim], p.kstride_b[k_fast_dim]) && (r_fast == 0 || r_fast > k_fast)) {
    p.kernel = OCN_KERNEL_RED_COLS;
    p.a_fast_bcast = p.kstride_a[k_fast_dim] == 0;
    p.b_fast_bcast = p.kstride_b[k_fast_dim] == 0;
    p.vec = all_aligned(p.nkept - 1, -1, p.a_fast_bcast, p.b_fast_bcast) ? vfull : 1;
    const int64_t nc = p.ksize[p.nkept - 1];
    // few columns: a wavefront covers 64 / cpw rows at a time
    const int64_t col_lanes = (nc + p.vec - 1) / p.vec;
    p.cpw = kWave;
    while (p.cpw > 1 && p.cpw / 2 >= col_lanes) p.cpw /= 2;
    const int rpw = kWave / p.cpw;
    const int64_t colblocks = (nc + (int64_t)p.cpw * p.vec - 1) / ((int64_t)p.cpw * p.vec);
    const int64_t blocks0 = colblocks * (p.nout / nc);
    int nw = 4;   // as in the plain column reduction: sixteen wavefronts keep the partial results small
    if (blocks0 * nw < kTargetWaves) {
      if (p.nredtot >= 16 * 64 * rpw && blocks0 * 16 * 2 <= kTargetWaves) nw = 16;
      const int64_t want = (kTargetWaves + blocks0 * nw - 1) / (blocks0 * nw);
      const int64_t most = std::max<int64_t>(1, p.nredtot / ((int64_t)nw * rpw * 16));
      p.split = std::max<int64_t>(1, std::min(want, most));
    }
    p.block = nw * kWave;
    // inputs far larger than the caches, each read as one 16-byte piece per lane and broadcast
    // along no dim: streaming loads
    {
      bool plain = p.vec > 1 && (int64_t)p.vec * es_a == 16 && (int64_t)p.vec * es_b == 16;
      for (int d = 0; d < p.nkept; ++d) plain = plain && p.kstride_a[d] != 0 && p.kstride_b[d] != 0;
      for (int d = 0; d < p.nred; ++d) plain = plain && p.rstride_a[d] != 0 && p.rstride_b[d] != 0;
      p.nt_load = plain && p.nout * p.nredtot * es_a >= kStreamBytes;
    }
    p.chunk = (p.nredtot + p.split - 1) / p.split;
    p.split = (p.nredtot + p.chunk - 1) / p.chunk;
    p.grid = blocks0 * p.split;
  } else {
    p.kernel = OCN_KERNEL_RED_GENERIC;
    p.vec = 1;
    p.chunk = p.nredtot;
    p.grid = std::min<int64_t>((p.nout + kBlock - 1) / kBlock, max_launch_blocks());
  }
  p.passes = p.split > 1 ? 2 : 1;
  p.workspace_bytes = p.split > 1 ? (size_t)(p.nout * p.split * acc_es) : 0;
}

}  // namespace

int plan_binary_reduce(int ew_op, int red_op, const ocn_tensor *a, const ocn_tensor *b,
                       const int32_t *axes, int32_t naxes, const ocn_tensor *out, int mid_dtype,
                       char *workspace, FusedPlan *plan) {
  FusedPlan fp;
  RedPlan &p = fp.red;
  int rc;
  if ((rc = check_tensor(a)) != OCN_OK) return rc;
  if ((rc = check_tensor(b)) != OCN_OK) return rc;
  if ((rc = check_tensor(out)) != OCN_OK) return rc;
  if (ew_op < 0 || ew_op >= B_COUNT || red_op < 0 || red_op >= R_COUNT) return OCN_ERR_OP;
  if (!valid_dtype(mid_dtype)) return OCN_ERR_DTYPE;
  if (a->device != out->device || b->device != out->device) return OCN_ERR_DEVICE;
  // the fused kernels take operands in native byte order only (one-byte scalars have no order):
  // with an operand in the other order the call runs as the two calls it abbreviates, whose
  // kernels reverse on load and on store
  bool other_order = false;
  for (const ocn_tensor *t : {a, b, out})
    if (t->byteswapped && scalar_size(t->dtype) > 1) other_order = true;
  // broadcast shape of the two inputs (missing leading dims count as size 1)
  const int nd = std::max(a->ndim, b->ndim);
  int64_t shape[kMaxDims], sa[kMaxDims], sb[kMaxDims];
  for (int d = 0; d < nd; ++d) {
    const int da = d - (nd - a->ndim), db = d - (nd - b->ndim);
    const int64_t na = da >= 0 ? a->size[da] : 1, nb = db >= 0 ? b->size[db] : 1;
    if (na != nb && na != 1 && nb != 1) return OCN_ERR_SHAPE;
    shape[d] = na == 1 ? nb : na;
    sa[d] = (da >= 0 && na != 1) ? a->stride[da] : 0;
    sb[d] = (db >= 0 && nb != 1) ? b->stride[db] : 0;
  }
  if (naxes < 0 || naxes > nd) return OCN_ERR_SHAPE;
  if (naxes > 0 && !axes) return OCN_ERR_NULLPTR;
  bool reduced[kMaxDims] = {false};
  for (int i = 0; i < naxes; ++i) {
    if (axes[i] < 0 || axes[i] >= nd || reduced[axes[i]]) return OCN_ERR_SHAPE;
    reduced[axes[i]] = true;
  }
  if (out->ndim != nd - naxes) return OCN_ERR_SHAPE;
  const int promoted = promote(a->dtype, b->dtype);
  const int T = binary_compute_dtype(ew_op, a->dtype, b->dtype, mid_dtype, promoted, promote(promoted, mid_dtype));
  if (!binary_supported(ew_op, T) || !reduce_supported(red_op, mid_dtype)) return OCN_ERR_DTYPE;

  RDim kd[kMaxDims], rd[kMaxDims];
  int nk = 0, nr = 0, j = 0;
  int64_t nout = 1, nred = 1;
  for (int d = 0; d < nd; ++d) {
    if (reduced[d]) {
      nred *= shape[d];
      rd[nr++] = RDim{shape[d], sa[d], 0, sb[d]};
    } else {
      if (out->size[j] != shape[d]) return OCN_ERR_SHAPE;
      nout *= shape[d];
      kd[nk++] = RDim{shape[d], sa[d], out->stride[j], sb[d]};
      ++j;
    }
  }
  p.op = red_op;
  p.fused = true;
  p.ew_op = ew_op;
  p.nout = nout;
  p.nredtot = nred;
  p.a_dtype = a->dtype;
  p.b_dtype = b->dtype;
  p.mid_dtype = mid_dtype;
  p.out_dtype = out->dtype;
  p.acc_dtype = reduce_acc_dtype(red_op, mid_dtype);
  if (nout == 0) { *plan = fp; return OCN_OK; }
  if ((red_op == R_MIN || red_op == R_MAX) && nred == 0) return OCN_ERR_EMPTY;
  if ((rc = check_alignment(a)) != OCN_OK) return rc;
  if ((rc = check_alignment(b)) != OCN_OK) return rc;
  if ((rc = check_alignment(out)) != OCN_OK) return rc;
  if (!provably_non_overlapping(out)) return OCN_ERR_OVERLAP_OUT;
  if (nred > 0) {
    intptr_t olo, ohi, ilo, ihi;
    byte_range(out, &olo, &ohi);
    byte_range(a, &ilo, &ihi);
    if (ilo < ohi && olo < ihi) return OCN_ERR_ALIAS;
    byte_range(b, &ilo, &ihi);
    if (ilo < ohi && olo < ihi) return OCN_ERR_ALIAS;
  }

  // elementwise into a temporary, then reduce it
  auto plan_unfused = [&]() -> int {
    fp.unfused = true;
    ocn_tensor &m = fp.mid;
    m.base = workspace;
    m.offset = 0;
    m.dtype = mid_dtype;
    m.ndim = nd;
    m.device = out->device;
    int64_t acc = dt_size(mid_dtype);
    for (int d = nd - 1; d >= 0; --d) { m.size[d] = shape[d]; m.stride[d] = acc; acc *= shape[d]; }
    fp.mid_bytes = ((size_t)acc + 255) / 256 * 256;
    // planned against a stand-in address when the caller only wants sizes
    if (!workspace) m.base = (void *)(uintptr_t)0x1000;
    int rc2;
    if ((rc2 = plan_elementwise(2, ew_op, a, b, &m, 0, &fp.ew)) != OCN_OK) return rc2;
    if ((rc2 = plan_reduce(red_op, &m, axes, naxes, out, &fp.red)) != OCN_OK) return rc2;
    fp.workspace_bytes = fp.mid_bytes + fp.red.workspace_bytes;
    *plan = fp;
    return OCN_OK;
  };
  // no fused kernel for these types
  if (other_order || !fused_specialised(ew_op, a->dtype, b->dtype, mid_dtype, red_op) || nred == 0) return plan_unfused();

  const int es_a = dt_size(a->dtype), es_b = dt_size(b->dtype);
  int64_t off_a = a->offset, off_b = b->offset, off_o = out->offset;
  // kept dims: drop size 1, flip to forward output strides, sort by output stride, merge
  int n = 0;
  for (int d = 0; d < nk; ++d) {
    if (kd[d].size == 1) continue;
    RDim x = kd[d];
    if (x.so < 0) {
      off_o += (x.size - 1) * x.so; off_a += (x.size - 1) * x.sa; off_b += (x.size - 1) * x.sb;
      x.so = -x.so; x.sa = -x.sa; x.sb = -x.sb;
    }
    kd[n++] = x;
  }
  nk = sort_merge(kd, n, true);
  // the column kernel walks the fastest kept dim forward through the inputs: turn it around
  // again if the flip above left both inputs walking backwards (or broadcast) there
  if (nk > 0) {
    RDim &x = kd[nk - 1];
    const bool a_back = x.sa == -(int64_t)es_a, b_back = x.sb == -(int64_t)es_b;
    if ((a_back && (b_back || x.sb == 0)) || (b_back && x.sa == 0)) {
      off_o += (x.size - 1) * x.so; off_a += (x.size - 1) * x.sa; off_b += (x.size - 1) * x.sb;
      x.so = -x.so; x.sa = -x.sa; x.sb = -x.sb;
    }
  }
  // reduced dims: drop size 1, flip so the faster-moving input walks forward, sort, merge
  n = 0;
  for (int d = 0; d < nr; ++d) {
    if (rd[d].size == 1) continue;
    RDim x = rd[d];
    const int64_t lead = x.sa != 0 ? x.sa : x.sb;
    if (lead < 0) {
      off_a += (x.size - 1) * x.sa; off_b += (x.size - 1) * x.sb;
      x.sa = -x.sa; x.sb = -x.sb;
    }
    rd[n++] = x;
  }
  nr = sort_merge_by(rd, n, [&](const RDim &x) { return std::max(iabs64(x.sa) / es_a, iabs64(x.sb) / es_b); });
  p.nkept = nk;
  p.nred = nr;
  for (int d = 0; d < nk; ++d) {
    p.ksize[d] = kd[d].size; p.kstride_a[d] = kd[d].sa; p.kstride_b[d] = kd[d].sb; p.kstride_o[d] = kd[d].so;
  }
  for (int d = 0; d < nr; ++d) { p.rsize[d] = rd[d].size; p.rstride_a[d] = rd[d].sa; p.rstride_b[d] = rd[d].sb; }
  p.off_a = off_a; p.off_b = off_b; p.off_out = off_o;
  p.a_ptr = (char *)a->base + off_a;
  p.b_ptr = (char *)b->base + off_b;
  p.out_ptr = (char *)out->base + off_o;
  choose_fused_launch(p);
  // The fused kernels cover the two layouts with a contiguous axis.  Anything else would fold
  // each output in a single lane: for long reductions the two-launch route, whose kernels
  // spread every layout over the device, is faster despite the temporary.
  if (p.kernel == OCN_KERNEL_RED_GENERIC && p.nredtot >= 1024) return plan_unfused();
  // more workgroups than one launch may have: the two calls, whose kernels loop
  if (p.grid > max_launch_blocks()) return plan_unfused();
  fp.workspace_bytes = p.workspace_bytes;
  *plan = fp;
  return OCN_OK;
}

void plan_second_pass(const RedPlan &first, char *workspace, RedPlan *second) {
  RedPlan q;
  q.op = first.op;  // every supported reduction folds its own partial results
  q.a_dtype = first.acc_dtype;
  q.out_dtype = first.out_dtype;
  q.acc_dtype = reduce_acc_dtype(q.op, q.a_dtype);
  q.nout = first.nout;
  q.nredtot = first.split;
  q.a_ptr = workspace;
  q.out_ptr = first.out_ptr;
  q.off_a = 0;
  q.off_out = first.off_out;
  const int64_t es = dt_size(q.a_dtype);
  q.nkept = first.nkept;
  const bool rows_layout = first.kernel == OCN_KERNEL_RED_ROWS;  // [nout][split], else [split][nout]
  int64_t lin = rows_layout ? first.split * es : es;
  for (int d = first.nkept - 1; d >= 0; --d) {
    q.ksize[d] = first.ksize[d];
    q.kstride_o[d] = first.kstride_o[d];
    q.kstride_a[d] = lin;
    lin *= first.ksize[d];
  }
  q.nred = 1;
  q.rsize[0] = first.split;
  q.rstride_a[0] = rows_layout ? es : first.nout * es;
  q.split = 1;
  q.swap_o = first.swap_o;   // the partial results are in native order, the output as the caller declared it
  q.chunk = first.split;
  q.passes = 1;
  q.workspace_bytes = 0;
  q.vec = 1;
  if (rows_layout) {
    q.kernel = OCN_KERNEL_RED_ROWS;
    q.group = 1;                       // lanes per output: the partials of one output are adjacent
    while (q.group < first.split && q.group < kWave) q.group <<= 1;
    if (first.split >= 4 * kBlock) q.group = kBlock;   // as in the first pass: four partials per lane and more
    q.chunk = first.split;  // vectors (vec = 1) per output
    q.grid = (q.nout * q.group + kBlock - 1) / kBlock;
    // Eight-byte partial results in whole, aligned 16-byte vectors, at most one kept dim: the
    // lean form of the kernel, whose few arguments arrive with the first scalar loads (this
    // launch is nothing but a chain of latencies)
    const int64_t nv = first.split / 2;
    if (es == 8 && first.split % 2 == 0 && nv >= kWave && nv < ((int64_t)1 << 31) && first.nkept <= 1 &&
        q.nout < ((int64_t)1 << 31) && (intptr_t)workspace % 16 == 0) {
      q.lean = true;
      q.vec = 2;
      q.chunk = nv;
      q.group = nv < 4 * kBlock ? kWave : kBlock;
      q.grid = (q.nout + kBlock / q.group - 1) / (kBlock / q.group);
    }
  } else if (!rows_layout && first.nkept >= 1 && q.nout < ((int64_t)1 << 31)) {
    q.kernel = OCN_KERNEL_RED_COLS;
    const int64_t nc = q.ksize[q.nkept - 1];
    while (q.cpw > 1 && q.cpw / 2 >= nc) q.cpw /= 2;
    const int64_t colblocks = (nc + q.cpw - 1) / q.cpw;
    q.grid = colblocks * (q.nout / nc);
    if (first.split >= 64) q.block = 16 * kWave;   // many partials per column: more wavefronts share them
    // eight-byte partial results of a single kept dim: the kernel made for this launch
    if (es == 8 && first.nkept == 1 && first.split < ((int64_t)1 << 31) && max_launch_blocks() >= (q.nout + kWave - 1) / kWave) {
      q.fold = true;
      q.block = kWave;
      q.grid = (q.nout + kWave - 1) / kWave;
    }
  } else {
    q.kernel = OCN_KERNEL_RED_GENERIC;
    q.grid = std::min<int64_t>((q.nout + kBlock - 1) / kBlock, max_launch_blocks());
  }
  *second = q;
}

// ---------------------------------------------------------------------------------------
// plan inspection
// ---------------------------------------------------------------------------------------

void fill_info(const EwPlan &p, ocn_plan_info *info) {
  std::memset(info, 0, sizeof *info);
  info->kernel = p.kernel;
  info->compute_dtype = p.T;
  info->ndim = p.ndim;
  for (int d = 0; d < p.ndim; ++d) {
    info->size[d] = p.size[d];
    info->stride_out[d] = p.out.stride[d];
    info->stride_a[d] = p.a.stride[d];
    info->stride_b[d] = p.b.stride[d];
    info->tile_log2[d] = p.tile_log2[d];
  }
  info->offset_out = p.off_out;
  info->offset_a = p.off_a;
  info->offset_b = p.off_b;
  info->vec = p.vec;
  info->stage_a = p.stage_a;
  info->stage_b = p.stage_b;
  info->specialised = p.specialised;
  info->passes = p.kernel == OCN_KERNEL_NONE ? 0 : 1;
  info->grid = p.grid;
  info->block = kBlock;
  info->split = 1;
  info->lds_bytes = p.lds_bytes;
  info->unclipped = p.fast_tiled ? 1 : 0;
  info->tile_group = p.fast_tiled && p.pair_dim >= 0 ? (int64_t)1 << p.pair_log2 : 1;
}

void fill_info(const RedPlan &p, ocn_plan_info *info) {
  std::memset(info, 0, sizeof *info);
  info->kernel = p.kernel;
  info->compute_dtype = p.acc_dtype;
  info->ndim = p.nkept;
  info->nred = p.nred;
  for (int d = 0; d < p.nkept; ++d) {
    info->size[d] = p.ksize[d];
    info->stride_out[d] = p.kstride_o[d];
    info->stride_a[d] = p.kstride_a[d];
  }
  for (int d = 0; d < p.nred; ++d) {
    info->red_size[d] = p.rsize[d];
    info->red_stride_a[d] = p.rstride_a[d];
  }
  info->offset_out = p.off_out;
  info->offset_a = p.off_a;
  info->vec = p.vec;
  info->specialised = 1;
  info->passes = p.kernel == OCN_KERNEL_NONE ? 0 : p.passes;
  info->grid = p.grid;
  info->block = p.block;
  info->split = p.split;
}

}  // namespace ocn
