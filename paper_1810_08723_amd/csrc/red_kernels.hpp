// Reduction kernels of the tensor engine for gfx950 (section 3.2 of the paper: tensor
// reductions along one or more axes).
//
//   red_rows_kernel     lanes share an output: a power-of-two group of 1 to 64 lanes (short
//                       rows: a wavefront then covers several outputs) or a whole workgroup
//                       (long rows) streams one output's addends, with 128-bit loads when the
//                       reduced axis is the input's fastest; lanes fold privately, then a
//                       shuffle tree and an LDS step combine them.  Long reductions with few outputs are split over
//                       several workgroups; each writes a partial result to the workspace and a
//                       second launch folds the partials (two-pass grid reduction).
//   red_rows_short_kernel  the same for rows of at most one vector per lane, without loops
//   red_cols_kernel     a kept axis is the input's fastest: lanes own adjacent output columns
//                       (with few columns a wavefront covers several rows at a time), the
//                       wavefronts of a workgroup take interleaved rows and are combined
//                       through LDS; row ranges can be split the same way.
//   red_generic_kernel  any layout and 64-bit extents: one output per lane, sequential fold.
// No floating-point atomics anywhere: the grouping of addends is fixed by the launch
// geometry, so results are reproducible bit for bit.
#pragma once

#include <type_traits>

#include "dev_types.hpp"
#include "planner.hpp"

namespace ocn {

struct RedArgs {
  const char *a;
  char *out;                        // final output (used when split == 1)
  char *partial;                    // workspace (used when split > 1)
  int32_t nkept, nred, out_dtype, vec, group;
  int64_t ksa[kMaxDims], kso[kMaxDims];    // kept dims: input / output byte strides, fastest first
  FastDiv kdiv[kMaxDims];                  // kept sizes, same order
  int64_t rsa[kMaxDims];                   // reduced dims: input byte strides, fastest first
  FastDiv rdiv[kMaxDims];                  // reduced sizes, same order
  int64_t ksize[kMaxDims], rsize[kMaxDims];// the same sizes in 64 bits (generic kernel)
  int64_t nout, nredtot;
  int64_t n0;                              // length of the fastest reduced dim (rows)
  FastDiv vpr_div;                         // rows: vectors per innermost run
  int64_t nvec;                            // rows: vectors per output
  int64_t split, chunk;
  int64_t nc;                              // cols: number of columns (fastest kept dim)
  FastDiv colblocks_div;                   // cols: column blocks per row of outputs
  // second input of a fused elementwise+reduce kernel (unused by the plain kernels)
  const char *b;
  int64_t ksb[kMaxDims], rsb[kMaxDims];    // its byte strides, same order as ksa / rsa
  int32_t a_bcast, b_bcast;                // broadcast along the vectorised dim
  int32_t cpw;                             // cols: lanes per row of columns (power of two <= 64)
  int32_t nt_load;                         // vector loads carry the streaming (non-temporal) hint
  int32_t swap_a, swap_o;                  // the input / the output is stored in the other byte order
};

// arguments of the kernel that folds [split][output] partial results
struct RedFoldArgs {
  const char *partial;
  char *out;
  int64_t kso;             // byte stride of the (one) kept dim in the output
  uint32_t nout, split;
  int32_t out_dtype, swap_o;
};

// arguments of the lean rows kernel: one reduced dim read in whole 16-byte vectors, at most one
// kept dim, everything below 2^31
struct RedLeanArgs {
  const char *a;
  const char *b;           // second input of a fused elementwise+reduce call
  char *out, *partial;
  int64_t ksa, kso;        // byte strides of the kept dim in the input and the output
  int64_t ksb;             // ... in the second input
  uint32_t nout, split;    // outputs; partial results per output
  uint32_t nvec, chunk;    // vectors per output; vectors per split
  int32_t out_dtype, group, nt_load;
  int32_t swap_a, swap_o;  // the input / the output is stored in the other byte order
};

#if defined(__HIPCC__)

OCN_DEV uint32_t rfastdiv(uint32_t n, const FastDiv &f) { return (__umulhi(n, f.m) + n) >> f.s; }

// ---------------------------------------------------------------------------------------
// accumulators
// ---------------------------------------------------------------------------------------

constexpr int red_acc_dtype(int op, int dt) {
  const int k = dt_kind(dt);
  if (op == R_SUM || op == R_PROD) {
    if (k == K_BOOL || k == K_SINT) return DT_I64;
    if (k == K_UINT) return DT_U64;
    if (dt == DT_F16) return DT_F32;
    if (dt == DT_F32 || dt == DT_F64) return DT_F64;
    return dt == DT_C16 ? DT_C32 : DT_C64;
  }
  if (op == R_MIN || op == R_MAX) return dt;
  return DT_BOOL;
}
constexpr bool red_supported(int op, int dt) {
  return op == R_SUM || op == R_ANY || op == R_ALL || dt_kind(dt) != K_CPLX;
}

template <int S, int OP> struct Reducer {
  static constexpr int ACC = red_acc_dtype(OP, S);
  using A = reg_t<ACC>;     // accumulator register type
  using P = storage_t<ACC>; // how a partial result is stored

  OCN_DEV static A identity() {
    constexpr int k = dt_kind(ACC);
    if constexpr (OP == R_SUM) {
      if constexpr (k == K_CPLX) return A{0, 0};
      else return (A)0;
    } else if constexpr (OP == R_PROD) {
      return (A)1;
    } else if constexpr (OP == R_ANY) {
      return false;
    } else if constexpr (OP == R_ALL) {
      return true;
    } else {  // min / max start from the far end of the type's range
      constexpr bool mx = OP == R_MAX;
      if constexpr (k == K_BOOL) return !mx;
      else if constexpr (ACC == DT_F16) return hreg{mx ? -__builtin_inff() : __builtin_inff()};
      else if constexpr (ACC == DT_F32) return mx ? -__builtin_inff() : __builtin_inff();
      else if constexpr (ACC == DT_F64) return mx ? -__builtin_inf() : __builtin_inf();
      else return mx ? std::numeric_limits<A>::min() : std::numeric_limits<A>::max();
    }
  }

  OCN_DEV static A lift(reg_t<S> x) {
    if constexpr (OP == R_SUM || OP == R_PROD) return convert<ACC>(x);  // exact widening
    else if constexpr (OP == R_MIN || OP == R_MAX) return x;
    else return convert<DT_BOOL>(x);
  }

  OCN_DEV static A combine(A x, A y) {
    constexpr int k = dt_kind(ACC);
    if constexpr (OP == R_SUM) {
      if constexpr (k == K_CPLX) return A{x.re + y.re, x.im + y.im};
      else if constexpr (k == K_SINT) return (A)((uint64_t)x + (uint64_t)y);
      else return x + y;
    } else if constexpr (OP == R_PROD) {
      if constexpr (k == K_SINT) return (A)((uint64_t)x * (uint64_t)y);
      else return x * y;
    } else if constexpr (OP == R_ANY) {
      return x || y;
    } else if constexpr (OP == R_ALL) {
      return x && y;
    } else {
      constexpr bool mx = OP == R_MAX;
      if constexpr (k == K_BOOL) return mx ? (x || y) : (x && y);
      else if constexpr (ACC == DT_F16) return hreg{mx ? nan_max(x.v, y.v) : nan_min(x.v, y.v)};
      else if constexpr (k == K_REAL) return mx ? nan_max(x, y) : nan_min(x, y);
      else return mx ? (x > y ? x : y) : (x < y ? x : y);
    }
  }
};

// ---------------------------------------------------------------------------------------
// cross-lane movement of an accumulator of any size (32-bit pieces through the shuffle unit)
// ---------------------------------------------------------------------------------------

template <class A> OCN_DEV A shfl_down_any(A v, int delta) {
  constexpr int W = (sizeof(A) + 3) / 4;
  union { A a; uint32_t w[W]; } u, r;
#pragma unroll
  for (int i = 0; i < W; ++i) u.w[i] = 0;
  u.a = v;
#pragma unroll
  for (int i = 0; i < W; ++i) r.w[i] = (uint32_t)__shfl_down((int)u.w[i], delta, kWave);
  return r.a;
}

// after this, lane 0 of the wavefront holds the fold of all 64 lanes
template <class R> OCN_DEV typename R::A wave_fold(typename R::A v) {
#pragma unroll
  for (int d = kWave / 2; d >= 1; d >>= 1) v = R::combine(v, shfl_down_any(v, d));
  return v;
}

// lane i receives lane i + N of its row of 16 lanes (data-parallel primitive "row shift left";
// lanes past the end of the row read zero)
template <int N, class A> OCN_DEV A row_down_any(A v) {
  constexpr int W = (sizeof(A) + 3) / 4;
  union { A a; uint32_t w[W]; } u, r;
#pragma unroll
  for (int i = 0; i < W; ++i) u.w[i] = 0;
  u.a = v;
#pragma unroll
  for (int i = 0; i < W; ++i) r.w[i] = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)u.w[i], 0x100 + N, 0xf, 0xf, true);
  return r.a;
}

// the same over aligned groups of `width` lanes (a power of two, the same for the whole
// wavefront): the first lane of every group ends up with its group's fold.  Steps that stay
// inside a row of 16 lanes use the row shift, which costs one instruction per 32-bit word.
template <class R> OCN_DEV typename R::A group_fold(typename R::A v, int width) {
  if (width > 32) v = R::combine(v, shfl_down_any(v, 32));
  if (width > 16) v = R::combine(v, shfl_down_any(v, 16));
  if (width > 8) v = R::combine(v, row_down_any<8>(v));
  if (width > 4) v = R::combine(v, row_down_any<4>(v));
  if (width > 2) v = R::combine(v, row_down_any<2>(v));
  if (width > 1) v = R::combine(v, row_down_any<1>(v));
  return v;
}

// convert an accumulator to the runtime output dtype and store it (once per output)
template <class A> __device__ __noinline__ void store_result(char *p, int dt, A r, bool swapped = false) {
  switch (dt) {
#define OCN_CASE(D)                                      \
  case D: {                                              \
    storage_t<D> s = to_storage<D>(convert<D>(r));       \
    if (swapped) reverse_scalars<scalar_bytes(D)>(s);    \
    *reinterpret_cast<storage_t<D> *>(p) = s;            \
  } break;
    OCN_CASE(DT_BOOL) OCN_CASE(DT_I8) OCN_CASE(DT_I16) OCN_CASE(DT_I32) OCN_CASE(DT_I64)
    OCN_CASE(DT_U8) OCN_CASE(DT_U16) OCN_CASE(DT_U32) OCN_CASE(DT_U64)
    OCN_CASE(DT_F16) OCN_CASE(DT_F32) OCN_CASE(DT_F64)
    OCN_CASE(DT_C16) OCN_CASE(DT_C32) OCN_CASE(DT_C64)
#undef OCN_CASE
    default: break;
  }
}

// byte offsets of output number `o` (linear over the kept dims) in the input and the output
OCN_DEV void kept_offsets(const RedArgs &p, uint32_t o, int64_t &off_a, int64_t &off_o) {
  off_a = 0;
  off_o = 0;
#pragma unroll
  for (int k = 0; k < kMaxDims; ++k) {
    if (k < p.nkept) {
      const uint32_t q = (k == p.nkept - 1) ? 0u : rfastdiv(o, p.kdiv[k]);
      const uint32_t i = o - q * p.kdiv[k].d;
      o = q;
      off_a += (int64_t)i * p.ksa[k];
      off_o += (int64_t)i * p.kso[k];
    }
  }
}

// input byte offset of reduced index q over the reduced dims from `first` upward
OCN_DEV int64_t reduced_offset(const RedArgs &p, uint32_t q, int first) {
  int64_t off = 0;
#pragma unroll
  for (int k = 0; k < kMaxDims; ++k) {
    if (k >= first && k < p.nred) {
      const uint32_t qq = (k == p.nred - 1) ? 0u : rfastdiv(q, p.rdiv[k]);
      const uint32_t i = q - qq * p.rdiv[k].d;
      q = qq;
      off += (int64_t)i * p.rsa[k];
    }
  }
  return off;
}

// ---------------------------------------------------------------------------------------
// rows
// ---------------------------------------------------------------------------------------

// A lane's running fold over whole vectors of V consecutive elements.  The generic form
// folds element by element; two specialisations use packed instructions:
//   * sums of 8-bit integers add four bytes per instruction (dot product with ones) into a
//     32-bit register that is flushed into the 64-bit total long before it can overflow;
//   * min/max of half-precision values compares order-preserving 16-bit integer keys two at
//     a time and tracks NaNs on the side, which keeps the NaN-propagating, +0-above--0
//     semantics exact without any floating-point comparison.
template <int S, int OP, int V, class Enable = void> struct VecFold {
  using R = Reducer<S, OP>;
  using A = typename R::A;
  using St = storage_t<S>;
  struct alignas(sizeof(St) * V >= 16 ? 16 : sizeof(St) * V) Pk { St v[V]; };
  A acc;
  OCN_DEV void init() { acc = R::identity(); }
  OCN_DEV void add_full(const Pk &pk) {
#pragma unroll
    for (int i = 0; i < V; ++i) acc = R::combine(acc, R::lift(from_storage<S>(pk.v[i])));
  }
  OCN_DEV void add_partial(const Pk &pk, int n) {
#pragma unroll
    for (int i = 0; i < V; ++i)
      if (i < n) acc = R::combine(acc, R::lift(from_storage<S>(pk.v[i])));
  }
  OCN_DEV A result() { return acc; }
};

// sum of int8 / uint8, sixteen per vector
template <int S, int V>
struct VecFold<S, R_SUM, V, std::enable_if_t<(S == DT_I8 || S == DT_U8) && V == 16>> {
  using R = Reducer<S, R_SUM>;
  using A = typename R::A;  // int64_t or uint64_t
  using St = storage_t<S>;
  struct alignas(16) Pk { St v[V]; };
  A total;
  int32_t part;      // at most 2^11 per add_full in magnitude
  uint32_t pending;  // add_full calls since the last flush
  OCN_DEV void init() { total = 0; part = 0; pending = 0; }
  OCN_DEV void flush() {
    if constexpr (S == DT_I8) total += (A)part;
    else total += (A)(uint32_t)part;
    part = 0;
    pending = 0;
  }
  OCN_DEV void add_full(const Pk &pk) {
    const int32_t *w = reinterpret_cast<const int32_t *>(&pk);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if constexpr (S == DT_I8) part = __builtin_amdgcn_sdot4(w[k], 0x01010101, part, false);
      else part = (int32_t)__builtin_amdgcn_udot4((uint32_t)w[k], 0x01010101u, (uint32_t)part, false);
    }
    if (++pending == (1u << 19)) flush();  // 2^19 * 2^11 < 2^31 (uint8: 2^19 * 4080 < 2^32)
  }
  OCN_DEV void add_partial(const Pk &pk, int n) {
#pragma unroll
    for (int i = 0; i < V; ++i)
      if (i < n) total += (A)pk.v[i];
  }
  OCN_DEV A result() { flush(); return total; }
};

// min / max of half precision, eight per vector: the packed IEEE 754-2019 maximum / minimum of
// gfx950 (NaN-propagating, +0 above -0) folds two elements per instruction
template <int OP, int V>
struct VecFold<DT_F16, OP, V, std::enable_if_t<(OP == R_MIN || OP == R_MAX) && V == 8>> {
  using R = Reducer<DT_F16, OP>;
  using A = typename R::A;  // hreg
  using St = storage_t<DT_F16>;
  struct alignas(16) Pk { St v[V]; };
  using h2 = _Float16 __attribute__((ext_vector_type(2)));
  static constexpr bool MX = OP == R_MAX;
  h2 best;
  OCN_DEV void init() {
    const _Float16 start = MX ? (_Float16)-__builtin_inff() : (_Float16)__builtin_inff();
    best = h2{start, start};
  }
  OCN_DEV void add_word(uint32_t w) {
    const h2 x = __builtin_bit_cast(h2, w);
    best = MX ? __builtin_elementwise_maximum(best, x) : __builtin_elementwise_minimum(best, x);
  }
  OCN_DEV void add_full(const Pk &pk) {
    const uint32_t *w = reinterpret_cast<const uint32_t *>(&pk);
#pragma unroll
    for (int k = 0; k < 4; ++k) add_word(w[k]);
  }
  OCN_DEV void add_partial(const Pk &pk, int n) {
    // pad the missing slots by repeating the first element (n >= 1 here).  The bits are taken
    // element by element from the values that were stored (no access through another type: the
    // elements were written as halves, and only the first n of them).
    uint32_t h[V];
#pragma unroll
    for (int i = 0; i < V; ++i) h[i] = __builtin_bit_cast(uint16_t, pk.v[i < n ? i : 0]);
#pragma unroll
    for (int k = 0; k < 4; ++k) add_word(h[2 * k] | (h[2 * k + 1] << 16));
  }
  OCN_DEV A result() {
    const _Float16 r = MX ? __builtin_elementwise_maximum(best.x, best.y) : __builtin_elementwise_minimum(best.x, best.y);
    return hreg{(float)r};
  }
};

// NT: the load carries the streaming (non-temporal) hint.  An input far larger than the caches
// is read once and never again; read this way a wavefront's whole-line requests stream about
// 7 % faster from HBM (fp32 row sums over 256 MiB: 43.9 -> 40.4 us).  Only for 16-byte pieces
// that neighbouring lanes read side by side: with partial lines the hint costs time.
// A pack whose tensor is stored in the other byte order is put right as soon as it is loaded.
template <int S, class Pk> OCN_DEV void order_pack(bool swapped, Pk &pk) {
  if constexpr (scalar_bytes(S) > 1) {
    if (swapped) reverse_scalars<scalar_bytes(S)>(pk);
  }
}
template <int S> OCN_DEV storage_t<S> load_one(bool swapped, const char *src) {
  storage_t<S> v = *reinterpret_cast<const storage_t<S> *>(src);
  order_pack<S>(swapped, v);
  return v;
}

template <class St, int V, bool NT = false, class Pk> OCN_DEV void load_vec(const char *src, Pk &pk) {
  if constexpr (sizeof(St) * V >= 16) {
    using Q = uint32_t __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int i = 0; i < (int)(sizeof(St) * V / 16); ++i) {
      if constexpr (NT) reinterpret_cast<Q *>(&pk)[i] = __builtin_nontemporal_load(reinterpret_cast<const Q *>(src) + i);
      else reinterpret_cast<Q *>(&pk)[i] = reinterpret_cast<const Q *>(src)[i];
    }
  } else {
#pragma unroll
    for (int i = 0; i < V; ++i) pk.v[i] = reinterpret_cast<const St *>(src)[i];
  }
}

// Fold vectors t0 .. t1-1 of one output's addends, `lanes` lanes cooperating.  The bulk runs
// in a loop without any per-lane condition (every lane loads U whole vectors per trip); the
// ragged remainder - the last few vectors, and the partial vector at the end of a run whose
// length is not a multiple of V - goes through a checked loop.
template <int S, int OP, int V, bool SINGLE, bool NT>
OCN_DEV typename Reducer<S, OP>::A rows_accumulate_impl(const RedArgs &p, const char *base, int64_t t0,
                                                        int64_t t1, int lane, int lanes) {
  using R = Reducer<S, OP>;
  using St = storage_t<S>;
  using F = VecFold<S, OP, V>;
  using Pk = typename F::Pk;
  constexpr int U = 4;  // independent folds and loads in flight per lane
  auto address = [&](int64_t tt, int64_t &e0) -> const char * {
    int64_t off = 0, iv = tt;
    if constexpr (!SINGLE) {
      const uint32_t q = rfastdiv((uint32_t)tt, p.vpr_div);
      iv = (uint32_t)tt - q * p.vpr_div.d;
      off = reduced_offset(p, q, 1);
    }
    e0 = iv * V;
    // single elements may be strided along the innermost reduced dim, vectors are contiguous
    return base + off + e0 * (V == 1 ? p.rsa[0] : (int64_t)sizeof(St));
  };
  if (t1 - t0 <= lanes) {  // short rows: at most one vector per lane, no loops
    F one;
    one.init();
    const int64_t tt = t0 + lane;
    if (tt < t1) {
      Pk pk;
      int64_t e0;
      const char *src = address(tt, e0);
      const int64_t left = p.n0 - e0;
      if (left >= V) {
        load_vec<St, V, NT>(src, pk);
        order_pack<S>(p.swap_a != 0, pk); one.add_full(pk);
      } else {
#pragma unroll
        for (int i = 0; i < V; ++i)
          if (i < (int)left) pk.v[i] = reinterpret_cast<const St *>(src)[i];
        order_pack<S>(p.swap_a != 0, pk); one.add_partial(pk, (int)left);
      }
    }
    return one.result();
  }
  F fold[U];
#pragma unroll
  for (int u = 0; u < U; ++u) fold[u].init();
  // vectors below t_full are known to be whole
  int64_t t_full = t0;
  if constexpr (SINGLE) {
    t_full = p.n0 / V;
    if (t_full > t1) t_full = t1;
  } else if (p.n0 % V == 0) {
    t_full = t1;
  }
  int64_t t = t0;
  for (; t + (int64_t)lanes * U <= t_full; t += (int64_t)lanes * U) {
    Pk pk[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int64_t e0;
      load_vec<St, V, NT>(address(t + (int64_t)u * lanes + lane, e0), pk[u]);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      order_pack<S>(p.swap_a != 0, pk[u]);
      fold[u].add_full(pk[u]);
    }
  }
  for (; t + lanes <= t_full; t += lanes) {  // whole vectors, one per lane and trip
    Pk pk;
    int64_t e0;
    load_vec<St, V, NT>(address(t + lane, e0), pk);
    order_pack<S>(p.swap_a != 0, pk); fold[0].add_full(pk);
  }
  for (int64_t tt = t + lane; tt < t1; tt += lanes) {
    Pk pk;
    int64_t e0;
    const char *src = address(tt, e0);
    const int64_t left = p.n0 - e0;
    if (left >= V) {
      load_vec<St, V, NT>(src, pk);
      order_pack<S>(p.swap_a != 0, pk); fold[0].add_full(pk);
    } else {
#pragma unroll
      for (int i = 0; i < V; ++i)
        if (i < (int)left) pk.v[i] = reinterpret_cast<const St *>(src)[i];
      order_pack<S>(p.swap_a != 0, pk); fold[0].add_partial(pk, (int)left);
    }
  }
  typename R::A acc = fold[0].result();
#pragma unroll
  for (int u = 1; u < U; ++u) acc = R::combine(acc, fold[u].result());
  return acc;
}

// Fold vectors t0 .. t1-1 of one output's addends, `lanes` lanes cooperating.  The bulk runs
// in a loop without any per-lane condition (every lane loads U whole vectors per trip); the
// ragged remainder - the last few vectors, and the partial vector at the end of a run whose
// length is not a multiple of V - goes through a checked loop.  A single reduced dimension
// (the common case) needs no index decomposition at all.
template <int S, int OP, int V>
OCN_DEV typename Reducer<S, OP>::A rows_accumulate(const RedArgs &p, const char *base, int64_t t0, int64_t t1,
                                                   int lane, int lanes) {
  if (p.nred == 1) {
    if (V > 1 && p.nt_load) return rows_accumulate_impl<S, OP, V, true, (V > 1)>(p, base, t0, t1, lane, lanes);
    return rows_accumulate_impl<S, OP, V, true, false>(p, base, t0, t1, lane, lanes);
  }
  return rows_accumulate_impl<S, OP, V, false, false>(p, base, t0, t1, lane, lanes);
}

// Eight wavefronts per SIMD (at most 64 vector registers): 16384 one-wavefront rows then fill
// the chip in exactly two rounds instead of two and two thirds.
#ifndef OCN_ROWS_OCC
#define OCN_ROWS_OCC __attribute__((amdgpu_waves_per_eu(8, 8)))
#endif
template <int S, int OP> __global__ __launch_bounds__(kBlock) OCN_ROWS_OCC void red_rows_kernel(const RedArgs p) {
  using R = Reducer<S, OP>;
  using A = typename R::A;
  constexpr int VF = 16 / (int)sizeof(storage_t<S>) > 0 ? 16 / (int)sizeof(storage_t<S>) : 1;
  __shared__ A lds[kBlock / kWave];

  const int tid = threadIdx.x;
  const int lane_in_wave = tid & (kWave - 1);
  const int wave = tid / kWave;
  // p.group lanes share one output: a whole workgroup, or a power of two up to a wavefront
  const bool per_block = p.group == kBlock;
  const int width = per_block ? kWave : p.group;
  const int64_t gidx = per_block ? (int64_t)blockIdx.x : ((int64_t)blockIdx.x * kBlock + tid) >> (__ffs(width) - 1);
  const int64_t ngroups = p.nout * p.split;
  const bool active = gidx < ngroups;
  const int lane = per_block ? tid : (lane_in_wave & (width - 1));
  A acc = R::identity();
  int64_t o = 0, s = 0, off_o = 0;
  if (active) {
    int64_t t0 = 0, t1 = p.nvec;
    o = gidx;
    if (p.split != 1) {
      o = gidx / p.split;
      s = gidx - o * p.split;
      t0 = s * p.chunk;
      t1 = t0 + p.chunk;
      if (t1 > p.nvec) t1 = p.nvec;
    }
    int64_t off_a;
    kept_offsets(p, (uint32_t)o, off_a, off_o);
    const int lanes = per_block ? kBlock : width;
    if (p.vec > 1) acc = rows_accumulate<S, OP, VF>(p, p.a + off_a, t0, t1, lane, lanes);
    else acc = rows_accumulate<S, OP, 1>(p, p.a + off_a, t0, t1, lane, lanes);
  }
  acc = group_fold<R>(acc, width);   // every lane takes part, whether its group has work or not
  if (per_block) {  // combine the four wavefronts of the workgroup
    if (lane_in_wave == 0) lds[wave] = acc;
    __syncthreads();
    if (tid == 0) {
#pragma unroll
      for (int w = 1; w < kBlock / kWave; ++w) acc = R::combine(acc, lds[w]);
    }
  }
  if (active && lane == 0) {
    if (p.split == 1) {
      store_result<A>(p.out + off_o, p.out_dtype, acc, p.swap_o != 0);
    } else {
      reinterpret_cast<typename R::P *>(p.partial)[o * p.split + s] = to_storage<R::ACC>(acc);
    }
  }
}

// The common row reduction - one reduced dim, contiguous and read in whole 16-byte vectors, at
// most one kept dim, a wavefront or a workgroup per output (or per split of it) - without the
// index decomposition and the 64-bit bookkeeping of the general kernel.  A wavefront lives for
// only a few loop trips on rows of some KiB, so what it executes before its first load and
// after its last one is time during which it has nothing in flight (half-precision maxima
// over rows of 8 KiB: 24.6 us in the general kernel).  Same fold order as the general kernel.
// (SW, the input's byte order, is a template parameter like NT: decided per vector inside the
// loop, the reversal is computed for every vector and selected away - a quarter of the loop's
// instructions for half-precision maxima)
template <int S, int OP, bool NT, bool SW>
OCN_DEV typename Reducer<S, OP>::A lean_fold(const char *base, uint32_t t0, uint32_t t1, uint32_t lane, uint32_t lanes) {
  constexpr bool sw = SW;
  using R = Reducer<S, OP>;
  using St = storage_t<S>;
  constexpr int V = 16 / (int)sizeof(St);
  using F = VecFold<S, OP, V>;
  using Pk = typename F::Pk;
  constexpr int U = 4;
  F fold[U];
#pragma unroll
  for (int u = 0; u < U; ++u) fold[u].init();
  uint32_t t = t0 + lane;
  for (; t + (U - 1) * lanes < t1; t += U * lanes) {
    Pk pk[U];
#pragma unroll
    for (int u = 0; u < U; ++u) load_vec<St, V, NT>(base + (uint64_t)(t + u * lanes) * 16u, pk[u]);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      order_pack<S>(sw, pk[u]);
      fold[u].add_full(pk[u]);
    }
  }
  // two vectors at a time while they last: a row of two or three vectors per lane takes one
  // round trip less
  for (; t + lanes < t1; t += 2 * lanes) {
    Pk pk[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) load_vec<St, V, NT>(base + (uint64_t)(t + u * lanes) * 16u, pk[u]);
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      order_pack<S>(sw, pk[u]);
      fold[u].add_full(pk[u]);
    }
  }
  for (; t < t1; t += lanes) {
    Pk pk;
    load_vec<St, V, NT>(base + (uint64_t)t * 16u, pk);
    order_pack<S>(sw, pk); fold[0].add_full(pk);
  }
  typename R::A acc = fold[0].result();
#pragma unroll
  for (int u = 1; u < U; ++u) acc = R::combine(acc, fold[u].result());
  return acc;
}

template <int S, int OP> __global__ __launch_bounds__(kBlock) OCN_ROWS_OCC void red_rows_lean_kernel(const RedLeanArgs q) {
  using R = Reducer<S, OP>;
  using A = typename R::A;
  if constexpr (sizeof(storage_t<S>) < 16) {
    RedLeanArgs p = q;
    OCN_ARGS_NOW("s"(p.a), "s"(p.out), "s"(p.partial), "s"(p.ksa), "s"(p.kso), "s"(p.nout), "s"(p.split), "s"(p.nvec),
                 "s"(p.chunk), "s"(p.out_dtype), "s"(p.group), "s"(p.nt_load), "s"(p.swap_a), "s"(p.swap_o));
    __shared__ A lds[kBlock / kWave];
    const uint32_t tid = threadIdx.x, lane_in_wave = tid & (kWave - 1), wave = tid / kWave;
    const bool per_block = p.group == kBlock;
    const uint32_t gidx = per_block ? blockIdx.x : blockIdx.x * (kBlock / kWave) + wave;
    const bool active = gidx < p.nout * p.split;
    const uint32_t lane = per_block ? tid : lane_in_wave;
    uint32_t o = gidx, sp = 0, t0 = 0, t1 = p.nvec;
    A acc = R::identity();
    // (the row's address is formed before the branch, for every wavefront: inside it, the
    // compiler fetches the pointer with a scalar load of its own, one more round trip
    // before the wavefront's first load)
    if (p.split != 1) {
      o = gidx / p.split;
      sp = gidx - o * p.split;
      t0 = sp * p.chunk;
      t1 = t0 + p.chunk < p.nvec ? t0 + p.chunk : p.nvec;
    }
    const char *base = p.a + (int64_t)o * p.ksa;
    if (active) {
      const uint32_t lanes = per_block ? kBlock : kWave;
      if (p.swap_a) {
        if (p.nt_load) acc = lean_fold<S, OP, true, true>(base, t0, t1, lane, lanes);
        else acc = lean_fold<S, OP, false, true>(base, t0, t1, lane, lanes);
      } else {
        if (p.nt_load) acc = lean_fold<S, OP, true, false>(base, t0, t1, lane, lanes);
        else acc = lean_fold<S, OP, false, false>(base, t0, t1, lane, lanes);
      }
    }
    acc = group_fold<R>(acc, kWave);
    if (per_block) {
      if (lane_in_wave == 0) lds[wave] = acc;
      __syncthreads();
      if (tid == 0) {
#pragma unroll
        for (int w = 1; w < kBlock / kWave; ++w) acc = R::combine(acc, lds[w]);
      }
    }
    if (active && lane == 0) {
      if (p.split == 1) store_result<A>(p.out + (int64_t)o * p.kso, p.out_dtype, acc, p.swap_o != 0);
      else reinterpret_cast<typename R::P *>(p.partial)[(uint64_t)o * p.split + sp] = to_storage<R::ACC>(acc);
    }
  }
}

// Rows of at most one vector per lane of their group, a single reduced dim, no split: the
// same groups, loads and fold order as red_rows_kernel without its loops and its 64-bit
// bookkeeping (short rows are bound by instruction issue, not by memory).
template <int S, int OP, int V, bool NT>
OCN_DEV typename Reducer<S, OP>::A short_row_fold(const RedArgs &p, const char *base, uint32_t lane) {
  using St = storage_t<S>;
  using F = VecFold<S, OP, V>;
  using Pk = typename F::Pk;
  F one;
  one.init();
  if (lane < (uint32_t)p.nvec) {
    Pk pk;
    const uint32_t e0 = lane * V;
    const char *src = base + (int64_t)e0 * (V == 1 ? p.rsa[0] : (int64_t)sizeof(St));
    const uint32_t left = (uint32_t)p.n0 - e0;
    if (left >= (uint32_t)V) {
      load_vec<St, V, NT>(src, pk);
      order_pack<S>(p.swap_a != 0, pk); one.add_full(pk);
    } else {
#pragma unroll
      for (int i = 0; i < V; ++i)
        if (i < (int)left) pk.v[i] = reinterpret_cast<const St *>(src)[i];
      order_pack<S>(p.swap_a != 0, pk); one.add_partial(pk, (int)left);
    }
  }
  return one.result();
}

template <int S, int OP> __global__ __launch_bounds__(kBlock) void red_rows_short_kernel(const RedArgs p) {
  using R = Reducer<S, OP>;
  using A = typename R::A;
  constexpr int VF = 16 / (int)sizeof(storage_t<S>) > 0 ? 16 / (int)sizeof(storage_t<S>) : 1;
  const uint32_t width = (uint32_t)p.group;
  const uint32_t gl = blockIdx.x * kBlock + threadIdx.x;
  const uint32_t o = gl >> (__ffs(p.group) - 1), lane = gl & (width - 1);
  const bool active = o < (uint32_t)p.nout;
  A acc = R::identity();
  int64_t off_o = 0;
  if (active) {
    int64_t off_a;
    kept_offsets(p, o, off_a, off_o);
    if (p.vec > 1) {
      if (p.nt_load) acc = short_row_fold<S, OP, VF, (VF > 1)>(p, p.a + off_a, lane);
      else acc = short_row_fold<S, OP, VF, false>(p, p.a + off_a, lane);
    } else {
      acc = short_row_fold<S, OP, 1, false>(p, p.a + off_a, lane);
    }
  }
  acc = group_fold<R>(acc, (int)width);
  if (active && lane == 0) store_result<A>(p.out + off_o, p.out_dtype, acc, p.swap_o != 0);
}

// The second launch of a split column reduction: partial results [split][output] of eight bytes
// each, one output per lane, all loads of a lane issued eight at a time and folded in the order
// of the splits.  The launch is a chain of latencies (arguments, partial results, store), so it
// gets few arguments and no index arithmetic (fp32 column sums of [16384, 4096], 16 x 4096
// partial results: 7.1 us in the column kernel).
template <int S, int OP> __global__ __launch_bounds__(kWave) void red_fold_kernel(const RedFoldArgs p) {
  using R = Reducer<S, OP>;
  using A = typename R::A;
  using St = storage_t<S>;
  if constexpr (sizeof(St) == 8) {
    const uint32_t o = blockIdx.x * kWave + threadIdx.x;
    if (o >= p.nout) return;
    const St *src = reinterpret_cast<const St *>(p.partial) + o;
    A acc = R::identity();
    constexpr uint32_t U = 8;
    uint32_t s = 0;
    for (; s + U <= p.split; s += U) {
      St v[U];
#pragma unroll
      for (uint32_t u = 0; u < U; ++u) v[u] = src[(uint64_t)(s + u) * p.nout];
#pragma unroll
      for (uint32_t u = 0; u < U; ++u) acc = R::combine(acc, R::lift(from_storage<S>(v[u])));
    }
    for (; s < p.split; ++s) acc = R::combine(acc, R::lift(from_storage<S>(src[(uint64_t)s * p.nout])));
    store_result<A>(p.out + (int64_t)o * p.kso, p.out_dtype, acc, p.swap_o != 0);
  }
}

// ---------------------------------------------------------------------------------------
// cols
// ---------------------------------------------------------------------------------------

constexpr int kColsMaxWaves = 16;  // the cols kernel runs with 4 or 16 wavefronts per workgroup
// columns of a lane's vector that the wavefronts of a workgroup combine through LDS at a time
// (32 KiB for sixteen wavefronts; the launcher sizes the dynamic LDS accordingly)
template <class A> OCN_HD constexpr int cols_lds_columns() { return sizeof(A) <= 8 ? 4 : 2; }
template <class A> OCN_HD constexpr size_t cols_lds_bytes(int block, int vec) {
  return (size_t)(block / kWave) * kWave * sizeof(A) * (size_t)(cols_lds_columns<A>() < vec ? cols_lds_columns<A>() : vec);
}

// SINGLE: one reduced dim, so that row r lies r strides further on (no index decomposition)
template <int S, int OP, int V, bool NT, bool SINGLE>
OCN_DEV void cols_body(const RedArgs &p, typename Reducer<S, OP>::A *lds) {
  using R = Reducer<S, OP>;
  using A = typename R::A;
  using St = storage_t<S>;
  auto row_offset = [&](int64_t r) -> int64_t {
    if constexpr (SINGLE) return r * p.rsa[0];
    else return reduced_offset(p, (uint32_t)r, 0);
  };
  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wave = tid / kWave;
  const int NW = (int)blockDim.x / kWave;

  // block -> (split, other kept dims, column block)
  uint32_t b = blockIdx.x;
  const uint32_t per_split = (uint32_t)(p.colblocks_div.d * (uint32_t)(p.nout / p.nc));
  const uint32_t s = b / per_split;
  b -= s * per_split;
  const uint32_t other = rfastdiv(b, p.colblocks_div);
  const uint32_t cb = b - other * p.colblocks_div.d;
  // p.cpw lanes (a power of two) cover one row of columns; with fewer than 64 of them a
  // wavefront takes 64 / cpw rows at a time
  const int cpw_log2 = __ffs(p.cpw) - 1;
  const int lc = lane & (p.cpw - 1), lr = lane >> cpw_log2;
  const int RPW = kWave >> cpw_log2;
  const int64_t col0 = ((int64_t)cb * p.cpw + lc) * V;
  const int64_t left = p.nc - col0;
  const int ncol = left >= V ? V : (left > 0 ? (int)left : 0);

  // offsets of the other kept dims (kept dim 0 is the column dim)
  int64_t off_a = col0 * (int64_t)sizeof(St), off_o = col0 * p.kso[0];
  {
    uint32_t o = other;
#pragma unroll
    for (int k = 1; k < kMaxDims; ++k) {
      if (k < p.nkept) {
        const uint32_t q = (k == p.nkept - 1) ? 0u : rfastdiv(o, p.kdiv[k]);
        const uint32_t i = o - q * p.kdiv[k].d;
        o = q;
        off_a += (int64_t)i * p.ksa[k];
        off_o += (int64_t)i * p.kso[k];
      }
    }
  }

  A acc[V];
#pragma unroll
  for (int i = 0; i < V; ++i) acc[i] = R::identity();
  const int64_t r0 = (int64_t)s * p.chunk;
  int64_t r1 = r0 + p.chunk;
  if (r1 > p.nredtot) r1 = p.nredtot;
  constexpr int U = 4;  // rows in flight per wavefront
  struct alignas(sizeof(St) * V >= 16 ? 16 : sizeof(St) * V) Pk { St v[V]; };
  // Each wavefront takes one contiguous run of the workgroup's rows (RPW rows at a time).
  // Dealing the rows out in turn instead - wavefront w taking rows w, w + NW, ... - measured
  // 10 % slower (fp32 column sums of [16384, 4096]: 46.2 against 41.5 us).
  const int RS = RPW;                // rows between two rows of the same lane
  const int64_t per_wave = (((r1 - r0) + NW - 1) / NW + RPW - 1) / RPW * RPW;
  const int64_t w0 = r0 + (int64_t)wave * per_wave;   // this wavefront's rows: w0 .. r1 - 1
  if (w0 + per_wave < r1) r1 = w0 + per_wave;
  int64_t r = w0 + lr;
  // Sums of 8-bit integers: the sixteen columns of a vector are added two at a time, as 16-bit
  // halves of 32-bit words (signed bytes biased by 128 to make them unsigned), and spilled into
  // the 64-bit accumulators every 256 rows, before a half can overflow (256 * 255 < 2^16).
  constexpr bool PACKED8 = (S == DT_I8 || S == DT_U8) && OP == R_SUM && V == 16;
  bool packed_done = false;
  if constexpr (PACKED8) {
    if (ncol == V) {
      packed_done = true;
      uint32_t even[4] = {0, 0, 0, 0}, odd[4] = {0, 0, 0, 0};  // bytes 0 and 2 / 1 and 3 of each word
      uint32_t pending = 0;                                    // rows added since the last spill
      auto spill = [&]() {
        const A bias = S == DT_I8 ? (A)128 * (A)pending : (A)0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          acc[4 * k + 0] += (A)(even[k] & 0xffffu) - bias;
          acc[4 * k + 1] += (A)(odd[k] & 0xffffu) - bias;
          acc[4 * k + 2] += (A)(even[k] >> 16) - bias;
          acc[4 * k + 3] += (A)(odd[k] >> 16) - bias;
          even[k] = odd[k] = 0;
        }
        pending = 0;
      };
      auto add_row = [&](const Pk &pk) {
        uint32_t w[4];
        __builtin_memcpy(w, &pk, 16);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const uint32_t x = S == DT_I8 ? w[k] ^ 0x80808080u : w[k];
          even[k] += x & 0x00ff00ffu;
          odd[k] += (x >> 8) & 0x00ff00ffu;
        }
        if (++pending == 256) spill();
      };
      for (; r + (int64_t)(U - 1) * RS < r1; r += RS * U) {
        Pk pk[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
          load_vec<St, V, NT>(p.a + off_a + row_offset(r + (int64_t)u * RS), pk[u]);
#pragma unroll
        for (int u = 0; u < U; ++u) add_row(pk[u]);
      }
      for (; r < r1; r += RS) {
        Pk pk;
        load_vec<St, V, NT>(p.a + off_a + row_offset(r), pk);
        add_row(pk);
      }
      spill();
    }
  }
  if (packed_done) {
    // (nothing left to add)
  } else if (ncol == V) {  // whole vectors of columns: no per-element conditions
    // (one loop per byte order: decided per row inside the loop, the reversal is computed for
    // every vector and selected away)
    auto rows = [&](auto swapped) {
      constexpr bool SW = decltype(swapped)::value;
      for (; r + (int64_t)(U - 1) * RS < r1; r += RS * U) {
        Pk pk[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
          load_vec<St, V, NT>(p.a + off_a + row_offset(r + (int64_t)u * RS), pk[u]);
#pragma unroll
        for (int u = 0; u < U; ++u) {
          order_pack<S>(SW, pk[u]);
#pragma unroll
          for (int i = 0; i < V; ++i) acc[i] = R::combine(acc[i], R::lift(from_storage<S>(pk[u].v[i])));
        }
      }
      for (; r < r1; r += RS) {
        Pk pk;
        load_vec<St, V, NT>(p.a + off_a + row_offset(r), pk);
        order_pack<S>(SW, pk);
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] = R::combine(acc[i], R::lift(from_storage<S>(pk.v[i])));
      }
    };
    if (p.swap_a) rows(std::true_type{});
    else rows(std::false_type{});
  } else if (ncol > 0) {  // the ragged last column block
    for (; r < r1; r += RS) {
      const char *src = p.a + off_a + row_offset(r);
#pragma unroll
      for (int i = 0; i < V; ++i)
        if (i < ncol) acc[i] = R::combine(acc[i], R::lift(from_storage<S>(load_one<S>(p.swap_a != 0, src + (int64_t)i * (int64_t)sizeof(St)))));
    }
  }
  // lanes of a wavefront that hold the same columns of different rows: fold onto the first
  if (RPW > 1) {
#pragma unroll
    for (int i = 0; i < V; ++i)
#pragma unroll
      for (int d = kWave / 2; d >= 1; d >>= 1)
        if (d >= p.cpw) acc[i] = R::combine(acc[i], shfl_down_any(acc[i], d));
  }
  // Combine the wavefronts (same columns, different rows): CH columns of the vector go through
  // LDS at a time, and wavefront c folds column c over all wavefronts, in wavefront order.  (One
  // column at a time, folded by the first wavefront alone, was four rounds of a barrier and a
  // chain of sixteen LDS reads and adds at the end of every workgroup - and the workgroups of
  // a split reduction all end together.)
  constexpr int CH = cols_lds_columns<A>() < V ? cols_lds_columns<A>() : V;
#pragma unroll
  for (int i0 = 0; i0 < V; i0 += CH) {
#pragma unroll
    for (int c = 0; c < CH; ++c) lds[((size_t)wave * CH + c) * kWave + lane] = acc[i0 + c];
    __syncthreads();
    if (wave < CH && lr == 0 && i0 + wave < ncol) {
      const int c = wave, i = i0 + wave;
      A v = lds[(size_t)c * kWave + lane];
      for (int w = 1; w < NW; ++w) v = R::combine(v, lds[((size_t)w * CH + c) * kWave + lane]);
      if (p.split == 1) {
        store_result<A>(p.out + off_o + (int64_t)i * p.kso[0], p.out_dtype, v, p.swap_o != 0);
      } else {
        const int64_t olin = (int64_t)other * p.nc + col0 + i;
        reinterpret_cast<typename R::P *>(p.partial)[(int64_t)s * p.nout + olin] = to_storage<R::ACC>(v);
      }
    }
    if (i0 + CH < V) __syncthreads();
  }
}

template <int S, int OP> __global__ __launch_bounds__(kColsMaxWaves * kWave) void red_cols_kernel(const RedArgs p) {
  using A = typename Reducer<S, OP>::A;
  constexpr int VF = 16 / (int)sizeof(storage_t<S>) > 0 ? 16 / (int)sizeof(storage_t<S>) : 1;
  extern __shared__ __align__(16) unsigned char red_cols_lds_raw[];
  A *lds = reinterpret_cast<A *>(red_cols_lds_raw);
  if (p.vec > 1 && p.nred == 1) {
    if (p.nt_load) cols_body<S, OP, VF, (VF > 1), true>(p, lds);
    else cols_body<S, OP, VF, false, true>(p, lds);
  } else if (p.vec > 1) {
    cols_body<S, OP, VF, false, false>(p, lds);
  } else {
    cols_body<S, OP, 1, false, false>(p, lds);
  }
}

// ---------------------------------------------------------------------------------------
// generic
// ---------------------------------------------------------------------------------------

template <int S, int OP> __global__ __launch_bounds__(kBlock) void red_generic_kernel(const RedArgs p) {
  using R = Reducer<S, OP>;
  using A = typename R::A;
  using St = storage_t<S>;
  // the grid is capped (a launch cannot have 2^32 lanes): more outputs than lanes loop
  for (int64_t o = (int64_t)blockIdx.x * kBlock + threadIdx.x; o < p.nout; o += (int64_t)gridDim.x * kBlock) {
  // 64-bit decomposition over the kept dims (fastest first)
  int64_t off_a = 0, off_o = 0, t = o;
#pragma unroll
  for (int k = 0; k < kMaxDims; ++k) {
    if (k < p.nkept) {
      const int64_t n = p.ksize[k];
      const int64_t q = t / n;
      const int64_t i = t - q * n;
      t = q;
      off_a += i * p.ksa[k];
      off_o += i * p.kso[k];
    }
  }
  A acc = R::identity();
  for (int64_t r = 0; r < p.nredtot; ++r) {
    int64_t off = 0, q = r;
#pragma unroll
    for (int k = 0; k < kMaxDims; ++k) {
      if (k < p.nred) {
        const int64_t n = p.rsize[k];
        const int64_t qq = q / n;
        off += (q - qq * n) * p.rsa[k];
        q = qq;
      }
    }
    acc = R::combine(acc, R::lift(from_storage<S>(load_one<S>(p.swap_a != 0, p.a + off_a + off))));
  }
  store_result<A>(p.out + off_o, p.out_dtype, acc, p.swap_o != 0);
  }
}

#endif  // __HIPCC__

}  // namespace ocn
