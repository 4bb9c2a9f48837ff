// Reduction kernels of the tensor engine for gfx950 (section 3.2 of the paper: tensor
// reductions along one or more axes).
//
//   red_rows_kernel     the reduced axis is the input's fastest: a wavefront (short rows) or a
//                       whole workgroup (long rows) streams one output's addends with 128-bit
//                       loads, lanes fold privately, then a wavefront shuffle tree and an LDS
//                       step combine them.  Long reductions with few outputs are split over
//                       several workgroups; each writes a partial result to the workspace and a
//                       second launch folds the partials (two-pass grid reduction).
//   red_cols_kernel     a kept axis is the input's fastest: lanes own adjacent output columns,
//                       the four wavefronts of a workgroup take interleaved rows and are
//                       combined through LDS; row ranges can be split the same way.
//   red_generic_kernel  any layout: one output per lane, sequential fold.
// No floating-point atomics anywhere: the grouping of addends is fixed by the launch
// geometry, so results are reproducible bit for bit.
#pragma once

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

// convert an accumulator to the runtime output dtype and store it (once per output)
template <class A> __device__ __noinline__ void store_result(char *p, int dt, A r) {
  switch (dt) {
#define OCN_CASE(D) \
  case D: *reinterpret_cast<storage_t<D> *>(p) = to_storage<D>(convert<D>(r)); break;
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

template <class R, int S, int V>
OCN_DEV typename R::A rows_accumulate(const RedArgs &p, const char *base, int64_t t0, int64_t t1,
                                      int lane, int lanes) {
  using St = storage_t<S>;
  using A = typename R::A;
  constexpr int U = 4;  // independent accumulators and loads in flight per lane
  A acc[U];
#pragma unroll
  for (int u = 0; u < U; ++u) acc[u] = R::identity();
  const bool single_run = p.nred == 1;
  for (int64_t t = t0 + lane; t < t1; t += (int64_t)lanes * U) {
    struct alignas(sizeof(St) * V >= 16 ? 16 : sizeof(St) * V) Pk { St v[V]; } pk[U];
    int nval[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t tt = t + (int64_t)u * lanes;
      nval[u] = 0;
      if (tt < t1) {
        int64_t off, iv;
        if (single_run) {
          iv = tt;
          off = 0;
        } else {
          const uint32_t q = rfastdiv((uint32_t)tt, p.vpr_div);
          iv = (uint32_t)tt - q * p.vpr_div.d;
          off = reduced_offset(p, q, 1);
        }
        const int64_t e0 = iv * V;
        const int64_t left = p.n0 - e0;
        const int n = left >= V ? V : (int)left;
        nval[u] = n;
        const char *src = base + off + e0 * (int64_t)sizeof(St);
        if (n == V) {
          if constexpr (sizeof(St) * V >= 16) {
            using Q = uint32_t __attribute__((ext_vector_type(4)));
#pragma unroll
            for (int i = 0; i < (int)(sizeof(St) * V / 16); ++i)
              reinterpret_cast<Q *>(&pk[u])[i] = reinterpret_cast<const Q *>(src)[i];
          } else {
#pragma unroll
            for (int i = 0; i < V; ++i) pk[u].v[i] = reinterpret_cast<const St *>(src)[i];
          }
        } else {
#pragma unroll
          for (int i = 0; i < V; ++i)
            if (i < n) pk[u].v[i] = reinterpret_cast<const St *>(src)[i];
        }
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (nval[u] == V) {
#pragma unroll
        for (int i = 0; i < V; ++i) acc[u] = R::combine(acc[u], R::lift(from_storage<S>(pk[u].v[i])));
      } else {
#pragma unroll
        for (int i = 0; i < V; ++i)
          if (i < nval[u]) acc[u] = R::combine(acc[u], R::lift(from_storage<S>(pk[u].v[i])));
      }
    }
  }
#pragma unroll
  for (int u = 1; u < U; ++u) acc[0] = R::combine(acc[0], acc[u]);
  return acc[0];
}

template <int S, int OP> __global__ __launch_bounds__(kBlock) void red_rows_kernel(const RedArgs p) {
  using R = Reducer<S, OP>;
  using A = typename R::A;
  constexpr int VF = 16 / (int)sizeof(storage_t<S>) > 0 ? 16 / (int)sizeof(storage_t<S>) : 1;
  __shared__ A lds[kBlock / kWave];

  const int tid = threadIdx.x;
  const int lane_in_wave = tid & (kWave - 1);
  const int wave = tid / kWave;
  const bool per_wave = p.group == kWave;
  const int64_t gidx = per_wave ? (int64_t)blockIdx.x * (kBlock / kWave) + wave : (int64_t)blockIdx.x;
  const int64_t ngroups = p.nout * p.split;
  const bool active = gidx < ngroups;
  A acc = R::identity();
  int64_t o = 0, s = 0;
  if (active) {
    o = p.split == 1 ? gidx : gidx / p.split;
    s = gidx - o * p.split;
    int64_t off_a, off_o;
    kept_offsets(p, (uint32_t)o, off_a, off_o);
    const int64_t t0 = s * p.chunk;
    int64_t t1 = t0 + p.chunk;
    if (t1 > p.nvec) t1 = p.nvec;
    const int lane = per_wave ? lane_in_wave : tid;
    const int lanes = per_wave ? kWave : kBlock;
    if (p.vec > 1) acc = rows_accumulate<R, S, VF>(p, p.a + off_a, t0, t1, lane, lanes);
    else acc = rows_accumulate<R, S, 1>(p, p.a + off_a, t0, t1, lane, lanes);
    acc = wave_fold<R>(acc);
  }
  if (!per_wave) {  // combine the four wavefronts of the workgroup
    if (lane_in_wave == 0) lds[wave] = acc;
    __syncthreads();
    if (tid == 0) {
#pragma unroll
      for (int w = 1; w < kBlock / kWave; ++w) acc = R::combine(acc, lds[w]);
    }
  }
  const bool writer = active && (per_wave ? lane_in_wave == 0 : tid == 0);
  if (writer) {
    if (p.split == 1) {
      int64_t off_a, off_o;
      kept_offsets(p, (uint32_t)o, off_a, off_o);
      store_result<A>(p.out + off_o, p.out_dtype, acc);
    } else {
      reinterpret_cast<typename R::P *>(p.partial)[o * p.split + s] = to_storage<R::ACC>(acc);
    }
  }
}

// ---------------------------------------------------------------------------------------
// cols
// ---------------------------------------------------------------------------------------

template <int S, int OP, int V, int VF>
OCN_DEV void cols_body(const RedArgs &p, typename Reducer<S, OP>::A (*lds)[kWave][VF]) {
  using R = Reducer<S, OP>;
  using A = typename R::A;
  using St = storage_t<S>;
  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wave = tid / kWave;
  constexpr int NW = kBlock / kWave;

  // block -> (split, other kept dims, column block)
  uint32_t b = blockIdx.x;
  const uint32_t per_split = (uint32_t)(p.colblocks_div.d * (uint32_t)(p.nout / p.nc));
  const uint32_t s = b / per_split;
  b -= s * per_split;
  const uint32_t other = rfastdiv(b, p.colblocks_div);
  const uint32_t cb = b - other * p.colblocks_div.d;
  const int64_t col0 = ((int64_t)cb * kWave + lane) * V;
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
  constexpr int U = 4;
  if (ncol > 0) {
    for (int64_t r = r0 + wave; r < r1; r += NW * U) {
      struct alignas(sizeof(St) * V >= 16 ? 16 : sizeof(St) * V) Pk { St v[V]; } pk[U];
      bool ok[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int64_t rr = r + (int64_t)u * NW;
        ok[u] = rr < r1;
        if (ok[u]) {
          const char *src = p.a + off_a + reduced_offset(p, (uint32_t)rr, 0);
          if (ncol == V) {
            if constexpr (sizeof(St) * V >= 16) {
              using Q = uint32_t __attribute__((ext_vector_type(4)));
#pragma unroll
              for (int i = 0; i < (int)(sizeof(St) * V / 16); ++i)
                reinterpret_cast<Q *>(&pk[u])[i] = reinterpret_cast<const Q *>(src)[i];
            } else {
#pragma unroll
              for (int i = 0; i < V; ++i) pk[u].v[i] = reinterpret_cast<const St *>(src)[i];
            }
          } else {
#pragma unroll
            for (int i = 0; i < V; ++i)
              if (i < ncol) pk[u].v[i] = reinterpret_cast<const St *>(src)[i];
          }
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (ok[u]) {
#pragma unroll
          for (int i = 0; i < V; ++i)
            if (i < ncol) acc[i] = R::combine(acc[i], R::lift(from_storage<S>(pk[u].v[i])));
        }
      }
    }
  }
  // combine the wavefronts: each holds the same columns, different rows
#pragma unroll
  for (int i = 0; i < V; ++i) lds[wave][lane][i] = acc[i];
  __syncthreads();
  if (wave == 0 && ncol > 0) {
#pragma unroll
    for (int i = 0; i < V; ++i) {
      A v = lds[0][lane][i];
#pragma unroll
      for (int w = 1; w < NW; ++w) v = R::combine(v, lds[w][lane][i]);
      if (i < ncol) {
        if (p.split == 1) {
          store_result<A>(p.out + off_o + (int64_t)i * p.kso[0], p.out_dtype, v);
        } else {
          const int64_t olin = (int64_t)other * p.nc + col0 + i;
          reinterpret_cast<typename R::P *>(p.partial)[(int64_t)s * p.nout + olin] = to_storage<R::ACC>(v);
        }
      }
    }
  }
}

template <int S, int OP> __global__ __launch_bounds__(kBlock) void red_cols_kernel(const RedArgs p) {
  using A = typename Reducer<S, OP>::A;
  constexpr int VF = 16 / (int)sizeof(storage_t<S>) > 0 ? 16 / (int)sizeof(storage_t<S>) : 1;
  __shared__ A lds[kBlock / kWave][kWave][VF];
  if (p.vec > 1) cols_body<S, OP, VF, VF>(p, lds);
  else cols_body<S, OP, 1, VF>(p, lds);
}

// ---------------------------------------------------------------------------------------
// generic
// ---------------------------------------------------------------------------------------

template <int S, int OP> __global__ __launch_bounds__(kBlock) void red_generic_kernel(const RedArgs p) {
  using R = Reducer<S, OP>;
  using A = typename R::A;
  using St = storage_t<S>;
  const int64_t o = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (o >= p.nout) return;
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
    acc = R::combine(acc, R::lift(from_storage<S>(*reinterpret_cast<const St *>(p.a + off_a + off))));
  }
  store_result<A>(p.out + off_o, p.out_dtype, acc);
}

#endif  // __HIPCC__

}  // namespace ocn
