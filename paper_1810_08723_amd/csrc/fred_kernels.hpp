// Fused elementwise+reduce kernels for gfx950: out = reduce(op, g(a, b)) without the
// intermediate tensor (sections 3.2 and 5 of the paper: elementwise functions followed by a
// reduction along axes, e.g. the inner product and norm of the QR example).
//
// Each element is produced exactly as the elementwise kernels would store it - converted to
// the intermediate type - and then folded exactly as the reduction kernels would fold it, so
// the result equals the two-step computation up to the order of a floating-point sum.  The
// three layouts and the launch geometry are those of red_kernels.hpp; split reductions write
// partial results that a plain second launch folds.
#pragma once

#include "ew_kernels.hpp"
#include "red_kernels.hpp"

namespace ocn {

#if defined(__HIPCC__)

// input byte offsets (a and b) of reduced index q over the reduced dims from `first` upward
OCN_DEV void reduced_offset2(const RedArgs &p, uint32_t q, int first, int64_t &oa, int64_t &ob) {
  oa = 0;
  ob = 0;
#pragma unroll
  for (int k = 0; k < kMaxDims; ++k) {
    if (k >= first && k < p.nred) {
      const uint32_t qq = (k == p.nred - 1) ? 0u : rfastdiv(q, p.rdiv[k]);
      const uint32_t i = q - qq * p.rdiv[k].d;
      q = qq;
      oa += (int64_t)i * p.rsa[k];
      ob += (int64_t)i * p.rsb[k];
    }
  }
}

// byte offsets of output number `o` in a, b and out
OCN_DEV void kept_offsets2(const RedArgs &p, uint32_t o, int64_t &off_a, int64_t &off_b, int64_t &off_o) {
  off_a = off_b = off_o = 0;
#pragma unroll
  for (int k = 0; k < kMaxDims; ++k) {
    if (k < p.nkept) {
      const uint32_t q = (k == p.nkept - 1) ? 0u : rfastdiv(o, p.kdiv[k]);
      const uint32_t i = o - q * p.kdiv[k].d;
      o = q;
      off_a += (int64_t)i * p.ksa[k];
      off_b += (int64_t)i * p.ksb[k];
      off_o += (int64_t)i * p.kso[k];
    }
  }
}

// V consecutive elements of one input, or V copies of one element where it is broadcast
template <class S, int V, bool NT = false> OCN_DEV void fused_load(const char *src, bool bcast, Pack<S, V> &dst) {
  if (bcast) {
    const S s = *reinterpret_cast<const S *>(src);
#pragma unroll
    for (int i = 0; i < V; ++i) dst.v[i] = s;
  } else {
    if constexpr (NT) load_vec<S, V, true>(src, dst);
    else load_pack<S, V>(src, dst);
  }
}

template <class G, int OP> struct FusedFold {
  static constexpr int E = G::SO_DT;  // type of the intermediate elements
  using R = Reducer<E, OP>;
  using A = typename R::A;
  OCN_DEV static A add(A acc, typename G::SAt a, typename G::SBt b) {
    return R::combine(acc, R::lift(from_storage<E>(G::eval(a, b))));
  }
};

// ---------------------------------------------------------------------------------------
// rows: the reduced axis is the fastest of the inputs
// ---------------------------------------------------------------------------------------

template <class G, int OP, int V>
OCN_DEV typename FusedFold<G, OP>::A fred_rows_accumulate(const RedArgs &p, const char *pa, const char *pb,
                                                          int64_t t0, int64_t t1, int lane, int lanes) {
  using F = FusedFold<G, OP>;
  using A = typename F::A;
  using SAt = typename G::SAt;
  using SBt = typename G::SBt;
#ifndef OCN_FRED_U
#define OCN_FRED_U 2
#endif
  constexpr int U = OCN_FRED_U;
  A acc[U];
#pragma unroll
  for (int u = 0; u < U; ++u) acc[u] = F::R::identity();
  const bool single = p.nred == 1;
  const bool abc = p.a_bcast, bbc = p.b_bcast;
  // vectors below t_full are known to be whole
  int64_t t_full = t0;
  if (p.n0 % V == 0) t_full = t1;
  else if (single) t_full = p.n0 / V < t1 ? p.n0 / V : t1;
  auto address = [&](int64_t tt, int64_t &e0, const char *&qa, const char *&qb) {
    int64_t oa = 0, ob = 0, iv = tt;
    if (!single) {
      const uint32_t q = rfastdiv((uint32_t)tt, p.vpr_div);
      iv = (uint32_t)tt - q * p.vpr_div.d;
      reduced_offset2(p, q, 1, oa, ob);
    }
    e0 = iv * V;
    qa = pa + oa + (abc ? 0 : e0 * (int64_t)sizeof(SAt));
    qb = pb + ob + (bbc ? 0 : e0 * (int64_t)sizeof(SBt));
  };
  int64_t t = t0;
  for (; t + (int64_t)lanes * U <= t_full; t += (int64_t)lanes * U) {
    Pack<SAt, V> va[U];
    Pack<SBt, V> vb[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int64_t e0;
      const char *qa, *qb;
      address(t + (int64_t)u * lanes + lane, e0, qa, qb);
      fused_load<SAt, V>(qa, abc, va[u]);
      fused_load<SBt, V>(qb, bbc, vb[u]);
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int i = 0; i < V; ++i) acc[u] = F::add(acc[u], va[u].v[i], vb[u].v[i]);
  }
  for (int64_t tt = t + lane; tt < t1; tt += lanes) {
    int64_t e0;
    const char *qa, *qb;
    address(tt, e0, qa, qb);
    const int64_t left = p.n0 - e0;
    const int n = left >= V ? V : (int)left;
#pragma unroll
    for (int i = 0; i < V; ++i) {
      if (i < n) {
        const SAt x = reinterpret_cast<const SAt *>(qa)[abc ? 0 : i];
        const SBt y = reinterpret_cast<const SBt *>(qb)[bbc ? 0 : i];
        acc[0] = F::add(acc[0], x, y);
      }
    }
  }
  A r = acc[0];
#pragma unroll
  for (int u = 1; u < U; ++u) r = F::R::combine(r, acc[u]);
  return r;
}

template <class G, int OP> __global__ __launch_bounds__(kBlock) void fred_rows_kernel(const RedArgs p) {
  using F = FusedFold<G, OP>;
  using R = typename F::R;
  using A = typename F::A;
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
    int64_t off_a, off_b;
    kept_offsets2(p, (uint32_t)o, off_a, off_b, off_o);
    const int lanes = per_block ? kBlock : width;
    if (p.vec > 1) acc = fred_rows_accumulate<G, OP, G::V>(p, p.a + off_a, p.b + off_b, t0, t1, lane, lanes);
    else acc = fred_rows_accumulate<G, OP, 1>(p, p.a + off_a, p.b + off_b, t0, t1, lane, lanes);
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
    if (p.split == 1) store_result<A>(p.out + off_o, p.out_dtype, acc);
    else reinterpret_cast<typename R::P *>(p.partial)[o * p.split + s] = to_storage<R::ACC>(acc);
  }
}

// The common fused row reduction - one reduced dim along which both inputs are contiguous and
// read in whole 16-byte vectors, at most one kept dim (along which either input may be
// broadcast), a wavefront or a workgroup per output or per split of it, everything below 2^31 -
// without the index decomposition and the 64-bit bookkeeping of the general kernel, and with
// every load a single 16-byte piece per lane, so that a wavefront's instruction covers whole
// lines of its input (the access shape streaming loads need; the general kernel reads 64 bytes
// per lane and input when the intermediate type is bool).
template <class G, int OP, bool NT>
OCN_DEV typename FusedFold<G, OP>::A fred_lean_fold(const char *pa, const char *pb, uint32_t t0, uint32_t t1,
                                                    uint32_t lane, uint32_t lanes) {
  using F = FusedFold<G, OP>;
  using A = typename F::A;
  using SAt = typename G::SAt;
  using SBt = typename G::SBt;
  static_assert(sizeof(SAt) == sizeof(SBt) && sizeof(SAt) <= 16, "equal input widths of at most 16 bytes");
  constexpr int V = 16 / (int)sizeof(SAt);
  constexpr int U = 2;
  A acc[U];
#pragma unroll
  for (int u = 0; u < U; ++u) acc[u] = F::R::identity();
  uint32_t t = t0 + lane;
  for (; t + (U - 1) * lanes < t1; t += U * lanes) {
    Pack<SAt, V> va[U];
    Pack<SBt, V> vb[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      load_vec<SAt, V, NT>(pa + (uint64_t)(t + u * lanes) * 16u, va[u]);
      load_vec<SBt, V, NT>(pb + (uint64_t)(t + u * lanes) * 16u, vb[u]);
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int i = 0; i < V; ++i) acc[u] = F::add(acc[u], va[u].v[i], vb[u].v[i]);
  }
  for (; t < t1; t += lanes) {
    Pack<SAt, V> va;
    Pack<SBt, V> vb;
    load_vec<SAt, V, NT>(pa + (uint64_t)t * 16u, va);
    load_vec<SBt, V, NT>(pb + (uint64_t)t * 16u, vb);
#pragma unroll
    for (int i = 0; i < V; ++i) acc[0] = F::add(acc[0], va.v[i], vb.v[i]);
  }
  A r = acc[0];
#pragma unroll
  for (int u = 1; u < U; ++u) r = F::R::combine(r, acc[u]);
  return r;
}

template <class G, int OP> __global__ __launch_bounds__(kBlock) OCN_ROWS_OCC void fred_rows_lean_kernel(const RedLeanArgs p) {
  using F = FusedFold<G, OP>;
  using R = typename F::R;
  using A = typename F::A;
  __shared__ A lds[kBlock / kWave];
  const uint32_t tid = threadIdx.x, lane_in_wave = tid & (kWave - 1), wave = tid / kWave;
  const bool per_block = p.group == kBlock;
  const uint32_t gidx = per_block ? blockIdx.x : blockIdx.x * (kBlock / kWave) + wave;
  const bool active = gidx < p.nout * p.split;
  const uint32_t lane = per_block ? tid : lane_in_wave;
  uint32_t o = gidx, sp = 0, t0 = 0, t1 = p.nvec;
  A acc = R::identity();
  if (active) {
    if (p.split != 1) {
      o = gidx / p.split;
      sp = gidx - o * p.split;
      t0 = sp * p.chunk;
      t1 = t0 + p.chunk < p.nvec ? t0 + p.chunk : p.nvec;
    }
    const char *pa = p.a + (int64_t)o * p.ksa;
    const char *pb = p.b + (int64_t)o * p.ksb;
    const uint32_t lanes = per_block ? kBlock : kWave;
    if (p.nt_load) acc = fred_lean_fold<G, OP, true>(pa, pb, t0, t1, lane, lanes);
    else acc = fred_lean_fold<G, OP, false>(pa, pb, t0, t1, lane, lanes);
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
    if (p.split == 1) store_result<A>(p.out + (int64_t)o * p.kso, p.out_dtype, acc);
    else reinterpret_cast<typename R::P *>(p.partial)[(uint64_t)o * p.split + sp] = to_storage<R::ACC>(acc);
  }
}

// Rows of at most one vector per lane of their group, a single reduced dim, no split: the same
// groups, loads and fold order as fred_rows_kernel without its loops and 64-bit bookkeeping.
template <class G, int OP, int V>
OCN_DEV typename FusedFold<G, OP>::A fred_short_row(const RedArgs &p, const char *pa, const char *pb, uint32_t lane) {
  using F = FusedFold<G, OP>;
  using A = typename F::A;
  using SAt = typename G::SAt;
  using SBt = typename G::SBt;
  A acc = F::R::identity();
  if (lane < (uint32_t)p.nvec) {
    const bool abc = p.a_bcast, bbc = p.b_bcast;
    const uint32_t e0 = lane * V;
    const char *qa = pa + (abc ? 0 : (int64_t)e0 * (int64_t)sizeof(SAt));
    const char *qb = pb + (bbc ? 0 : (int64_t)e0 * (int64_t)sizeof(SBt));
    const uint32_t left = (uint32_t)p.n0 - e0;
    if (left >= (uint32_t)V) {
      Pack<SAt, V> va;
      Pack<SBt, V> vb;
      fused_load<SAt, V>(qa, abc, va);
      fused_load<SBt, V>(qb, bbc, vb);
#pragma unroll
      for (int i = 0; i < V; ++i) acc = F::add(acc, va.v[i], vb.v[i]);
    } else {
#pragma unroll
      for (int i = 0; i < V; ++i)
        if (i < (int)left)
          acc = F::add(acc, reinterpret_cast<const SAt *>(qa)[abc ? 0 : i], reinterpret_cast<const SBt *>(qb)[bbc ? 0 : i]);
    }
  }
  return acc;
}

template <class G, int OP> __global__ __launch_bounds__(kBlock) void fred_rows_short_kernel(const RedArgs p) {
  using F = FusedFold<G, OP>;
  using R = typename F::R;
  using A = typename F::A;
  const uint32_t width = (uint32_t)p.group;
  const uint32_t gl = blockIdx.x * kBlock + threadIdx.x;
  const uint32_t o = gl >> (__ffs(p.group) - 1), lane = gl & (width - 1);
  const bool active = o < (uint32_t)p.nout;
  A acc = R::identity();
  int64_t off_o = 0;
  if (active) {
    int64_t off_a, off_b;
    kept_offsets2(p, o, off_a, off_b, off_o);
    if (p.vec > 1) acc = fred_short_row<G, OP, G::V>(p, p.a + off_a, p.b + off_b, lane);
    else acc = fred_short_row<G, OP, 1>(p, p.a + off_a, p.b + off_b, lane);
  }
  acc = group_fold<R>(acc, (int)width);
  if (active && lane == 0) store_result<A>(p.out + off_o, p.out_dtype, acc);
}

// ---------------------------------------------------------------------------------------
// cols: a kept axis is the fastest of the inputs; lanes own output columns
// ---------------------------------------------------------------------------------------

// NT: both inputs are read with streaming loads (one 16-byte piece per lane each).  SINGLE:
// one reduced dim, so that row r lies r strides further on (no index decomposition).
template <class G, int OP, int V, bool NT, bool SINGLE>
OCN_DEV void fred_cols_body(const RedArgs &p, typename FusedFold<G, OP>::A *lds) {
  using F = FusedFold<G, OP>;
  using R = typename F::R;
  using A = typename F::A;
  using SAt = typename G::SAt;
  using SBt = typename G::SBt;
  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wave = tid / kWave;
  const int NW = (int)blockDim.x / kWave;
  const bool abc = p.a_bcast, bbc = p.b_bcast;

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

  int64_t off_a = abc ? 0 : col0 * (int64_t)sizeof(SAt), off_b = bbc ? 0 : col0 * (int64_t)sizeof(SBt);
  int64_t off_o = col0 * p.kso[0];
  {
    uint32_t o = other;
#pragma unroll
    for (int k = 1; k < kMaxDims; ++k) {
      if (k < p.nkept) {
        const uint32_t q = (k == p.nkept - 1) ? 0u : rfastdiv(o, p.kdiv[k]);
        const uint32_t i = o - q * p.kdiv[k].d;
        o = q;
        off_a += (int64_t)i * p.ksa[k];
        off_b += (int64_t)i * p.ksb[k];
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
  constexpr int U = 2;
  // each wavefront takes one contiguous run of the workgroup's rows, RPW rows at a time (as in
  // red_cols_kernel: rows dealt out in turn measured 10 % slower there)
  const int RS = RPW;
  const int64_t per_wave = (((r1 - r0) + NW - 1) / NW + RPW - 1) / RPW * RPW;
  const int64_t w0 = r0 + (int64_t)wave * per_wave;
  if (w0 + per_wave < r1) r1 = w0 + per_wave;
  int64_t r = w0 + lr;
  auto row_offsets = [&](int64_t rr, int64_t &oa, int64_t &ob) {
    if constexpr (SINGLE) {
      oa = rr * p.rsa[0];
      ob = rr * p.rsb[0];
    } else {
      reduced_offset2(p, (uint32_t)rr, 0, oa, ob);
    }
  };
  if (ncol == V) {
    for (; r + (int64_t)(U - 1) * RS < r1; r += RS * U) {
      Pack<SAt, V> va[U];
      Pack<SBt, V> vb[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        int64_t oa, ob;
        row_offsets(r + (int64_t)u * RS, oa, ob);
        fused_load<SAt, V, NT>(p.a + off_a + oa, abc, va[u]);
        fused_load<SBt, V, NT>(p.b + off_b + ob, bbc, vb[u]);
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] = F::add(acc[i], va[u].v[i], vb[u].v[i]);
    }
  }
  if (ncol > 0) {  // remaining rows, and the ragged last column block
    for (; r < r1; r += RS) {
      int64_t oa, ob;
      row_offsets(r, oa, ob);
      const char *qa = p.a + off_a + oa, *qb = p.b + off_b + ob;
#pragma unroll
      for (int i = 0; i < V; ++i)
        if (i < ncol)
          acc[i] = F::add(acc[i], reinterpret_cast<const SAt *>(qa)[abc ? 0 : i],
                          reinterpret_cast<const SBt *>(qb)[bbc ? 0 : i]);
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
  // combine the wavefronts: CH columns per barrier, wavefront c folds column c (as red_cols_kernel)
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
        store_result<A>(p.out + off_o + (int64_t)i * p.kso[0], p.out_dtype, v);
      } else {
        const int64_t olin = (int64_t)other * p.nc + col0 + i;
        reinterpret_cast<typename R::P *>(p.partial)[(int64_t)s * p.nout + olin] = to_storage<R::ACC>(v);
      }
    }
    if (i0 + CH < V) __syncthreads();
  }
}

template <class G, int OP> __global__ __launch_bounds__(kColsMaxWaves * kWave) void fred_cols_kernel(const RedArgs p) {
  using A = typename FusedFold<G, OP>::A;
  extern __shared__ __align__(16) unsigned char fred_cols_lds_raw[];
  A *lds = reinterpret_cast<A *>(fred_cols_lds_raw);
  if (p.vec > 1 && p.nred == 1) {
    if (p.nt_load) fred_cols_body<G, OP, G::V, true, true>(p, lds);
    else fred_cols_body<G, OP, G::V, false, true>(p, lds);
  } else if (p.vec > 1) {
    fred_cols_body<G, OP, G::V, false, false>(p, lds);
  } else {
    fred_cols_body<G, OP, 1, false, false>(p, lds);
  }
}

// ---------------------------------------------------------------------------------------
// generic: any layout, one output per lane
// ---------------------------------------------------------------------------------------

template <class G, int OP> __global__ __launch_bounds__(kBlock) void fred_generic_kernel(const RedArgs p) {
  using F = FusedFold<G, OP>;
  using A = typename F::A;
  using SAt = typename G::SAt;
  using SBt = typename G::SBt;
  // the grid is capped (a launch cannot have 2^32 lanes): more outputs than lanes loop
  for (int64_t o = (int64_t)blockIdx.x * kBlock + threadIdx.x; o < p.nout; o += (int64_t)gridDim.x * kBlock) {
  int64_t off_a = 0, off_b = 0, off_o = 0, t = o;
#pragma unroll
  for (int k = 0; k < kMaxDims; ++k) {
    if (k < p.nkept) {
      const int64_t n = p.ksize[k];
      const int64_t q = t / n;
      const int64_t i = t - q * n;
      t = q;
      off_a += i * p.ksa[k];
      off_b += i * p.ksb[k];
      off_o += i * p.kso[k];
    }
  }
  A acc = F::R::identity();
  for (int64_t r = 0; r < p.nredtot; ++r) {
    int64_t oa = 0, ob = 0, q = r;
#pragma unroll
    for (int k = 0; k < kMaxDims; ++k) {
      if (k < p.nred) {
        const int64_t n = p.rsize[k];
        const int64_t qq = q / n;
        oa += (q - qq * n) * p.rsa[k];
        ob += (q - qq * n) * p.rsb[k];
        q = qq;
      }
    }
    acc = F::add(acc, *reinterpret_cast<const SAt *>(p.a + off_a + oa), *reinterpret_cast<const SBt *>(p.b + off_b + ob));
  }
  store_result<A>(p.out + off_o, p.out_dtype, acc);
  }
}

#endif  // __HIPCC__

}  // namespace ocn
