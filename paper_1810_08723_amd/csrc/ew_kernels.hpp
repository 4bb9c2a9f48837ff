// Elementwise kernels of the tensor engine for gfx950 (wave64, 256-lane workgroups).
//
// Three kernels cover every canonical plan the host planner can produce:
//   ew_rows_kernel    every operand is contiguous (or broadcast) along the innermost canonical
//                     dimension: 128-bit lane accesses, several vectors in flight per lane.
//   ew_tiled_kernel   operands disagree on their fastest axis: a power-of-two tile spanning
//                     those axes is staged through LDS so that every operand is read and
//                     written along its own fastest axis.  Without staging it is the plain
//                     strided kernel for specialised dtypes.
//   ew_interp_kernel  any dtype combination, conversions chosen by runtime switches.
// The operations follow sections 3.2 and 3.2.1 of the paper (elementwise arithmetic with
// implicit type casting fused into the kernel: no intermediate tensors).
#pragma once

#include "dev_types.hpp"
#include "planner.hpp"
#include "sigs.hpp"

namespace ocn {

// ---------------------------------------------------------------------------------------
// kernel arguments (plain data, passed by value)
// ---------------------------------------------------------------------------------------

struct RowsArgs {
  char *out;
  const char *a, *b;
  int64_t so[kMaxDims - 1], sa[kMaxDims - 1], sb[kMaxDims - 1];  // outer strides, fastest outer first
  FastDiv odiv[kMaxDims - 1];                                    // outer sizes, same order
  int32_t nouter;
  FastDiv vpr_div;   // vectors per row
  int64_t inner;     // elements per row
  int64_t nvec;      // vectors in total
  int32_t a_bcast, b_bcast;
};

struct TileOrder {
  int8_t width[kMaxDims];          // log2 tile extent of the k-th enumerated dim
  int8_t dim[kMaxDims];            // which canonical dim that is
  int8_t lds_shift[kMaxDims];      // bit position of that dim in the LDS slot number
  int64_t stride[3][kMaxDims];     // byte stride of that dim for out / a / b
};

struct TiledArgs {
  char *out;
  const char *a, *b;
  int32_t ndim, nord, tile_bits;
  int64_t size[kMaxDims];
  int64_t so[kMaxDims], sa[kMaxDims], sb[kMaxDims];
  int32_t tl[kMaxDims];
  FastDiv ntdiv[kMaxDims];
  int32_t stage_a, stage_b, pad_a, pad_b;
  uint32_t lds_off_b;              // byte offset of b's staging area in dynamic LDS
  TileOrder ord[3];                // enumeration orders: out's, a's, b's
};

struct InterpArgs {
  char *out;
  const char *a, *b;
  int32_t ndim, nin, op, T, dt_a, dt_b, dt_o;
  int64_t size[kMaxDims], so[kMaxDims], sa[kMaxDims], sb[kMaxDims];
  int64_t numel;
};

#if defined(__HIPCC__)

OCN_DEV uint32_t fastdiv(uint32_t n, const FastDiv &f) { return (__umulhi(n, f.m) + n) >> f.s; }

// ---------------------------------------------------------------------------------------
// raw vector access
// ---------------------------------------------------------------------------------------

template <class S, int V> struct alignas(sizeof(S) * V >= 16 ? 16 : sizeof(S) * V) Pack {
  S v[V];
};

template <class S, int V> OCN_DEV void load_pack(const char *p, Pack<S, V> &dst) {
  constexpr int B = sizeof(S) * V;
  if constexpr (B >= 16) {
    using Q = uint32_t __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int i = 0; i < B / 16; ++i) reinterpret_cast<Q *>(&dst)[i] = reinterpret_cast<const Q *>(p)[i];
  } else if constexpr (B == 8) {
    using D = uint32_t __attribute__((ext_vector_type(2)));
    *reinterpret_cast<D *>(&dst) = *reinterpret_cast<const D *>(p);
  } else if constexpr (B == 4) {
    *reinterpret_cast<uint32_t *>(&dst) = *reinterpret_cast<const uint32_t *>(p);
  } else if constexpr (B == 2) {
    *reinterpret_cast<uint16_t *>(&dst) = *reinterpret_cast<const uint16_t *>(p);
  } else {
    *reinterpret_cast<uint8_t *>(&dst) = *reinterpret_cast<const uint8_t *>(p);
  }
}

template <class S, int V> OCN_DEV void store_pack(char *p, const Pack<S, V> &src) {
  constexpr int B = sizeof(S) * V;
  if constexpr (B >= 16) {
    using Q = uint32_t __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int i = 0; i < B / 16; ++i) reinterpret_cast<Q *>(p)[i] = reinterpret_cast<const Q *>(&src)[i];
  } else if constexpr (B == 8) {
    using D = uint32_t __attribute__((ext_vector_type(2)));
    *reinterpret_cast<D *>(p) = *reinterpret_cast<const D *>(&src);
  } else if constexpr (B == 4) {
    *reinterpret_cast<uint32_t *>(p) = *reinterpret_cast<const uint32_t *>(&src);
  } else if constexpr (B == 2) {
    *reinterpret_cast<uint16_t *>(p) = *reinterpret_cast<const uint16_t *>(&src);
  } else {
    *reinterpret_cast<uint8_t *>(p) = *reinterpret_cast<const uint8_t *>(&src);
  }
}

// ---------------------------------------------------------------------------------------
// one element: load-convert, operate, convert-store
// ---------------------------------------------------------------------------------------

template <int OP, int SA, int SB, int SO, int NIN> struct Sig {
  // compute type: inputs of a specialised comparison have equal types, so T is that type
  static constexpr int T = NIN == 2 ? (is_logical(OP) ? (int)DT_BOOL : is_compare(OP) ? SA : SO)
                                    : unary_compute_dtype(OP, SO);
  using SAt = storage_t<SA>;
  using SBt = storage_t<SB>;
  using SOt = storage_t<SO>;
  static constexpr int ES_MIN = imin(imin((int)sizeof(SAt), (int)sizeof(SOt)), NIN == 2 ? (int)sizeof(SBt) : 16);
  static constexpr int ES_MAX = imax(imax((int)sizeof(SAt), (int)sizeof(SOt)), NIN == 2 ? (int)sizeof(SBt) : 1);
  static constexpr bool NIN2 = NIN == 2;
  static constexpr int V = rows_vec(ES_MIN, ES_MAX);
  static constexpr int U = rows_unroll(V, ES_MAX);

  OCN_DEV static SOt eval(SAt a, SBt b) {
    reg_t<T> ra = convert<T>(from_storage<SA>(a));
    if constexpr (NIN == 2) {
      reg_t<T> rb = convert<T>(from_storage<SB>(b));
      auto r = apply_binary<OP, T>(ra, rb);
      return to_storage<SO>(convert<SO>(r));
    } else {
      auto r = apply_unary<OP, T>(ra);
      return to_storage<SO>(convert<SO>(r));
    }
  }
};

// ---------------------------------------------------------------------------------------
// rows kernel
// ---------------------------------------------------------------------------------------

template <class G> __global__ __launch_bounds__(kBlock) void ew_rows_kernel(const RowsArgs p) {
  constexpr int V = G::V, U = G::U;
  using SAt = typename G::SAt;
  using SBt = typename G::SBt;
  using SOt = typename G::SOt;
  constexpr bool BIN = G::NIN2;

  const int64_t g0 = (int64_t)blockIdx.x * (kBlock * U) + threadIdx.x;
  Pack<SAt, V> va[U];
  Pack<SBt, V> vb[U];
  int64_t oo[U];
  int nvalid[U];

#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int64_t g = g0 + (int64_t)u * kBlock;
    nvalid[u] = 0;
    oo[u] = 0;
    if (g < p.nvec) {
      int64_t col, off_o = 0, off_a = 0, off_b = 0;
      if (p.nouter == 0) {
        col = g;
      } else {
        uint32_t row = fastdiv((uint32_t)g, p.vpr_div);
        col = (uint32_t)g - row * p.vpr_div.d;
#pragma unroll
        for (int k = 0; k < kMaxDims - 1; ++k) {
          if (k < p.nouter) {
            uint32_t q = (k == p.nouter - 1) ? 0u : fastdiv(row, p.odiv[k]);
            uint32_t i = row - q * p.odiv[k].d;
            row = q;
            off_o += (int64_t)i * p.so[k];
            off_a += (int64_t)i * p.sa[k];
            if constexpr (BIN) off_b += (int64_t)i * p.sb[k];
          }
        }
      }
      const int64_t e0 = col * V;
      const int64_t left = p.inner - e0;
      const int n = left >= V ? V : (int)left;
      nvalid[u] = n;
      oo[u] = off_o + e0 * (int64_t)sizeof(SOt);
      const char *pa = p.a + off_a + (p.a_bcast ? 0 : e0 * (int64_t)sizeof(SAt));
      const char *pb = nullptr;
      if constexpr (BIN) pb = p.b + off_b + (p.b_bcast ? 0 : e0 * (int64_t)sizeof(SBt));
      if (n == V) {
        if (p.a_bcast) {
          SAt s = *reinterpret_cast<const SAt *>(pa);
#pragma unroll
          for (int i = 0; i < V; ++i) va[u].v[i] = s;
        } else {
          load_pack<SAt, V>(pa, va[u]);
        }
        if constexpr (BIN) {
          if (p.b_bcast) {
            SBt s = *reinterpret_cast<const SBt *>(pb);
#pragma unroll
            for (int i = 0; i < V; ++i) vb[u].v[i] = s;
          } else {
            load_pack<SBt, V>(pb, vb[u]);
          }
        }
      } else {
#pragma unroll
        for (int i = 0; i < V; ++i) {
          if (i < n) {
            va[u].v[i] = reinterpret_cast<const SAt *>(pa)[p.a_bcast ? 0 : i];
            if constexpr (BIN) vb[u].v[i] = reinterpret_cast<const SBt *>(pb)[p.b_bcast ? 0 : i];
          }
        }
      }
    }
  }

#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int n = nvalid[u];
    if (n == 0) continue;
    Pack<SOt, V> r;
#pragma unroll
    for (int i = 0; i < V; ++i) {
      if constexpr (BIN) r.v[i] = G::eval(va[u].v[i], vb[u].v[i]);
      else r.v[i] = G::eval(va[u].v[i], SBt{});
    }
    char *po = p.out + oo[u];
    if (n == V) {
      store_pack<SOt, V>(po, r);
    } else {
#pragma unroll
      for (int i = 0; i < V; ++i)
        if (i < n) reinterpret_cast<SOt *>(po)[i] = r.v[i];
    }
  }
}

// ---------------------------------------------------------------------------------------
// tiled kernel
// ---------------------------------------------------------------------------------------

// lane part and block-uniform part of a tile-local enumeration index e = lane + (j << 8):
// every tile extent is a power of two, so the bits of e map to coordinates independently
struct TilePos {
  int64_t off[3];   // byte offsets for out / a / b
  uint32_t slot;    // LDS slot (position in out's enumeration order)
};

template <int NOPS> OCN_DEV TilePos tile_pos(const TileOrder &o, int nord, uint32_t e) {
  TilePos r;
  r.off[0] = r.off[1] = r.off[2] = 0;
  r.slot = 0;
  uint32_t shift = 0;
#pragma unroll
  for (int k = 0; k < kMaxDims; ++k) {
    if (k < nord) {
      const uint32_t w = o.width[k];
      const uint32_t c = (e >> shift) & ((1u << w) - 1u);
      shift += w;
#pragma unroll
      for (int x = 0; x < NOPS; ++x) r.off[x] += (int64_t)c * o.stride[x][k];
      r.slot += c << o.lds_shift[k];
    }
  }
  return r;
}

// is element e of the enumeration inside the (possibly clipped) tile?
OCN_DEV bool tile_inside(const TileOrder &o, int nord, uint32_t e, const uint32_t *lim) {
  bool ok = true;
  uint32_t shift = 0;
#pragma unroll
  for (int k = 0; k < kMaxDims; ++k) {
    if (k < nord) {
      const uint32_t w = o.width[k];
      const uint32_t c = (e >> shift) & ((1u << w) - 1u);
      shift += w;
      ok = ok && (c < lim[k]);
    }
  }
  return ok;
}

template <class S>
OCN_DEV void stage_operand(const TiledArgs &p, const TileOrder &ord, int which, const char *base,
                           S *lds, int pad, bool full, const uint32_t (*lim)[kMaxDims], uint32_t tile_elems) {
  constexpr int J = 4;  // loads in flight per lane
  const uint32_t tid = threadIdx.x;
  const TilePos lo = tile_pos<3>(ord, p.nord, tid);
  for (uint32_t j0 = 0; j0 < tile_elems; j0 += kBlock * J) {
    S vals[J];
    uint32_t slots[J];
    bool ok[J];
#pragma unroll
    for (int j = 0; j < J; ++j) {
      const uint32_t ehi = j0 + j * kBlock;
      const uint32_t e = ehi + tid;
      ok[j] = e < tile_elems && (full || tile_inside(ord, p.nord, e, lim[which]));
      const TilePos hi = tile_pos<3>(ord, p.nord, ehi);
      slots[j] = lo.slot + hi.slot;
      if (ok[j]) vals[j] = *reinterpret_cast<const S *>(base + lo.off[which] + hi.off[which]);
    }
#pragma unroll
    for (int j = 0; j < J; ++j)
      if (ok[j]) lds[slots[j] + (slots[j] >> pad)] = vals[j];
  }
}

extern __shared__ uint4 ocn_lds_raw[];

template <class G> __global__ __launch_bounds__(kBlock) void ew_tiled_kernel(const TiledArgs p) {
  using SAt = typename G::SAt;
  using SBt = typename G::SBt;
  using SOt = typename G::SOt;
  constexpr bool BIN = G::NIN2;
  constexpr int J = 4;

  // tile origin, clipped extents (block-uniform)
  uint32_t t = blockIdx.x;
  int64_t base_o = 0, base_a = 0, base_b = 0;
  uint32_t lim_dim[kMaxDims];
  bool full = true;
#pragma unroll
  for (int d = kMaxDims - 1; d >= 0; --d) {
    lim_dim[d] = 1;
    if (d < p.ndim) {
      const uint32_t q = (d == 0) ? 0u : fastdiv(t, p.ntdiv[d]);
      const uint32_t tc = t - q * p.ntdiv[d].d;
      t = q;
      const int64_t i0 = (int64_t)tc << p.tl[d];
      const int64_t ext = (int64_t)1 << p.tl[d];
      const int64_t rem = p.size[d] - i0;
      lim_dim[d] = (uint32_t)(rem < ext ? rem : ext);
      full = full && rem >= ext;
      base_o += i0 * p.so[d];
      base_a += i0 * p.sa[d];
      if constexpr (BIN) base_b += i0 * p.sb[d];
    }
  }
  // clipped extents in each enumeration order
  uint32_t lim[3][kMaxDims];
#pragma unroll
  for (int x = 0; x < 3; ++x)
#pragma unroll
    for (int k = 0; k < kMaxDims; ++k) {
      lim[x][k] = 1;
      if (k < p.nord) {
        const int d = p.ord[x].dim[k];
        uint32_t l = 1;
#pragma unroll
        for (int dd = 0; dd < kMaxDims; ++dd)
          if (dd == d) l = lim_dim[dd];
        lim[x][k] = l;
      }
    }

  const uint32_t tile_elems = 1u << p.tile_bits;
  SAt *lds_a = reinterpret_cast<SAt *>(ocn_lds_raw);
  SBt *lds_b = reinterpret_cast<SBt *>(reinterpret_cast<char *>(ocn_lds_raw) + p.lds_off_b);

  if (p.stage_a) stage_operand<SAt>(p, p.ord[1], 1, p.a + base_a, lds_a, p.pad_a, full, lim, tile_elems);
  if constexpr (BIN)
    if (p.stage_b) stage_operand<SBt>(p, p.ord[2], 2, p.b + base_b, lds_b, p.pad_b, full, lim, tile_elems);
  if (p.stage_a || p.stage_b) __syncthreads();

  // compute phase, in the output's enumeration order (LDS slot == enumeration index)
  const uint32_t tid = threadIdx.x;
  const TileOrder &oo = p.ord[0];
  const TilePos lo = tile_pos<3>(oo, p.nord, tid);
  char *out = p.out + base_o;
  const char *pa = p.a + base_a;
  const char *pb = BIN ? p.b + base_b : nullptr;
  for (uint32_t j0 = 0; j0 < tile_elems; j0 += kBlock * J) {
    SAt av[J];
    SBt bv[J];
    int64_t offo[J];
    bool ok[J];
#pragma unroll
    for (int j = 0; j < J; ++j) {
      const uint32_t ehi = j0 + j * kBlock;
      const uint32_t e = ehi + tid;
      ok[j] = e < tile_elems && (full || tile_inside(oo, p.nord, e, lim[0]));
      const TilePos hi = tile_pos<3>(oo, p.nord, ehi);
      offo[j] = lo.off[0] + hi.off[0];
      if (ok[j]) {
        if (p.stage_a) av[j] = lds_a[e + (e >> p.pad_a)];
        else av[j] = *reinterpret_cast<const SAt *>(pa + lo.off[1] + hi.off[1]);
        if constexpr (BIN) {
          if (p.stage_b) bv[j] = lds_b[e + (e >> p.pad_b)];
          else bv[j] = *reinterpret_cast<const SBt *>(pb + lo.off[2] + hi.off[2]);
        }
      }
    }
#pragma unroll
    for (int j = 0; j < J; ++j) {
      if (ok[j]) {
        SOt r;
        if constexpr (BIN) r = G::eval(av[j], bv[j]);
        else r = G::eval(av[j], SBt{});
        *reinterpret_cast<SOt *>(out + offo[j]) = r;
      }
    }
  }
}

#endif  // __HIPCC__

}  // namespace ocn
