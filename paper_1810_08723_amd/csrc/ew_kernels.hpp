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
  int32_t nt_store;  // stream the output past the caches
  int32_t nt_a, nt_b; // read that input with streaming (non-temporal) loads
  int32_t swap;       // operands stored in the other byte order: bit 0 a, bit 1 b, bit 2 out
};

constexpr int kMaxTilePasses = 16;  // a tile holds at most 4096 elements = 16 passes of 256 lanes

// One enumeration order of a tile's elements (fastest dim of some operand first).
struct TileOrder {
  int8_t nord;                     // tiled dims
  int8_t vecw;                     // log2 of the vector length along the first enumerated dim
  int8_t width[kMaxDims];          // log2 tile extent of the k-th enumerated dim
  int8_t dim[kMaxDims];            // which canonical dim that is
  int8_t lds_shift[kMaxDims];      // bit position of that dim in the LDS slot number
  int32_t niter;                   // passes of 256 lanes that cover the tile
  int64_t stride[3][kMaxDims];     // byte stride of that dim for out / a / b
  int64_t hi_off[3][kMaxTilePasses];  // byte offsets contributed by the pass number
  uint32_t hi_slot[kMaxTilePasses];   // LDS slot contributed by the pass number
};

// slot -> physical LDS element: slot ^ (((slot >> src) & mask) << dst)
struct TileSwizzle {
  uint32_t src, mask, dst;
};

struct TiledArgs {
  char *out;
  const char *a, *b;
  int32_t ndim, tile_bits;
  uint32_t total_tiles;
  int64_t size[kMaxDims];
  int64_t so[kMaxDims], sa[kMaxDims], sb[kMaxDims];
  int32_t tl[kMaxDims];
  FastDiv ntdiv[kMaxDims];
  int32_t stage_a, stage_b;
  int32_t nt_store;                // stream the output past the caches
  int32_t swap;                    // operands stored in the other byte order: bit 0 a, bit 1 b, bit 2 out
  uint32_t lds_off_b;              // byte offset of b's staging area in dynamic LDS
  TileSwizzle swz[2];              // for a, b
  TileOrder ord[3];                // enumeration orders: out's, a's, b's
};

// Arguments of the unclipped, all-vector form of the tiled kernel.  Everything that does not
// depend on the lane is tabulated by the host, and all offsets inside a tile are unsigned
// 32-bit, so that an access costs one scalar add (tile base + pass offset) and no vector
// address arithmetic.  LDS addresses are XORs of three host- or once-computed terms: the
// swizzle is linear over GF(2) and the lane, pass and element-in-vector parts of a slot number
// occupy disjoint bits, so swizzle(lane + pass + element) is the XOR of their swizzles.
constexpr int kFastLaneDims = 8;
struct FastOrder {
  int32_t nlane;                            // dims reached by the 8 lane bits
  int32_t niter;                            // passes of 256 lanes
  uint32_t shift[kFastLaneDims];            // bit field of the lane number holding dim k's index
  uint32_t mask[kFastLaneDims];
  uint32_t up[kFastLaneDims];               // left shift of the extracted index (vector length for k = 0)
  uint32_t slot_shift[kFastLaneDims];       // bit position of dim k in the LDS slot number
  uint32_t stride[3][kFastLaneDims];        // byte strides for out / a / b
  uint32_t hi_off[3][kMaxTilePasses];       // byte offsets contributed by the pass number
};
struct FastTiledArgs {
  char *out;
  const char *a, *b;
  int32_t ntd;                              // entries of the tile-number decomposition, fastest first
  int32_t stage_a, stage_b;
  int32_t nt_store;                         // stream the output past the caches
  int32_t swap;                             // operands stored in the other byte order: bit 0 a, bit 1 b, bit 2 out
  int32_t pair_log2;                        // groups of 1 << pair_log2 consecutive tiles share input lines
  int32_t nt_a, nt_b;                       // read that input with streaming loads (its runs inside a tile are whole lines)
  uint32_t lds_base[2];                     // byte offset of a's / b's staging area
  FastDiv ntdiv[kMaxDims + 1];              // (one more than dims: a dim's tile index may be split in two)
  int64_t step[3][kMaxDims + 1];            // bytes from one tile to the next along that dim
  TileSwizzle swz[2];
  uint32_t es_log2[2];
  uint32_t vc_log2;                         // log2 of the compute vector length
  FastOrder ord[3];
  uint32_t st_hi[2][kMaxTilePasses];        // staging writes: swizzled byte address from the pass number
  uint32_t st_el[2][16];                    // ... from the element number inside a vector
  uint32_t rd_hi[2][kMaxTilePasses];        // compute-phase reads: from the pass number
  uint32_t rd_ch[2][16];                    // ... from the 16-byte chunk inside a vector
};

struct InterpArgs {
  char *out;
  const char *a, *b;
  int32_t ndim, nin, op, T, dt_a, dt_b, dt_o;
  int64_t size[kMaxDims], so[kMaxDims], sa[kMaxDims], sb[kMaxDims];
  int64_t numel;
  int32_t idx32;              // fewer than 2^31 elements: 32-bit multiply-shift index arithmetic
  int32_t swap;               // operands stored in the other byte order: bit 0 a, bit 1 b, bit 2 out
  int32_t vec;                // 4: a lane takes four consecutive elements of the innermost dim (sizes, strides and
                              // numel then count groups of four); 1: one element
  int32_t inner_a, inner_b;   // vec == 4: the input is contiguous along the innermost dim (else broadcast there)
  FastDiv div[kMaxDims];
};

#if defined(__HIPCC__)

#define OCN_HDF __host__ __device__ __forceinline__

OCN_HDF uint32_t fastdiv(uint32_t n, const FastDiv &f) {
  return (uint32_t)((((uint64_t)n * f.m) >> 32) + n) >> f.s;
}

// ---------------------------------------------------------------------------------------
// raw vector access
// ---------------------------------------------------------------------------------------

template <class S, int V> struct alignas(sizeof(S) * V >= 16 ? 16 : sizeof(S) * V) Pack {
  S v[V];
};

#define OCN_KEEP_BRANCH() asm volatile("")
// `nt`: a streaming (non-temporal) load, for inputs too large to be found in a cache again
// (the hint is only ever set for a single piece of at most 16 bytes per lane).  The empty asm
// statements keep the two branches apart; merged, the hint would be dropped.
template <class S, int V> OCN_DEV void load_pack(const char *p, Pack<S, V> &dst, bool nt = false) {
  constexpr int B = sizeof(S) * V;
  if constexpr (B >= 16) {
    using Q = uint32_t __attribute__((ext_vector_type(4)));
    if (B == 16 && nt) {
      OCN_KEEP_BRANCH();
      reinterpret_cast<Q *>(&dst)[0] = __builtin_nontemporal_load(reinterpret_cast<const Q *>(p));
      OCN_KEEP_BRANCH();
    } else {
#pragma unroll
      for (int i = 0; i < B / 16; ++i) {
        reinterpret_cast<Q *>(&dst)[i] = reinterpret_cast<const Q *>(p)[i];
      }
    }
  } else if constexpr (B == 8) {
    using D = uint32_t __attribute__((ext_vector_type(2)));
    if (nt) {
      OCN_KEEP_BRANCH();
      *reinterpret_cast<D *>(&dst) = __builtin_nontemporal_load(reinterpret_cast<const D *>(p));
      OCN_KEEP_BRANCH();
    } else {
      *reinterpret_cast<D *>(&dst) = *reinterpret_cast<const D *>(p);
    }
  } else if constexpr (B == 4) {
    if (nt) {
      OCN_KEEP_BRANCH();
      *reinterpret_cast<uint32_t *>(&dst) = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(p));
      OCN_KEEP_BRANCH();
    } else {
      *reinterpret_cast<uint32_t *>(&dst) = *reinterpret_cast<const uint32_t *>(p);
    }
  } else if constexpr (B == 2) {
    *reinterpret_cast<uint16_t *>(&dst) = *reinterpret_cast<const uint16_t *>(p);
  } else {
    *reinterpret_cast<uint8_t *>(&dst) = *reinterpret_cast<const uint8_t *>(p);
  }
}

// `nt`: a streaming (non-temporal) store.  Outputs too large to stay in the Infinity Cache are
// written this way: an ordinary store leaves the lines dirty in that cache, and the next
// kernel then pays for writing them back while it reads (measured: up to a third of its time).
// (The empty asm statements fence the streaming branch: without them the compiler merges the
// two stores of an if/else into one and drops the hint.)
template <class S, int V> OCN_DEV void store_pack(char *p, const Pack<S, V> &src, bool nt = false) {
  constexpr int B = sizeof(S) * V;
  if constexpr (B >= 16) {
    using Q = uint32_t __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int i = 0; i < B / 16; ++i) {
      if (nt) {
        OCN_KEEP_BRANCH();
        __builtin_nontemporal_store(reinterpret_cast<const Q *>(&src)[i], reinterpret_cast<Q *>(p) + i);
        OCN_KEEP_BRANCH();
      } else {
        reinterpret_cast<Q *>(p)[i] = reinterpret_cast<const Q *>(&src)[i];
      }
    }
  } else if constexpr (B == 8) {
    using D = uint32_t __attribute__((ext_vector_type(2)));
    if (nt) {
      OCN_KEEP_BRANCH();
      __builtin_nontemporal_store(*reinterpret_cast<const D *>(&src), reinterpret_cast<D *>(p));
      OCN_KEEP_BRANCH();
    } else {
      *reinterpret_cast<D *>(p) = *reinterpret_cast<const D *>(&src);
    }
  } else if constexpr (B == 4) {
    if (nt) {
      OCN_KEEP_BRANCH();
      __builtin_nontemporal_store(*reinterpret_cast<const uint32_t *>(&src), reinterpret_cast<uint32_t *>(p));
      OCN_KEEP_BRANCH();
    } else {
      *reinterpret_cast<uint32_t *>(p) = *reinterpret_cast<const uint32_t *>(&src);
    }
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
                                    : unary_compute_dtype(OP, SA, SO);
  using SAt = storage_t<SA>;
  using SBt = storage_t<SB>;
  using SOt = storage_t<SO>;
  static constexpr int ES_MIN = imin(imin((int)sizeof(SAt), (int)sizeof(SOt)), NIN == 2 ? (int)sizeof(SBt) : 16);
  static constexpr int ES_MAX = imax(imax((int)sizeof(SAt), (int)sizeof(SOt)), NIN == 2 ? (int)sizeof(SBt) : 1);
  static constexpr bool NIN2 = NIN == 2;
  static constexpr int SA_DT = SA, SB_DT = SB, SO_DT = SO;
  static constexpr int V = rows_vec((int)sizeof(SOt), ES_MAX);
  static constexpr int U = rows_unroll(V, ES_MAX);
  static constexpr int VR = rows_stream_vec((int)sizeof(SOt), ES_MIN, ES_MAX);  // the rows kernel's vector
  static constexpr int UR = rows_stream_unroll(VR, ES_MIN);

  // operands stored in the other byte order: un-reverse inputs after the load, reverse the
  // result before the store (sw: bit 0 a, bit 1 b, bit 2 out; uniform over the launch)
  template <class PA, class PB> OCN_DEV static void order_inputs(int sw, PA &a, PB &b) {
    if (sw & 1) reverse_scalars<scalar_bytes(SA)>(a);
    if constexpr (NIN == 2) {
      if (sw & 2) reverse_scalars<scalar_bytes(SB)>(b);
    }
  }
  template <class PO> OCN_DEV static void order_output(int sw, PO &r) {
    if (sw & 4) reverse_scalars<scalar_bytes(SO)>(r);
  }

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

template <class G> OCN_DEV void rows_general(const RowsArgs &p) {
  constexpr int V = G::VR, U = G::UR;
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
          load_pack<SAt, V>(pa, va[u], p.nt_a != 0);
        }
        if constexpr (BIN) {
          if (p.b_bcast) {
            SBt s = *reinterpret_cast<const SBt *>(pb);
#pragma unroll
            for (int i = 0; i < V; ++i) vb[u].v[i] = s;
          } else {
            load_pack<SBt, V>(pb, vb[u], p.nt_b != 0);
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
    if (p.swap) G::order_inputs(p.swap, va[u], vb[u]);
#pragma unroll
    for (int i = 0; i < V; ++i) {
      if constexpr (BIN) r.v[i] = G::eval(va[u].v[i], vb[u].v[i]);
      else r.v[i] = G::eval(va[u].v[i], SBt{});
    }
    if (p.swap) G::order_output(p.swap, r);
    char *po = p.out + oo[u];
    if (n == V) {
      store_pack<SOt, V>(po, r, p.nt_store != 0);
    } else {
#pragma unroll
      for (int i = 0; i < V; ++i)
        if (i < n) reinterpret_cast<SOt *>(po)[i] = r.v[i];
    }
  }
}

// The common shapes - at most one outer dim, rows of whole vectors, fewer than 2^31 vectors -
// get a kernel of their own.  With one vector per lane a wavefront lives for one memory round
// trip, so what it executes before its first load is time during which it has nothing in
// flight: this kernel reads 72 bytes of arguments with two scalar loads (the general kernel's
// 340 bytes of strides and divisors arrive in eight loads that are all waited for), needs one
// division per vector and no per-element conditions, and issues every load of a lane before it
// waits for any (2^26 floats negated: 84.4 us in the general kernel's body for these shapes,
// a plain copy of the same size written for the purpose 80.7 us).
struct RowsSlimArgs {
  char *out;
  const char *a, *b;
  int64_t so, sa, sb;   // byte strides of the outer dim (zero and unused without one)
  uint32_t nvec;        // vectors in total
  FastDiv vpr_div;      // vectors per row
  uint32_t flags;       // kSlim* bits; operands in the other byte order in bits 8..10
};
enum : uint32_t { kSlimABcast = 1, kSlimBBcast = 2, kSlimNtA = 4, kSlimNtB = 8, kSlimNtStore = 16, kSlimSwapShift = 8 };
#ifndef OCN_SLIM_BLOCK
#define OCN_SLIM_BLOCK 64
#endif
constexpr int kSlimBlock = OCN_SLIM_BLOCK;

template <class G> __global__ __launch_bounds__(kSlimBlock) void ew_rows_slim_kernel(const RowsSlimArgs q) {
  constexpr int V = G::VR, U = G::UR;
  RowsSlimArgs p = q;
  OCN_ARGS_NOW("s"(p.out), "s"(p.a), "s"(p.b), "s"(p.so), "s"(p.sa), "s"(p.sb), "s"(p.nvec), "s"(p.vpr_div.d),
               "s"(p.vpr_div.m), "s"(p.vpr_div.s), "s"(p.flags));
  using SAt = typename G::SAt;
  using SBt = typename G::SBt;
  using SOt = typename G::SOt;
  constexpr bool BIN = G::NIN2;
  const uint32_t g0 = blockIdx.x * (uint32_t)(kSlimBlock * U) + threadIdx.x;
  const uint32_t flags = p.flags;
  Pack<SAt, V> va[U];
  Pack<SBt, V> vb[U];
  int64_t oo[U];
  // every load of the lane is issued before anything waits for one
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const uint32_t g = g0 + (uint32_t)u * kSlimBlock;
    oo[u] = 0;
    if (g < p.nvec) {
      const uint32_t row = fastdiv(g, p.vpr_div);
      const int64_t e0 = (int64_t)(g - row * p.vpr_div.d) * V;
      oo[u] = (int64_t)row * p.so + e0 * (int64_t)sizeof(SOt);
      const char *pa = p.a + (int64_t)row * p.sa;
      // (an operand broadcast along the row: its one element lands in the vector's first slot
      // and is spread out after the loads; a register of its own would have to be cleared on
      // the other path, which the compiler does behind a wait for the loads issued so far)
      if (flags & kSlimABcast) va[u].v[0] = *reinterpret_cast<const SAt *>(pa);
      else load_pack<SAt, V>(pa + e0 * (int64_t)sizeof(SAt), va[u], (flags & kSlimNtA) != 0);
      if constexpr (BIN) {
        const char *pb = p.b + (int64_t)row * p.sb;
        if (flags & kSlimBBcast) vb[u].v[0] = *reinterpret_cast<const SBt *>(pb);
        else load_pack<SBt, V>(pb + e0 * (int64_t)sizeof(SBt), vb[u], (flags & kSlimNtB) != 0);
      }
    }
  }
  const int swap = (int)(flags >> kSlimSwapShift);
#pragma unroll
  for (int u = 0; u < U; ++u) {
    if (g0 + (uint32_t)u * kSlimBlock < p.nvec) {
      if (flags & kSlimABcast) {
#pragma unroll
        for (int i = 1; i < V; ++i) va[u].v[i] = va[u].v[0];
      }
      if constexpr (BIN) {
        if (flags & kSlimBBcast) {
#pragma unroll
          for (int i = 1; i < V; ++i) vb[u].v[i] = vb[u].v[0];
        }
      }
      Pack<SOt, V> r;
      if (swap) G::order_inputs(swap, va[u], vb[u]);
#pragma unroll
      for (int i = 0; i < V; ++i) {
        if constexpr (BIN) r.v[i] = G::eval(va[u].v[i], vb[u].v[i]);
        else r.v[i] = G::eval(va[u].v[i], SBt{});
      }
      if (swap) G::order_output(swap, r);
      store_pack<SOt, V>(p.out + oo[u], r, (flags & kSlimNtStore) != 0);
    }
  }
}

template <class G> __global__ __launch_bounds__(kBlock) void ew_rows_kernel(const RowsArgs p) {
  rows_general<G>(p);
}

// ---------------------------------------------------------------------------------------
// tiled kernel
// ---------------------------------------------------------------------------------------
//
// A workgroup owns one tile: a box of power-of-two extents over the canonical dims that are
// the fastest axis of the output or of an input.  The tile's elements are enumerated in up to
// three orders (the output's and each staged input's own fastest-axis-first order).  Because
// every extent is a power of two, an enumeration index e = lane + 256 * pass splits into a
// lane part (computed once per lane) and a pass part (the same for every lane and every
// workgroup, tabulated by the host), so the inner loops only add two offsets.
//
// Staged inputs are copied global -> LDS along their own fastest axis (128-bit loads when
// the layout allows), stored at slot = position in the OUTPUT's enumeration order, and read
// back along the output's fastest axis.  Slots are XOR-swizzled so that neither the
// column-wise writes nor the row-wise reads pile onto one LDS bank.

struct LanePos {
  int64_t off[3];   // byte offsets for out / a / b
  uint32_t slot;    // LDS slot (element position in the output's enumeration order)
};

// lane part of the position of vector number e (bits below 8 only) in enumeration order o
template <class O> OCN_HDF LanePos lane_pos(const O &o, uint32_t e) {
  LanePos r;
  r.off[0] = r.off[1] = r.off[2] = 0;
  r.slot = 0;
  uint32_t shift = 0;
#pragma unroll
  for (int k = 0; k < kMaxDims; ++k) {
    if (k < o.nord) {
      const uint32_t vw = k == 0 ? (uint32_t)o.vecw : 0u;
      const uint32_t w = (uint32_t)o.width[k] - vw;
      const uint32_t c = ((e >> shift) & ((1u << w) - 1u)) << vw;
      shift += w;
#pragma unroll
      for (int x = 0; x < 3; ++x) r.off[x] += (int64_t)c * o.stride[x][k];
      r.slot += c << o.lds_shift[k];
    }
  }
  return r;
}

// How many elements of vector number e lie inside a clipped tile (0 .. 1 << vecw).
template <class O> OCN_HDF int vec_inside(const O &o, uint32_t e, const uint32_t *lim_dim) {
  int n = 1 << o.vecw;
  uint32_t shift = 0;
#pragma unroll
  for (int k = 0; k < kMaxDims; ++k) {
    if (k < o.nord) {
      const uint32_t vw = k == 0 ? (uint32_t)o.vecw : 0u;
      const uint32_t w = (uint32_t)o.width[k] - vw;
      const uint32_t c = ((e >> shift) & ((1u << w) - 1u)) << vw;
      shift += w;
      uint32_t lim = 1;
#pragma unroll
      for (int dd = 0; dd < kMaxDims; ++dd)
        if (dd == o.dim[k]) lim = lim_dim[dd];
      if (k == 0) {
        const int left = (int)lim - (int)c;
        n = left < n ? left : n;
      } else if (c >= lim) {
        n = 0;
      }
    }
  }
  return n < 0 ? 0 : n;
}

OCN_HDF uint32_t swizzle(uint32_t slot, uint32_t src, uint32_t mask, uint32_t dst) {
  return slot ^ (((slot >> src) & mask) << dst);
}
OCN_HDF uint32_t swizzle(uint32_t slot, const TileSwizzle &z) { return swizzle(slot, z.src, z.mask, z.dst); }

extern __shared__ uint4 ocn_lds_raw[];

// The kernel reads its argument struct through the constant address space (the kernarg
// segment itself): indexing the per-pass tables with a runtime pass number then becomes a
// scalar load instead of forcing a private copy of the whole struct.
using KTiledArgs = const __attribute__((address_space(4))) TiledArgs;
using KTileOrder = const __attribute__((address_space(4))) TileOrder;

// global -> LDS copy of one staged input, enumerated in that input's own order
// FULL: the tile is not clipped and every lane has a whole vector in every pass, so the loop
// body carries no per-lane conditions at all.
template <class S, int V, int WHICH, bool FULL>
OCN_DEV void stage_operand(KTiledArgs &p, const char *base, S *lds,
                           const uint32_t *lim_dim, uint32_t nvec) {
  constexpr int J = V > 1 ? 2 : 4;  // vectors in flight per lane
  KTileOrder &o = p.ord[WHICH];
  const uint32_t zsrc = p.swz[WHICH - 1].src, zmask = p.swz[WHICH - 1].mask, zdst = p.swz[WHICH - 1].dst;
  const uint32_t tid = threadIdx.x;
  const LanePos lo = lane_pos(o, tid);
  const uint32_t step = 1u << o.lds_shift[0];  // slot distance between a vector's elements
  const int niter = o.niter;
  for (int j0 = 0; j0 < niter; j0 += J) {
    Pack<S, V> v[J];
    uint32_t slot[J];
    int nv[J];
#pragma unroll
    for (int j = 0; j < J; ++j) {
      const int jj = j0 + j;
      nv[j] = 0;
      if (jj < niter) {
        const uint32_t e = tid + (uint32_t)jj * kBlock;
        int n = V;
        if constexpr (!FULL) {
          n = e < nvec ? V : 0;
          if (n) n = vec_inside(o, e, lim_dim);
        }
        nv[j] = n;
        slot[j] = lo.slot + o.hi_slot[jj];
        const char *src = base + lo.off[WHICH] + o.hi_off[WHICH][jj];
        if (FULL || n == V) {
          load_pack<S, V>(src, v[j]);
        } else {
#pragma unroll
          for (int i = 0; i < V; ++i)
            if (i < n) v[j].v[i] = reinterpret_cast<const S *>(src)[i];
        }
      }
    }
#pragma unroll
    for (int j = 0; j < J; ++j) {
      if (j0 + j >= niter) break;  // uniform: the last batch of passes may be short
#pragma unroll
      for (int i = 0; i < V; ++i)
        if (FULL || i < nv[j]) lds[swizzle(slot[j] + (uint32_t)i * step, zsrc, zmask, zdst)] = v[j].v[i];
    }
  }
}

// read V consecutive slots of a staged operand (consecutive along the output's fastest axis)
template <class S, int V>
OCN_DEV void read_staged(const S *lds, uint32_t slot0, uint32_t zsrc, uint32_t zmask, uint32_t zdst, Pack<S, V> &dst) {
  constexpr int EPC = (16 / (int)sizeof(S)) < V ? (16 / (int)sizeof(S)) : V;  // elements per LDS access
  using Chunk = Pack<S, EPC>;
#pragma unroll
  for (int c = 0; c < V / EPC; ++c)
    *reinterpret_cast<Chunk *>(&dst.v[c * EPC]) =
        *reinterpret_cast<const Chunk *>(&lds[swizzle(slot0 + c * EPC, zsrc, zmask, zdst)]);
}

// V elements of a non-staged input along the output's fastest axis (byte stride s0 there)
template <class S, int V> OCN_DEV void read_direct(const char *src, int64_t s0, int n, Pack<S, V> &dst) {
  if (s0 == (int64_t)sizeof(S) && n == V) {
    load_pack<S, V>(src, dst);
  } else {
#pragma unroll
    for (int i = 0; i < V; ++i)
      if (i < n) dst.v[i] = *reinterpret_cast<const S *>(src + (int64_t)i * s0);
  }
}

template <class G, int V, bool FULL>
OCN_DEV void tiled_compute(KTiledArgs &p, char *out, const char *pa, const char *pb,
                           const typename G::SAt *lds_a, const typename G::SBt *lds_b,
                           const uint32_t *lim_dim, uint32_t nvec) {
  using SAt = typename G::SAt;
  using SBt = typename G::SBt;
  using SOt = typename G::SOt;
  constexpr bool BIN = G::NIN2;
  constexpr int J = V > 1 ? 2 : 4;
  KTileOrder &o = p.ord[0];
  const uint32_t tid = threadIdx.x;
  const LanePos lo = lane_pos(o, tid);
  const int64_t sa0 = o.stride[1][0], sb0 = o.stride[2][0];
  const bool stage_a = p.stage_a, stage_b = p.stage_b;
  const uint32_t asrc = p.swz[0].src, amask = p.swz[0].mask, adst = p.swz[0].dst;
  const uint32_t bsrc = p.swz[1].src, bmask = p.swz[1].mask, bdst = p.swz[1].dst;
  const int niter = o.niter;
  for (int j0 = 0; j0 < niter; j0 += J) {
    Pack<SAt, V> av[J];
    Pack<SBt, V> bv[J];
    int64_t offo[J];
    int nv[J];
#pragma unroll
    for (int j = 0; j < J; ++j) {
      const int jj = j0 + j;
      nv[j] = 0;
      if (jj < niter) {
        const uint32_t e = tid + (uint32_t)jj * kBlock;
        int n = V;
        if constexpr (!FULL) {
          n = e < nvec ? V : 0;
          if (n) n = vec_inside(o, e, lim_dim);
        }
        nv[j] = n;
        offo[j] = lo.off[0] + o.hi_off[0][jj];
        if (FULL || n) {
          const uint32_t slot0 = e * V;  // the output's order is the slot order
          if (stage_a) read_staged<SAt, V>(lds_a, slot0, asrc, amask, adst, av[j]);
          else read_direct<SAt, V>(pa + lo.off[1] + o.hi_off[1][jj], sa0, n, av[j]);
          if constexpr (BIN) {
            if (stage_b) read_staged<SBt, V>(lds_b, slot0, bsrc, bmask, bdst, bv[j]);
            else read_direct<SBt, V>(pb + lo.off[2] + o.hi_off[2][jj], sb0, n, bv[j]);
          }
        }
      }
    }
#pragma unroll
    for (int j = 0; j < J; ++j) {
      if (j0 + j >= niter) break;  // uniform: the last batch of passes may be short
      const int n = nv[j];
      if (!FULL && n == 0) continue;
      Pack<SOt, V> r;
      if (p.swap) G::order_inputs(p.swap, av[j], bv[j]);
#pragma unroll
      for (int i = 0; i < V; ++i) {
        if constexpr (BIN) r.v[i] = G::eval(av[j].v[i], bv[j].v[i]);
        else r.v[i] = G::eval(av[j].v[i], SBt{});
      }
      if (p.swap) G::order_output(p.swap, r);
      char *po = out + offo[j];
      if (FULL || n == V) {
        store_pack<SOt, V>(po, r, p.nt_store != 0);
      } else {
#pragma unroll
        for (int i = 0; i < V; ++i)
          if (i < n) reinterpret_cast<SOt *>(po)[i] = r.v[i];
      }
    }
  }
}

template <class S, int V, int WHICH>
OCN_DEV void stage_dispatch(KTiledArgs &p, const char *base, S *lds, bool full, const uint32_t *lim_dim,
                            uint32_t nvec) {
  if (full && nvec >= (uint32_t)kBlock) stage_operand<S, V, WHICH, true>(p, base, lds, lim_dim, nvec);
  else stage_operand<S, V, WHICH, false>(p, base, lds, lim_dim, nvec);
}

// One tile per loop trip; workgroup b takes tiles b, b + gridDim.x, ...
template <class G> __global__ __launch_bounds__(kBlock) void ew_tiled_kernel(const TiledArgs by_value) {
  using SAt = typename G::SAt;
  using SBt = typename G::SBt;
  constexpr bool BIN = G::NIN2;
  constexpr int VA = 16 / (int)sizeof(SAt) > 1 ? 16 / (int)sizeof(SAt) : 1;
  constexpr int VB = 16 / (int)sizeof(SBt) > 1 ? 16 / (int)sizeof(SBt) : 1;
  constexpr int VC = G::V;
  (void)by_value;  // read through the kernarg segment instead (it is the only argument)
  KTiledArgs &p = *(KTiledArgs *)__builtin_amdgcn_kernarg_segment_ptr();

  const uint32_t tile_elems = 1u << p.tile_bits;
  SAt *lds_a = reinterpret_cast<SAt *>(ocn_lds_raw);
  SBt *lds_b = reinterpret_cast<SBt *>(reinterpret_cast<char *>(ocn_lds_raw) + p.lds_off_b);
  const bool stage_a = p.stage_a, stage_b = BIN && p.stage_b;
  const bool staged = stage_a || stage_b;
  const uint32_t total_tiles = p.total_tiles;
  const int ndim = p.ndim;

  for (uint32_t tile = blockIdx.x; tile < total_tiles; tile += gridDim.x) {
    // tile origin and clipped extents (uniform over the workgroup)
    uint32_t t = tile;
    int64_t base_o = 0, base_a = 0, base_b = 0;
    uint32_t lim_dim[kMaxDims];
    bool full = true;
#pragma unroll
    for (int d = kMaxDims - 1; d >= 0; --d) {
      lim_dim[d] = 1;
      if (d < ndim) {
        const uint32_t dv = p.ntdiv[d].d, dm = p.ntdiv[d].m, ds = p.ntdiv[d].s;
        const uint32_t q = (d == 0) ? 0u : (uint32_t)((((uint64_t)t * dm) >> 32) + t) >> ds;
        const uint32_t tc = t - q * dv;
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

    if (stage_a) {
      if (p.ord[1].vecw) stage_dispatch<SAt, VA, 1>(p, p.a + base_a, lds_a, full, lim_dim, tile_elems >> p.ord[1].vecw);
      else stage_dispatch<SAt, 1, 1>(p, p.a + base_a, lds_a, full, lim_dim, tile_elems);
    }
    if constexpr (BIN) {
      if (stage_b) {
        if (p.ord[2].vecw) stage_dispatch<SBt, VB, 2>(p, p.b + base_b, lds_b, full, lim_dim, tile_elems >> p.ord[2].vecw);
        else stage_dispatch<SBt, 1, 2>(p, p.b + base_b, lds_b, full, lim_dim, tile_elems);
      }
    }
    if (staged) __syncthreads();

    char *out = p.out + base_o;
    const char *pa = p.a + base_a;
    const char *pb = BIN ? p.b + base_b : nullptr;
    if (p.ord[0].vecw) {
      const uint32_t nvec = tile_elems >> p.ord[0].vecw;
      if (full && nvec >= (uint32_t)kBlock) tiled_compute<G, VC, true>(p, out, pa, pb, lds_a, lds_b, lim_dim, nvec);
      else tiled_compute<G, VC, false>(p, out, pa, pb, lds_a, lds_b, lim_dim, nvec);
    } else {
      if (full && tile_elems >= (uint32_t)kBlock) tiled_compute<G, 1, true>(p, out, pa, pb, lds_a, lds_b, lim_dim, tile_elems);
      else tiled_compute<G, 1, false>(p, out, pa, pb, lds_a, lds_b, lim_dim, tile_elems);
    }
    if (staged && tile + gridDim.x < total_tiles) __syncthreads();  // LDS is reused by the next tile
  }
}

// ---------------------------------------------------------------------------------------
// tiled kernel, unclipped all-vector form
// ---------------------------------------------------------------------------------------
//
// Same tiles, enumeration orders, LDS layout and swizzle as ew_tiled_kernel, for the plans the
// host proves simple: no tile is clipped, every order moves whole 16-byte vectors, inputs
// that are not staged are contiguous along the output's fastest axis, and all strides inside
// a tile are non-negative and small enough for 32-bit offsets.

using KFastArgs = const __attribute__((address_space(4))) FastTiledArgs;
using KFastOrder = const __attribute__((address_space(4))) FastOrder;

#ifndef OCN_FAST_J
#define OCN_FAST_J 2
#endif

// lane part of byte offsets (operands selected by WANT: bit 0 out, 1 a, 2 b) and of the slot
template <int WANT, class O> OCN_HDF void fast_lane(const O &o, uint32_t tid, uint32_t (&off)[3], uint32_t &slot) {
  off[0] = off[1] = off[2] = 0;
  slot = 0;
  const int n = o.nlane;
  for (int k = 0; k < n; ++k) {
    const uint32_t c = ((tid >> o.shift[k]) & o.mask[k]) << o.up[k];
    if constexpr ((WANT & 1) != 0) off[0] += c * o.stride[0][k];
    if constexpr ((WANT & 2) != 0) off[1] += c * o.stride[1][k];
    if constexpr ((WANT & 4) != 0) off[2] += c * o.stride[2][k];
    slot += c << o.slot_shift[k];
  }
}

template <class G> __global__ __launch_bounds__(kBlock) void ew_tiled_fast_kernel(const FastTiledArgs by_value) {
  using SAt = typename G::SAt;
  using SBt = typename G::SBt;
  using SOt = typename G::SOt;
  constexpr bool BIN = G::NIN2;
  constexpr int VA = 16 / (int)sizeof(SAt) > 1 ? 16 / (int)sizeof(SAt) : 1;
  constexpr int VB = 16 / (int)sizeof(SBt) > 1 ? 16 / (int)sizeof(SBt) : 1;
  constexpr int VC = G::V;
  constexpr int J = OCN_FAST_J;  // vectors in flight per lane and operand
  (void)by_value;  // read through the kernarg segment instead (it is the only argument)
  KFastArgs &p = *(KFastArgs *)__builtin_amdgcn_kernarg_segment_ptr();
  char *lds = reinterpret_cast<char *>(ocn_lds_raw);

  // tile origin (uniform over the workgroup).  Workgroups go to the eight XCDs in turn, each
  // with an L2 of its own: tiles that share input lines (consecutive tile numbers, in groups
  // of 2 or 4) are given to workgroups b, b + 8, ... which the same XCD starts one after the
  // other, so that the line is fetched from memory once.
  uint32_t t = blockIdx.x;
  if (p.pair_log2) {
    const uint32_t lg = (uint32_t)p.pair_log2, r = t & 7u, h = (t >> 3) & ((1u << lg) - 1u), q = t >> (3 + lg);
    t = (q << (3 + lg)) | (r << lg) | h;
  }
  int64_t bo = 0, ba = 0, bb = 0;
  const int ntd = p.ntd;
  for (int j = 0; j < ntd; ++j) {
    const uint32_t dv = p.ntdiv[j].d, dm = p.ntdiv[j].m, ds = p.ntdiv[j].s;
    const uint32_t q = (uint32_t)((((uint64_t)t * dm) >> 32) + t) >> ds;
    const uint32_t tc = t - q * dv;
    t = q;
    bo += (int64_t)tc * p.step[0][j];
    ba += (int64_t)tc * p.step[1][j];
    if constexpr (BIN) bb += (int64_t)tc * p.step[2][j];
  }
  char *out = p.out + bo;
  const char *pa = p.a + ba;
  const char *pb = BIN ? p.b + bb : nullptr;

  const uint32_t tid = threadIdx.x;
  const bool stage_a = p.stage_a, stage_b = BIN && p.stage_b;

  if (stage_a || stage_b) {
    uint32_t offa[3] = {0, 0, 0}, offb[3] = {0, 0, 0}, slot;
    uint32_t la = 0, lb = 0;  // lane part of the swizzled LDS byte address
    int na = 0, nb = 0;
    if (stage_a) {
      fast_lane<2>(p.ord[1], tid, offa, slot);
      la = (swizzle(slot, p.swz[0].src, p.swz[0].mask, p.swz[0].dst) << p.es_log2[0]) | p.lds_base[0];
      na = p.ord[1].niter;
    }
    if constexpr (BIN) {
      if (stage_b) {
        fast_lane<4>(p.ord[2], tid, offb, slot);
        lb = (swizzle(slot, p.swz[1].src, p.swz[1].mask, p.swz[1].dst) << p.es_log2[1]) | p.lds_base[1];
        nb = p.ord[2].niter;
      }
    }
    const int nmax = na > nb ? na : nb;
    for (int j0 = 0; j0 < nmax; j0 += J) {
      Pack<SAt, VA> va[J];
      Pack<SBt, VB> vb[J];
#pragma unroll
      for (int j = 0; j < J; ++j)
        if (j0 + j < na) load_pack<SAt, VA>(pa + p.ord[1].hi_off[1][j0 + j] + offa[1], va[j], p.nt_a != 0);
      if constexpr (BIN) {
#pragma unroll
        for (int j = 0; j < J; ++j)
          if (j0 + j < nb) load_pack<SBt, VB>(pb + p.ord[2].hi_off[2][j0 + j] + offb[2], vb[j], p.nt_b != 0);
      }
#pragma unroll
      for (int j = 0; j < J; ++j) {
        if (j0 + j < na) {
          const uint32_t h = p.st_hi[0][j0 + j];
#pragma unroll
          for (int i = 0; i < VA; ++i) *reinterpret_cast<SAt *>(lds + (la ^ (h ^ p.st_el[0][i]))) = va[j].v[i];
        }
      }
      if constexpr (BIN) {
#pragma unroll
        for (int j = 0; j < J; ++j) {
          if (j0 + j < nb) {
            const uint32_t h = p.st_hi[1][j0 + j];
#pragma unroll
            for (int i = 0; i < VB; ++i) *reinterpret_cast<SBt *>(lds + (lb ^ (h ^ p.st_el[1][i]))) = vb[j].v[i];
          }
        }
      }
    }
    __syncthreads();
  }

  // compute phase, in the output's order
  uint32_t off[3], slot_unused;
  fast_lane<BIN ? 7 : 3>(p.ord[0], tid, off, slot_unused);
  (void)slot_unused;
  const uint32_t lane_slot = tid << p.vc_log2;
  uint32_t ra = 0, rb = 0;
  if (stage_a) ra = (swizzle(lane_slot, p.swz[0].src, p.swz[0].mask, p.swz[0].dst) << p.es_log2[0]) | p.lds_base[0];
  if (stage_b) rb = (swizzle(lane_slot, p.swz[1].src, p.swz[1].mask, p.swz[1].dst) << p.es_log2[1]) | p.lds_base[1];
  constexpr int EPA = (16 / (int)sizeof(SAt)) < VC ? (16 / (int)sizeof(SAt)) : VC;  // elements per LDS access
  constexpr int EPB = (16 / (int)sizeof(SBt)) < VC ? (16 / (int)sizeof(SBt)) : VC;
  const int no = p.ord[0].niter;
  for (int j0 = 0; j0 < no; j0 += J) {
    Pack<SAt, VC> av[J];
    Pack<SBt, VC> bv[J];
#pragma unroll
    for (int j = 0; j < J; ++j) {
      const int jj = j0 + j;
      if (jj < no) {
        if (stage_a) {
          const uint32_t h = p.rd_hi[0][jj];
#pragma unroll
          for (int c = 0; c < VC / EPA; ++c)
            *reinterpret_cast<Pack<SAt, EPA> *>(&av[j].v[c * EPA]) =
                *reinterpret_cast<const Pack<SAt, EPA> *>(lds + (ra ^ (h ^ p.rd_ch[0][c])));
        } else {
          load_pack<SAt, VC>(pa + p.ord[0].hi_off[1][jj] + off[1], av[j], p.nt_a != 0);
        }
        if constexpr (BIN) {
          if (stage_b) {
            const uint32_t h = p.rd_hi[1][jj];
#pragma unroll
            for (int c = 0; c < VC / EPB; ++c)
              *reinterpret_cast<Pack<SBt, EPB> *>(&bv[j].v[c * EPB]) =
                  *reinterpret_cast<const Pack<SBt, EPB> *>(lds + (rb ^ (h ^ p.rd_ch[1][c])));
          } else {
            load_pack<SBt, VC>(pb + p.ord[0].hi_off[2][jj] + off[2], bv[j], p.nt_b != 0);
          }
        }
      }
    }
#pragma unroll
    for (int j = 0; j < J; ++j) {
      const int jj = j0 + j;
      if (jj >= no) break;  // uniform: the last batch of passes may be short
      Pack<SOt, VC> r;
      if (p.swap) G::order_inputs(p.swap, av[j], bv[j]);
#pragma unroll
      for (int i = 0; i < VC; ++i) {
        if constexpr (BIN) r.v[i] = G::eval(av[j].v[i], bv[j].v[i]);
        else r.v[i] = G::eval(av[j].v[i], SBt{});
      }
      if (p.swap) G::order_output(p.swap, r);
      store_pack<SOt, VC>(out + p.ord[0].hi_off[0][jj] + off[0], r, p.nt_store != 0);
    }
  }
}

#endif  // __HIPCC__

}  // namespace ocn
