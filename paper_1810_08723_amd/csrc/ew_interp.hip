// Generic-dtype elementwise kernel: any combination of the fifteen element types, with the
// conversions picked by (wavefront-uniform) runtime switches.  It serves the combinations for
// which no dtype-specialised kernel is instantiated; one element per lane; 32-bit multiply-shift
// index arithmetic below 2^31 elements, 64-bit division above.
#include <algorithm>

#include "ew_launch.hpp"

namespace ocn {

// Loads N consecutive elements (N = 1, or 4 along a contiguous innermost dim) of runtime dtype
// `dt` and converts them to compile-time type T.  `contiguous` false: the operand is broadcast
// along that dim, one element serves all N.  `swapped`: the tensor is stored in the other byte
// order, its scalars are reversed after the load / before the store.  One switch serves all N
// elements of a lane.
// (values travel between these functions by value, in registers: arrays handed over by
// reference would live in scratch memory)
template <class R, int N> struct Vals { R v[N]; };

template <int T, int N> __device__ __noinline__ Vals<reg_t<T>, N> load_as(const char *p, int dt, bool contiguous, bool swapped) {
  Vals<reg_t<T>, N> out{};
  switch (dt) {
#define OCN_CASE(D)                                                          \
  case D: {                                                                  \
    if (N > 1 && contiguous) {                                               \
      Pack<storage_t<D>, N> pk;                                              \
      load_pack<storage_t<D>, N>(p, pk);                                     \
      if (swapped) reverse_scalars<scalar_bytes(D)>(pk);                     \
      _Pragma("unroll") for (int i = 0; i < N; ++i) out.v[i] = convert<T>(from_storage<D>(pk.v[i])); \
    } else {                                                                 \
      storage_t<D> s = *reinterpret_cast<const storage_t<D> *>(p);           \
      if (swapped) reverse_scalars<scalar_bytes(D)>(s);                      \
      const reg_t<T> v = convert<T>(from_storage<D>(s));                     \
      _Pragma("unroll") for (int i = 0; i < N; ++i) out.v[i] = v;            \
    }                                                                        \
  } break;
    OCN_CASE(DT_BOOL) OCN_CASE(DT_I8) OCN_CASE(DT_I16) OCN_CASE(DT_I32) OCN_CASE(DT_I64)
    OCN_CASE(DT_U8) OCN_CASE(DT_U16) OCN_CASE(DT_U32) OCN_CASE(DT_U64)
    OCN_CASE(DT_F16) OCN_CASE(DT_F32) OCN_CASE(DT_F64)
    OCN_CASE(DT_C16) OCN_CASE(DT_C32) OCN_CASE(DT_C64)
#undef OCN_CASE
    default: break;
  }
  return out;
}

// converts N register values to runtime dtype `dt` and stores them side by side
template <class R, int N> __device__ __noinline__ void store_as(char *p, int dt, Vals<R, N> r, bool swapped) {
  switch (dt) {
#define OCN_CASE(D)                                                                              \
  case D: {                                                                                      \
    Pack<storage_t<D>, N> pk;                                                                    \
    _Pragma("unroll") for (int i = 0; i < N; ++i) pk.v[i] = to_storage<D>(convert<D>(r.v[i]));   \
    if (swapped) reverse_scalars<scalar_bytes(D)>(pk);                                           \
    store_pack<storage_t<D>, N>(p, pk);                                                          \
  } break;
    OCN_CASE(DT_BOOL) OCN_CASE(DT_I8) OCN_CASE(DT_I16) OCN_CASE(DT_I32) OCN_CASE(DT_I64)
    OCN_CASE(DT_U8) OCN_CASE(DT_U16) OCN_CASE(DT_U32) OCN_CASE(DT_U64)
    OCN_CASE(DT_F16) OCN_CASE(DT_F32) OCN_CASE(DT_F64)
    OCN_CASE(DT_C16) OCN_CASE(DT_C32) OCN_CASE(DT_C64)
#undef OCN_CASE
    default: break;
  }
}

// the values already have the output's type T
template <int T, int N> OCN_DEV void store_same(char *p, const Vals<reg_t<T>, N> &r, bool swapped) {
  Pack<storage_t<T>, N> pk;
#pragma unroll
  for (int i = 0; i < N; ++i) pk.v[i] = to_storage<T>(r.v[i]);
  if (swapped) reverse_scalars<scalar_bytes(T)>(pk);
  store_pack<storage_t<T>, N>(p, pk);
}

template <int T, int OP, int N>
OCN_DEV void binary_one(const InterpArgs &p, const Vals<reg_t<T>, N> &a, const Vals<reg_t<T>, N> &b, char *po) {
  // logical operations always compute in bool
  if constexpr (binary_supported(OP, T) && (!is_logical(OP) || T == DT_BOOL)) {
    Vals<reg_t<binary_result_dtype(OP, T)>, N> r;
#pragma unroll
    for (int i = 0; i < N; ++i) r.v[i] = apply_binary<OP, T>(a.v[i], b.v[i]);
    // arithmetic and bitwise results have type T: the output's own, or the operands' promoted
    // type, then converted on store; predicates give a bool
    if constexpr (is_arith(OP) || is_bitwise(OP)) {
      if (p.dt_o == T) store_same<T, N>(po, r, (p.swap & 4) != 0);
      else store_as<reg_t<T>, N>(po, p.dt_o, r, (p.swap & 4) != 0);
    } else {
      store_as<bool, N>(po, p.dt_o, r, (p.swap & 4) != 0);
    }
  }
}

template <int T, int OP, int N> OCN_DEV void unary_one(const InterpArgs &p, const Vals<reg_t<T>, N> &a, char *po) {
  if constexpr (unary_supported(OP, T) && (OP != U_LNOT || T == DT_BOOL)) {
    constexpr int RD = unary_result_dtype(OP, T);
    Vals<reg_t<RD>, N> r;
#pragma unroll
    for (int i = 0; i < N; ++i) r.v[i] = apply_unary<OP, T>(a.v[i]);
    // the result has the output type already, except for the logical not (bool) and the
    // modulus of a complex value (the real type of T), which are converted on store
    if constexpr (OP == U_LNOT || RD != T) store_as<reg_t<RD>, N>(po, p.dt_o, r, (p.swap & 4) != 0);
    else store_same<T, N>(po, r, (p.swap & 4) != 0);
  }
}

// ELEMENTARY: the kernel that holds the elementary functions (sin ... tanh), which in double
// precision need some 180 vector registers; everything else lives in the other kernel.
constexpr bool is_elementary(int op) {
  return (op >= U_SIN && op <= U_LOG) || (op >= U_ASIN && op <= U_TANH);
}

template <int T, bool ELEMENTARY, int N>
OCN_DEV void interp_body(const InterpArgs &p, const char *pa, const char *pb, char *po) {
  const Vals<reg_t<T>, N> a = load_as<T, N>(pa, p.dt_a, p.inner_a != 0, (p.swap & 1) != 0);
  if constexpr (ELEMENTARY) {
    switch (p.op) {
#define OCN_CASE(O) case O: unary_one<T, O, N>(p, a, po); break;
      OCN_CASE(U_SIN) OCN_CASE(U_COS) OCN_CASE(U_TAN) OCN_CASE(U_EXP) OCN_CASE(U_LOG)
      OCN_CASE(U_ASIN) OCN_CASE(U_ACOS) OCN_CASE(U_ATAN) OCN_CASE(U_SINH) OCN_CASE(U_COSH) OCN_CASE(U_TANH)
#undef OCN_CASE
      default: break;
    }
  } else if (p.nin == 2) {
    const Vals<reg_t<T>, N> b = load_as<T, N>(pb, p.dt_b, p.inner_b != 0, (p.swap & 2) != 0);
    switch (p.op) {
#define OCN_CASE(O) case O: binary_one<T, O, N>(p, a, b, po); break;
      OCN_CASE(B_ADD) OCN_CASE(B_SUB) OCN_CASE(B_MUL) OCN_CASE(B_DIV) OCN_CASE(B_MIN) OCN_CASE(B_MAX)
      OCN_CASE(B_BAND) OCN_CASE(B_BOR) OCN_CASE(B_BXOR) OCN_CASE(B_LAND) OCN_CASE(B_LOR) OCN_CASE(B_LXOR)
      OCN_CASE(B_EQ) OCN_CASE(B_NE) OCN_CASE(B_LT) OCN_CASE(B_LE) OCN_CASE(B_GT) OCN_CASE(B_GE)
      OCN_CASE(B_ABSGT)
#undef OCN_CASE
      default: break;
    }
  } else {
    switch (p.op) {
#define OCN_CASE(O) case O: unary_one<T, O, N>(p, a, po); break;
      OCN_CASE(U_IDENT) OCN_CASE(U_NEG) OCN_CASE(U_ABS) OCN_CASE(U_CONJ) OCN_CASE(U_LNOT)
      OCN_CASE(U_BNOT) OCN_CASE(U_SQRT) OCN_CASE(U_BSWAP)
#undef OCN_CASE
      default: break;
    }
  }
}

// (one lane item per trip: more were measured three times slower, the chains of a lane then
// run one after the other)

// Workgroup b takes elements b * 256 .. b * 256 + 255, then those gridDim.x * 256 further on, and
// so on: the grid is capped (a launch cannot have 2^32 lanes), larger tensors loop.
// One kernel per compute type T: each gets the registers its own operations need (a single
// kernel for all types needed 217 vector registers - the complex elementary functions - and ran
// everything else at two wavefronts per SIMD: int16 + float -> double over 2^25 elements 692 us).
template <int T, bool ELEMENTARY> __global__ __launch_bounds__(kBlock) void ew_interp_kernel(const InterpArgs p) {
  const int64_t lin0 = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  const int64_t step = (int64_t)gridDim.x * kBlock;
  for (int64_t lin_k = lin0; lin_k < p.numel; lin_k += step) {
    int64_t lin = lin_k;
    int64_t off_o = 0, off_a = 0, off_b = 0;
    if (p.idx32) {
      uint32_t l = (uint32_t)lin;
#pragma unroll
      for (int d = kMaxDims - 1; d >= 0; --d) {
        if (d < p.ndim) {
          const uint32_t q = d == 0 ? 0u : fastdiv(l, p.div[d]);   // the slowest dim takes what is left
          const uint32_t i = l - q * p.div[d].d;
          l = q;
          off_o += (int64_t)i * p.so[d];
          off_a += (int64_t)i * p.sa[d];
          off_b += (int64_t)i * p.sb[d];
        }
      }
    } else {
#pragma unroll
      for (int d = kMaxDims - 1; d >= 0; --d) {
        if (d < p.ndim) {
          const int64_t q = d == 0 ? 0 : lin / p.size[d];
          const int64_t i = lin - q * p.size[d];
          lin = q;
          off_o += i * p.so[d];
          off_a += i * p.sa[d];
          off_b += i * p.sb[d];
        }
      }
    }
    const char *pa = p.a + off_a;
    const char *pb = p.nin == 2 ? p.b + off_b : nullptr;
    char *po = p.out + off_o;
    // four elements per lane along a contiguous innermost dim (the index arithmetic above then
    // runs over groups of four), else one
    if (!ELEMENTARY && p.vec == 4) interp_body<T, ELEMENTARY, ELEMENTARY ? 1 : 4>(p, pa, pb, po);
    else interp_body<T, ELEMENTARY, 1>(p, pa, pb, po);
  }
}

hipError_t launch_interp(const EwPlan &p, hipStream_t stream) {
  const InterpArgs args = make_interp_args(p);
  const int64_t blocks = std::min<int64_t>((args.numel + kBlock - 1) / kBlock, max_launch_blocks());
  const bool elementary = p.nin == 1 && is_elementary(p.op);
  switch (p.T) {
#define OCN_CASE(D)                                                                                                     \
  case D:                                                                                                               \
    if (elementary) hipLaunchKernelGGL((ew_interp_kernel<D, true>), dim3((unsigned)blocks), dim3(kBlock), 0, stream, args);   \
    else hipLaunchKernelGGL((ew_interp_kernel<D, false>), dim3((unsigned)blocks), dim3(kBlock), 0, stream, args);             \
    break;
    OCN_CASE(DT_BOOL) OCN_CASE(DT_I8) OCN_CASE(DT_I16) OCN_CASE(DT_I32) OCN_CASE(DT_I64)
    OCN_CASE(DT_U8) OCN_CASE(DT_U16) OCN_CASE(DT_U32) OCN_CASE(DT_U64)
    OCN_CASE(DT_F16) OCN_CASE(DT_F32) OCN_CASE(DT_F64)
    OCN_CASE(DT_C16) OCN_CASE(DT_C32) OCN_CASE(DT_C64)
#undef OCN_CASE
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace ocn
