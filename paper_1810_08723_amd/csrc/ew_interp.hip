// Generic-dtype elementwise kernel: any combination of the fifteen element types, with the
// conversions picked by (wavefront-uniform) runtime switches.  It serves the combinations for
// which no dtype-specialised kernel is instantiated; one element per lane; 32-bit multiply-shift
// index arithmetic below 2^31 elements, 64-bit division above.
#include <algorithm>

#include "ew_launch.hpp"

namespace ocn {

// load an element of runtime dtype `dt` and convert it to compile-time type T
// (`swapped`: the tensor is stored in the other byte order, its scalars are reversed after
// the load / before the store)
template <int T> __device__ __noinline__ reg_t<T> load_as(const char *p, int dt, bool swapped) {
  switch (dt) {
#define OCN_CASE(D)                                                  \
  case D: {                                                          \
    storage_t<D> s = *reinterpret_cast<const storage_t<D> *>(p);     \
    if (swapped) reverse_scalars<scalar_bytes(D)>(s);                \
    return convert<T>(from_storage<D>(s));                           \
  }
    OCN_CASE(DT_BOOL) OCN_CASE(DT_I8) OCN_CASE(DT_I16) OCN_CASE(DT_I32) OCN_CASE(DT_I64)
    OCN_CASE(DT_U8) OCN_CASE(DT_U16) OCN_CASE(DT_U32) OCN_CASE(DT_U64)
    OCN_CASE(DT_F16) OCN_CASE(DT_F32) OCN_CASE(DT_F64)
    OCN_CASE(DT_C16) OCN_CASE(DT_C32) OCN_CASE(DT_C64)
#undef OCN_CASE
    default: return reg_t<T>{};
  }
}

// convert a register value to runtime dtype `dt` and store it
template <class R> __device__ __noinline__ void store_as(char *p, int dt, R r, bool swapped) {
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

// the value already has the output's type T
template <int T> OCN_DEV void store_same(char *p, reg_t<T> r, bool swapped) {
  storage_t<T> s = to_storage<T>(r);
  if (swapped) reverse_scalars<scalar_bytes(T)>(s);
  *reinterpret_cast<storage_t<T> *>(p) = s;
}

template <int T, int OP> OCN_DEV void binary_one(const InterpArgs &p, reg_t<T> a, reg_t<T> b, char *po) {
  // logical operations always compute in bool
  if constexpr (binary_supported(OP, T) && (!is_logical(OP) || T == DT_BOOL)) {
    auto r = apply_binary<OP, T>(a, b);
    // arithmetic and bitwise results already have the output type (T is out's dtype)
    if constexpr (is_arith(OP) || is_bitwise(OP)) store_same<T>(po, r, (p.swap & 4) != 0);
    else store_as<bool>(po, p.dt_o, r, (p.swap & 4) != 0);
  }
}

template <int T, int OP> OCN_DEV void unary_one(const InterpArgs &p, reg_t<T> a, char *po) {
  if constexpr (unary_supported(OP, T) && (OP != U_LNOT || T == DT_BOOL)) {
    auto r = apply_unary<OP, T>(a);
    // the result has the output type already, except for the logical not (bool) and the
    // modulus of a complex value (the real type of T), which are converted on store
    if constexpr (OP == U_LNOT || unary_result_dtype(OP, T) != T)
      store_as<reg_t<unary_result_dtype(OP, T)>>(po, p.dt_o, r, (p.swap & 4) != 0);
    else store_same<T>(po, r, (p.swap & 4) != 0);
  }
}

template <int T> OCN_DEV void interp_body(const InterpArgs &p, const char *pa, const char *pb, char *po) {
  const reg_t<T> a = load_as<T>(pa, p.dt_a, (p.swap & 1) != 0);
  if (p.nin == 2) {
    const reg_t<T> b = load_as<T>(pb, p.dt_b, (p.swap & 2) != 0);
    switch (p.op) {
#define OCN_CASE(O) case O: binary_one<T, O>(p, a, b, po); break;
      OCN_CASE(B_ADD) OCN_CASE(B_SUB) OCN_CASE(B_MUL) OCN_CASE(B_DIV) OCN_CASE(B_MIN) OCN_CASE(B_MAX)
      OCN_CASE(B_BAND) OCN_CASE(B_BOR) OCN_CASE(B_BXOR) OCN_CASE(B_LAND) OCN_CASE(B_LOR) OCN_CASE(B_LXOR)
      OCN_CASE(B_EQ) OCN_CASE(B_NE) OCN_CASE(B_LT) OCN_CASE(B_LE) OCN_CASE(B_GT) OCN_CASE(B_GE)
      OCN_CASE(B_ABSGT)
#undef OCN_CASE
      default: break;
    }
  } else {
    switch (p.op) {
#define OCN_CASE(O) case O: unary_one<T, O>(p, a, po); break;
      OCN_CASE(U_IDENT) OCN_CASE(U_NEG) OCN_CASE(U_ABS) OCN_CASE(U_CONJ) OCN_CASE(U_LNOT)
      OCN_CASE(U_BNOT) OCN_CASE(U_SQRT) OCN_CASE(U_SIN) OCN_CASE(U_COS) OCN_CASE(U_TAN) OCN_CASE(U_EXP)
      OCN_CASE(U_LOG) OCN_CASE(U_BSWAP) OCN_CASE(U_ASIN) OCN_CASE(U_ACOS) OCN_CASE(U_ATAN) OCN_CASE(U_SINH)
      OCN_CASE(U_COSH) OCN_CASE(U_TANH)
#undef OCN_CASE
      default: break;
    }
  }
}

// (one element per lane and trip: more were measured three times slower, the element chains of
// a lane then run one after the other)

// Workgroup b takes elements b * 256 .. b * 256 + 255, then those gridDim.x * 256 further on, and
// so on: the grid is capped (a launch cannot have 2^32 lanes), larger tensors loop.
__global__ __launch_bounds__(kBlock) void ew_interp_kernel(const InterpArgs p) {
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
    switch (p.T) {
#define OCN_CASE(D) case D: interp_body<D>(p, pa, pb, po); break;
      OCN_CASE(DT_BOOL) OCN_CASE(DT_I8) OCN_CASE(DT_I16) OCN_CASE(DT_I32) OCN_CASE(DT_I64)
      OCN_CASE(DT_U8) OCN_CASE(DT_U16) OCN_CASE(DT_U32) OCN_CASE(DT_U64)
      OCN_CASE(DT_F16) OCN_CASE(DT_F32) OCN_CASE(DT_F64)
      OCN_CASE(DT_C16) OCN_CASE(DT_C32) OCN_CASE(DT_C64)
#undef OCN_CASE
      default: break;
    }
  }
}

hipError_t launch_interp(const EwPlan &p, hipStream_t stream) {
  const InterpArgs args = make_interp_args(p);
  const int64_t blocks = std::min<int64_t>((p.numel + kBlock - 1) / kBlock, max_launch_blocks());
  hipLaunchKernelGGL(ew_interp_kernel, dim3((unsigned)blocks), dim3(kBlock), 0, stream, args);
  return hipGetLastError();
}

}  // namespace ocn
