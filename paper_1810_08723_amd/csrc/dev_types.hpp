// Device-side element types, conversions and operations of the tensor engine (gfx950).
//
// The fifteen element types are those of the paper's footnote in section 4; the casting
// rules are the library's reading of section 3.2.1 (see include/ocn.h, ocn_cast_copy).
// Every conversion here rounds exactly once; the code must be compiled with floating-point
// contraction off so that each operation below also rounds exactly once.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <limits>
#include <type_traits>

#include "dtypes.hpp"

#define OCN_DEV __device__ __forceinline__

namespace ocn {

// ---- register representations ---------------------------------------------------------
// Half-precision values live in float registers (every half is a float); arithmetic on them
// is done in single precision and rounded to half once, when stored.
struct hreg { float v; };
struct chreg { float re, im; };
struct cf32 { float re, im; };
struct cf64 { double re, im; };

// All of a kernel's arguments in scalar registers at the point of use: left alone, the compiler
// fetches each field just before its first use, in two to four batches of scalar loads that
// wait for one another - each a round trip during which the wavefront has nothing in flight.
#define OCN_ARGS_NOW(...) asm volatile("" ::__VA_ARGS__)

// ---- storage representations ----------------------------------------------------------
struct alignas(4) chalf_s { _Float16 re, im; };
struct alignas(8) cfloat_s { float re, im; };
struct alignas(16) cdouble_s { double re, im; };

template <int DT> struct TypeOf;
template <> struct TypeOf<DT_BOOL> { using S = uint8_t; using R = bool; };
template <> struct TypeOf<DT_I8> { using S = int8_t; using R = int8_t; };
template <> struct TypeOf<DT_I16> { using S = int16_t; using R = int16_t; };
template <> struct TypeOf<DT_I32> { using S = int32_t; using R = int32_t; };
template <> struct TypeOf<DT_I64> { using S = int64_t; using R = int64_t; };
template <> struct TypeOf<DT_U8> { using S = uint8_t; using R = uint8_t; };
template <> struct TypeOf<DT_U16> { using S = uint16_t; using R = uint16_t; };
template <> struct TypeOf<DT_U32> { using S = uint32_t; using R = uint32_t; };
template <> struct TypeOf<DT_U64> { using S = uint64_t; using R = uint64_t; };
template <> struct TypeOf<DT_F16> { using S = _Float16; using R = hreg; };
template <> struct TypeOf<DT_F32> { using S = float; using R = float; };
template <> struct TypeOf<DT_F64> { using S = double; using R = double; };
template <> struct TypeOf<DT_C16> { using S = chalf_s; using R = chreg; };
template <> struct TypeOf<DT_C32> { using S = cfloat_s; using R = cf32; };
template <> struct TypeOf<DT_C64> { using S = cdouble_s; using R = cf64; };

template <int DT> using storage_t = typename TypeOf<DT>::S;
template <int DT> using reg_t = typename TypeOf<DT>::R;

// ---- load / store between storage and register form -------------------------------------
template <int DT> OCN_DEV reg_t<DT> from_storage(storage_t<DT> s) {
  if constexpr (DT == DT_BOOL) return s != 0;
  else if constexpr (DT == DT_F16) return hreg{(float)s};
  else if constexpr (DT == DT_C16) return chreg{(float)s.re, (float)s.im};
  else if constexpr (DT == DT_C32) return cf32{s.re, s.im};
  else if constexpr (DT == DT_C64) return cf64{s.re, s.im};
  else return s;
}

// float -> half, nearest even.  The empty asm makes the operand opaque to the instruction
// selector: left alone, it fuses a preceding single-precision multiply into a mixed-precision
// multiply-add with a +0 addend, which turns a product of -0 into +0.
OCN_DEV _Float16 f32_to_half(float x) {
  asm("" : "+v"(x));
  return (_Float16)x;
}

// Rounds half-precision register values to half (nearest even) - the one rounding of a
// half-precision operation.
template <int DT> OCN_DEV storage_t<DT> to_storage(reg_t<DT> r) {
  if constexpr (DT == DT_BOOL) return r ? 1 : 0;
  else if constexpr (DT == DT_F16) return f32_to_half(r.v);
  else if constexpr (DT == DT_C16) return chalf_s{f32_to_half(r.re), f32_to_half(r.im)};
  else if constexpr (DT == DT_C32) return cfloat_s{r.re, r.im};
  else if constexpr (DT == DT_C64) return cdouble_s{r.re, r.im};
  else return r;
}

// ---- tensors stored in the other byte order (section 3.1.3) -------------------------------
// Every scalar - each component of a complex element - has its bytes reversed in memory.
// The kernels reverse them back right after a load and reverse results right before a store,
// on whole register packs: a handful of byte permutes next to a memory access, so that a
// foreign-endian operand needs no pass of its own.
template <int SCALAR_BYTES, class P> OCN_DEV void reverse_scalars(P &pk) {
  static_assert(sizeof(P) % SCALAR_BYTES == 0, "a pack holds whole scalars");
  if constexpr (SCALAR_BYTES == 2) {
    if constexpr (sizeof(P) % 4 == 0) {   // two scalars per 32-bit word: one byte permute
      uint32_t w[sizeof(P) / 4];
      __builtin_memcpy(w, &pk, sizeof(P));
#pragma unroll
      for (int i = 0; i < (int)(sizeof(P) / 4); ++i) w[i] = __builtin_amdgcn_perm(0u, w[i], 0x02030001u);
      __builtin_memcpy(&pk, w, sizeof(P));
    } else {
      uint16_t w[sizeof(P) / 2];
      __builtin_memcpy(w, &pk, sizeof(P));
#pragma unroll
      for (int i = 0; i < (int)(sizeof(P) / 2); ++i) w[i] = __builtin_bswap16(w[i]);
      __builtin_memcpy(&pk, w, sizeof(P));
    }
  } else if constexpr (SCALAR_BYTES == 4) {
    uint32_t w[sizeof(P) / 4];
    __builtin_memcpy(w, &pk, sizeof(P));
#pragma unroll
    for (int i = 0; i < (int)(sizeof(P) / 4); ++i) w[i] = __builtin_bswap32(w[i]);
    __builtin_memcpy(&pk, w, sizeof(P));
  } else if constexpr (SCALAR_BYTES == 8) {
    uint64_t w[sizeof(P) / 8];
    __builtin_memcpy(w, &pk, sizeof(P));
#pragma unroll
    for (int i = 0; i < (int)(sizeof(P) / 8); ++i) w[i] = __builtin_bswap64(w[i]);
    __builtin_memcpy(&pk, w, sizeof(P));
  }
}
// bytes of one scalar of an element type
constexpr int scalar_bytes(int dt) { return dt_size(dt_real_of(dt)); }

// ---- conversions ----------------------------------------------------------------------

// double -> half, nearest even in ONE step: round to odd into single precision first (the
// sticky low bit keeps the information a second rounding needs), then let the hardware round
// the float to half.  Single precision has 13 more significand bits than half, so the
// two-step result equals direct rounding.
OCN_DEV float double_to_half_value(double x) {
  float f = (float)x;  // nearest even
  double back = (double)f;
  if (back != x && x == x && __builtin_fabsf(f) != __builtin_inff()) {
    uint32_t bits = __float_as_uint(f);
    // step toward zero if rounding moved away from zero
    if (__builtin_fabs(back) > __builtin_fabs(x)) bits -= 1;
    bits |= 1u;  // inexact: force the low bit (round to odd)
    f = __uint_as_float(bits);
  }
  return (float)f32_to_half(f);
}

template <class DI, class SI> OCN_DEV DI sat_int(SI s) {
  constexpr DI dmax = std::numeric_limits<DI>::max();
  constexpr DI dmin = std::numeric_limits<DI>::min();
  if constexpr (std::is_signed_v<SI>) {
    if constexpr (std::is_signed_v<DI>) {
      if constexpr (sizeof(DI) >= sizeof(SI)) return (DI)s;
      else return s < (SI)dmin ? dmin : (s > (SI)dmax ? dmax : (DI)s);
    } else {
      if (s < 0) return 0;
      using US = std::make_unsigned_t<SI>;
      US u = (US)s;
      if constexpr (sizeof(DI) >= sizeof(SI)) return (DI)u;
      else return u > (US)dmax ? dmax : (DI)u;
    }
  } else {
    if constexpr (std::is_signed_v<DI>) {
      if constexpr (sizeof(DI) > sizeof(SI)) return (DI)s;
      else return s > (SI)dmax ? dmax : (DI)s;
    } else {
      if constexpr (sizeof(DI) >= sizeof(SI)) return (DI)s;
      else return s > (SI)dmax ? dmax : (DI)s;
    }
  }
}

// floating -> integer: NaN -> 0, truncate toward zero, saturate (infinities saturate).
// Without branches: the value is clamped to the largest F below 2^(bits-1) (2^bits) and to the
// lower end of the range, so that the conversion itself is always in range, and the two ends
// that the clamp cannot express - NaN, and everything from 2^(bits-1) (2^bits) up, whose
// result is not a value of F when F has fewer digits than the integer - are selected
// afterwards.  (With early returns the compiler built a branch per element around the
// conversion; the time of a double -> int16 cast of 2^24 elements is the same either way.)
template <class DI, class F> OCN_DEV DI sat_real(F x) {
  constexpr int bits = (int)sizeof(DI) * 8;
  constexpr DI dmax = std::numeric_limits<DI>::max();
  constexpr bool sgn = std::is_signed_v<DI>;
  constexpr F top = sgn ? (F)(1ull << (bits - 2)) * (F)2 : (F)(1ull << (bits - 1)) * (F)2;  // 2^(bits-1) / 2^bits, exact
  constexpr F below_top = top * ((F)1 - std::numeric_limits<F>::epsilon() / (F)2);           // the largest F below it
  constexpr F low = sgn ? -top : (F)0;
  const bool over = x >= top, nan = x != x;
  F c = x < low ? low : x;
  c = c > below_top ? below_top : c;
  c = nan ? (F)0 : c;
  DI r;
  if constexpr (sgn) {
    if constexpr (bits <= 32) r = (DI)(int32_t)c;
    else r = (DI)(int64_t)c;
  } else {
    if constexpr (bits <= 32) r = (DI)(uint32_t)c;
    else r = (DI)(uint64_t)c;
  }
  return over ? dmax : r;
}

template <class R> struct RegInfo;
template <> struct RegInfo<bool> { static constexpr int kind = K_BOOL; };
template <> struct RegInfo<int8_t> { static constexpr int kind = K_SINT; };
template <> struct RegInfo<int16_t> { static constexpr int kind = K_SINT; };
template <> struct RegInfo<int32_t> { static constexpr int kind = K_SINT; };
template <> struct RegInfo<int64_t> { static constexpr int kind = K_SINT; };
template <> struct RegInfo<uint8_t> { static constexpr int kind = K_UINT; };
template <> struct RegInfo<uint16_t> { static constexpr int kind = K_UINT; };
template <> struct RegInfo<uint32_t> { static constexpr int kind = K_UINT; };
template <> struct RegInfo<uint64_t> { static constexpr int kind = K_UINT; };
template <> struct RegInfo<hreg> { static constexpr int kind = K_REAL; };
template <> struct RegInfo<float> { static constexpr int kind = K_REAL; };
template <> struct RegInfo<double> { static constexpr int kind = K_REAL; };
template <> struct RegInfo<chreg> { static constexpr int kind = K_CPLX; };
template <> struct RegInfo<cf32> { static constexpr int kind = K_CPLX; };
template <> struct RegInfo<cf64> { static constexpr int kind = K_CPLX; };

// the plain float/double value of a real register
OCN_DEV float real_value(hreg r) { return r.v; }
OCN_DEV float real_value(float r) { return r; }
OCN_DEV double real_value(double r) { return r; }
OCN_DEV float re_of(chreg r) { return r.re; }
OCN_DEV float re_of(cf32 r) { return r.re; }
OCN_DEV double re_of(cf64 r) { return r.re; }
OCN_DEV float im_of(chreg r) { return r.im; }
OCN_DEV float im_of(cf32 r) { return r.im; }
OCN_DEV double im_of(cf64 r) { return r.im; }

// value of a float-held-half after rounding x (float) to half
OCN_DEV float round_f32_to_half_value(float x) { return (float)f32_to_half(x); }

// Real component of `s`, rounded once (nearest even) to the real type RT in {F16,F32,F64};
// returned as float (F16, F32) or double (F64).  `imag` selects the imaginary component of a
// complex source (zero for everything else).
template <int RT, bool imag, class RS> OCN_DEV auto real_component(RS s) {
  constexpr int ks = RegInfo<RS>::kind;
  using F = std::conditional_t<RT == DT_F64, double, float>;
  if constexpr (ks == K_BOOL) {
    return imag ? (F)0 : (s ? (F)1 : (F)0);
  } else if constexpr (ks == K_SINT || ks == K_UINT) {
    if constexpr (imag) return (F)0;
    else if constexpr (RT == DT_F64) return (double)s;
    else if constexpr (RT == DT_F32) return (float)s;
    else {
      // to half: any magnitude >= 65520 becomes infinity, so clamping to +-2^24 (exact in
      // float) changes nothing and keeps the int -> float step exact
      if constexpr (sizeof(RS) <= 2) return round_f32_to_half_value((float)s);
      else {
        constexpr RS lim = (RS)(1 << 24);
        RS c = s > lim ? lim : s;
        if constexpr (ks == K_SINT) c = c < (RS)(-lim) ? (RS)(-lim) : c;
        return round_f32_to_half_value((float)c);
      }
    }
  } else {
    auto v = [&] {
      if constexpr (ks == K_REAL) return real_value(s);
      else if constexpr (imag) return im_of(s);
      else return re_of(s);
    }();
    if constexpr (ks == K_REAL && imag) return (F)0;
    else if constexpr (RT == DT_F64) return (double)v;
    else if constexpr (RT == DT_F32) return (float)v;  // double -> float rounds nearest even
    else {
      if constexpr (std::is_same_v<decltype(v), double>) return double_to_half_value(v);
      else return round_f32_to_half_value(v);
    }
  }
}

// Convert a register value of any type to the register form of dtype D.
template <int D, class RS> OCN_DEV reg_t<D> convert(RS s) {
  constexpr int ks = RegInfo<RS>::kind;
  constexpr int kd = dt_kind(D);
  using RD = reg_t<D>;
  if constexpr (std::is_same_v<RS, RD>) {
    return s;
  } else if constexpr (kd == K_BOOL) {
    if constexpr (ks == K_SINT || ks == K_UINT) return s != 0;
    else if constexpr (ks == K_REAL) return real_value(s) != 0;  // NaN != 0: true
    else return re_of(s) != 0 || im_of(s) != 0;
  } else if constexpr (kd == K_SINT || kd == K_UINT) {
    if constexpr (ks == K_BOOL) return (RD)(s ? 1 : 0);
    else if constexpr (ks == K_SINT || ks == K_UINT) return sat_int<RD>(s);
    else if constexpr (ks == K_REAL) return sat_real<RD>(real_value(s));
    else return sat_real<RD>(re_of(s));  // complex -> integer: real part
  } else if constexpr (kd == K_REAL) {
    auto v = real_component<D, false>(s);
    if constexpr (D == DT_F16) return hreg{v};
    else return v;
  } else {
    constexpr int RT = dt_real_of(D);
    auto re = real_component<RT, false>(s);
    auto im = real_component<RT, true>(s);
    return RD{re, im};
  }
}

// ---- operations in a compute type ------------------------------------------------------

// NaN-propagating min/max with +0 ranked above -0 (independent of operand order)
// (IEEE 754-2019 maximum and minimum are exactly this; gfx950 has them as single instructions
// for single and packed half precision, and the compiler builds the double one from four)
template <class F> OCN_DEV F nan_max(F a, F b) { return __builtin_elementwise_maximum(a, b); }
template <class F> OCN_DEV F nan_min(F a, F b) { return __builtin_elementwise_minimum(a, b); }

template <class I> OCN_DEV I int_div(I a, I b) {
  if (b == 0) return 0;
  if constexpr (std::is_signed_v<I>) {
    using U = std::make_unsigned_t<I>;
    if (b == (I)-1) return (I)((U)0 - (U)a);  // the one overflowing quotient wraps
  }
  return (I)(a / b);
}

// a, b are register values of compute type T
template <int OP, int T> OCN_DEV reg_t<binary_result_dtype(OP, T)> apply_binary(reg_t<T> a, reg_t<T> b) {
  constexpr int k = dt_kind(T);
  using R = reg_t<T>;
  if constexpr (is_logical(OP)) {  // T is bool
    if constexpr (OP == B_LAND) return a && b;
    else if constexpr (OP == B_LOR) return a || b;
    else return a != b;
  } else if constexpr (OP == B_ABSGT) {
    if constexpr (k == K_BOOL) return a && !b;
    else if constexpr (k == K_SINT) {
      using U = std::make_unsigned_t<R>;
      U ma = a < 0 ? (U)((U)0 - (U)a) : (U)a;
      U mb = b < 0 ? (U)((U)0 - (U)b) : (U)b;
      return ma > mb;
    } else if constexpr (k == K_UINT) return a > b;
    else if constexpr (k == K_REAL) return __builtin_fabs((double)real_value(a)) > __builtin_fabs((double)real_value(b));
    else {  // squared magnitudes in double precision, one rounding per operation
      double ar = a.re, ai = a.im, br = b.re, bi = b.im;
      double ma = ar * ar + ai * ai;
      double mb = br * br + bi * bi;
      return ma > mb;
    }
  } else if constexpr (is_compare(OP)) {
    if constexpr (k == K_CPLX) {
      bool eq = (a.re == b.re) && (a.im == b.im);
      return OP == B_EQ ? eq : !eq;
    } else {
      auto x = [&] { if constexpr (k == K_REAL) return real_value(a); else return a; }();
      auto y = [&] { if constexpr (k == K_REAL) return real_value(b); else return b; }();
      if constexpr (OP == B_EQ) return x == y;
      else if constexpr (OP == B_NE) return x != y;
      else if constexpr (OP == B_LT) return x < y;
      else if constexpr (OP == B_LE) return x <= y;
      else if constexpr (OP == B_GT) return x > y;
      else return x >= y;
    }
  } else if constexpr (is_bitwise(OP)) {
    if constexpr (k == K_BOOL) return OP == B_BAND ? (a && b) : (OP == B_BOR ? (a || b) : (a != b));
    else return OP == B_BAND ? (R)(a & b) : (OP == B_BOR ? (R)(a | b) : (R)(a ^ b));
  } else if constexpr (k == K_SINT || k == K_UINT) {
    using U = std::make_unsigned_t<R>;
    if constexpr (OP == B_ADD) return (R)((U)a + (U)b);
    else if constexpr (OP == B_SUB) return (R)((U)a - (U)b);
    else if constexpr (OP == B_MUL) return (R)((U)a * (U)b);
    else if constexpr (OP == B_DIV) return int_div<R>(a, b);
    else if constexpr (OP == B_MIN) return a < b ? a : b;
    else return a > b ? a : b;
  } else if constexpr (k == K_REAL) {
    auto x = real_value(a);
    auto y = real_value(b);
    decltype(x) r;
    if constexpr (OP == B_ADD) r = x + y;
    else if constexpr (OP == B_SUB) r = x - y;
    else if constexpr (OP == B_MUL) r = x * y;
    else if constexpr (OP == B_DIV) r = x / y;
    else if constexpr (OP == B_MIN) r = nan_min(x, y);
    else r = nan_max(x, y);
    if constexpr (T == DT_F16) return hreg{r};
    else return r;
  } else {  // complex; chalf evaluates in single precision
    if constexpr (OP == B_ADD) return R{a.re + b.re, a.im + b.im};
    else if constexpr (OP == B_SUB) return R{a.re - b.re, a.im - b.im};
    else if constexpr (OP == B_MUL) {
      auto p0 = a.re * b.re, p1 = a.im * b.im, p2 = a.re * b.im, p3 = a.im * b.re;
      return R{p0 - p1, p2 + p3};
    } else {
      auto den = b.re * b.re + b.im * b.im;
      auto nre = a.re * b.re + a.im * b.im;
      auto nim = a.im * b.re - a.re * b.im;
      return R{nre / den, nim / den};
    }
  }
}

// ---------------------------------------------------------------------------------------
// elementary functions (section 3.2: trigonometric operations on real and complex floating
// types).  Real arguments use the device math library; complex ones are composed from it by
// the textbook identities, written so that no intermediate overflows before the result does.
// ---------------------------------------------------------------------------------------

template <int OP, class F> OCN_DEV F elementary_real(F x) {
  if constexpr (sizeof(F) == 4) {
    if constexpr (OP == U_SIN) return sinf(x);
    else if constexpr (OP == U_COS) return cosf(x);
    else if constexpr (OP == U_TAN) return tanf(x);
    else if constexpr (OP == U_EXP) return expf(x);
    else if constexpr (OP == U_LOG) return logf(x);
    else if constexpr (OP == U_ASIN) return asinf(x);
    else if constexpr (OP == U_ACOS) return acosf(x);
    else if constexpr (OP == U_ATAN) return atanf(x);
    else if constexpr (OP == U_SINH) return sinhf(x);
    else if constexpr (OP == U_COSH) return coshf(x);
    else return tanhf(x);
  } else {
    if constexpr (OP == U_SIN) return sin(x);
    else if constexpr (OP == U_COS) return cos(x);
    else if constexpr (OP == U_TAN) return tan(x);
    else if constexpr (OP == U_EXP) return exp(x);
    else if constexpr (OP == U_LOG) return log(x);
    else if constexpr (OP == U_ASIN) return asin(x);
    else if constexpr (OP == U_ACOS) return acos(x);
    else if constexpr (OP == U_ATAN) return atan(x);
    else if constexpr (OP == U_SINH) return sinh(x);
    else if constexpr (OP == U_COSH) return cosh(x);
    else return tanh(x);
  }
}

template <class F> OCN_DEV void sincos_any(F x, F &s, F &c) {  // one argument reduction for both
  if constexpr (sizeof(F) == 4) sincosf(x, &s, &c);
  else sincos(x, &s, &c);
}
template <class F> OCN_DEV F exp_any(F x) { if constexpr (sizeof(F) == 4) return expf(x); else return exp(x); }
template <class F> OCN_DEV F log_any(F x) { if constexpr (sizeof(F) == 4) return logf(x); else return log(x); }
template <class F> OCN_DEV F log1p_any(F x) { if constexpr (sizeof(F) == 4) return log1pf(x); else return log1p(x); }
template <class F> OCN_DEV F sqrt_any(F x) { if constexpr (sizeof(F) == 4) return __builtin_sqrtf(x); else return __builtin_sqrt(x); }
template <class F> OCN_DEV F hypot_any(F x, F y) { if constexpr (sizeof(F) == 4) return hypotf(x, y); else return hypot(x, y); }
template <class F> OCN_DEV F atan2_any(F y, F x) { if constexpr (sizeof(F) == 4) return atan2f(y, x); else return atan2(y, x); }
template <class F> OCN_DEV F sinh_any(F x) { if constexpr (sizeof(F) == 4) return sinhf(x); else return sinh(x); }
template <class F> OCN_DEV F cosh_any(F x) { if constexpr (sizeof(F) == 4) return coshf(x); else return cosh(x); }
template <class F> OCN_DEV F expm1_any(F x) { if constexpr (sizeof(F) == 4) return expm1f(x); else return expm1(x); }
template <class F> OCN_DEV F abs_any(F x) { if constexpr (sizeof(F) == 4) return __builtin_fabsf(x); else return __builtin_fabs(x); }
template <class F> OCN_DEV F copysign_any(F x, F y) { if constexpr (sizeof(F) == 4) return __builtin_copysignf(x, y); else return __builtin_copysign(x, y); }

// a * b where an exact zero wins: 0 * Inf = 0 and 0 * NaN = 0 (sign as for finite factors).
// In sin, cos and exp of a complex number a factor is an exact zero only when a component of
// the argument is a zero (or the exponential underflowed); the other factor may have overflowed
// to infinity, and the product is then the zero that C's complex functions return, not NaN.
template <class F> OCN_DEV F times_zero_wins(F a, F b) {
  if (a == 0 || b == 0) {
    const bool neg = (a == a && __builtin_signbit(a)) != (b == b && __builtin_signbit(b));
    return neg ? -(F)0 : (F)0;
  }
  return a * b;
}

template <class F> OCN_DEV F asin_any(F x) { if constexpr (sizeof(F) == 4) return asinf(x); else return asin(x); }
template <class F> OCN_DEV F acos_any(F x) { if constexpr (sizeof(F) == 4) return acosf(x); else return acos(x); }
template <class F> OCN_DEV F atan_any(F x) { if constexpr (sizeof(F) == 4) return atanf(x); else return atan(x); }
template <class F> OCN_DEV bool finite_any(F x) { return abs_any(x) < (F)__builtin_inff(); }   // false for NaN too
template <class F> struct FloatLimits;
template <> struct FloatLimits<float> {
  static constexpr float eps = 1.1920929e-7f, max = 3.4028235e38f, min = 1.1754944e-38f;
  static constexpr float safe_max = 2.3e18f;    // about sqrt(max) / 8
  static constexpr float safe_min = 4.4e-19f;   // about sqrt(min) * 4
};
template <> struct FloatLimits<double> {
  static constexpr double eps = 2.220446049250313e-16, max = 1.7976931348623157e308, min = 2.2250738585072014e-308;
  static constexpr double safe_max = 1.6e153;
  static constexpr double safe_min = 6.0e-154;
};

// The hyperbolic core: sinh, cosh and tanh of x + iy.  The trigonometric functions go through
// it as C defines them - sin z = -i sinh(iz), cos z = cosh(iz), tan z = -i tanh(iz) - so that
// both families share one set of conventions for infinite and NaN parts (C's Annex G: an
// infinite part of the result keeps its direction where the other part of the argument fixes
// one, and an exact zero times anything is that zero).
// sinh x and cosh x from one exponential: with t = e^|x| - 1 (no cancellation for small x),
// sinh |x| = (t + t / (t + 1)) / 2 and cosh x = ((t + 1) + 1 / (t + 1)) / 2, each a few roundings
// from exact.  For |x| below the overflow threshold of e^x only.
template <class F> OCN_DEV void sinh_cosh_any(F x, F &sh, F &ch) {
  const F t = expm1_any(abs_any(x)), e = t + (F)1;
  sh = copysign_any((t + t / e) * (F)0.5, x);
  ch = (e + (F)1 / e) * (F)0.5;
}

template <class F> OCN_DEV void sinh_cosh_complex(F x, F y, bool want_sinh, F &re, F &im) {
  const F half_range = sizeof(F) == 4 ? (F)88 : (F)709;
  const F inf = (F)__builtin_inff();
  if (abs_any(x) == inf && !finite_any(y)) {   // direction unknown: an infinity and a NaN
    re = inf;
    im = y - y;
    return;
  }
  F s, c;
  sincos_any(y, s, c);
  // sinh: sinh x cos y + i cosh x sin y;  cosh: cosh x cos y + i sinh x sin y
  if (abs_any(x) > half_range) {   // cosh x = |sinh x| = e^|x| / 2 to the last bit; applied in two halves
    const F h = exp_any(abs_any(x) * (F)0.5);
    const F ch = h * (F)0.5, sh = copysign_any(h * (F)0.5, x);
    re = times_zero_wins(times_zero_wins(c, h), want_sinh ? sh : ch);
    im = times_zero_wins(times_zero_wins(s, h), want_sinh ? ch : sh);
  } else {
    F sh, ch;
    sinh_cosh_any(x, sh, ch);
    re = times_zero_wins(want_sinh ? sh : ch, c);
    im = times_zero_wins(want_sinh ? ch : sh, s);
  }
}

template <class F> OCN_DEV void tanh_complex(F x, F y, F &re, F &im) {
  const F inf = (F)__builtin_inff();
  const F big = sizeof(F) == 4 ? (F)20 : (F)40;
  if (abs_any(x) == inf) {                       // +-1, and a zero that leans the way sin(2y) does
    re = copysign_any((F)1, x);
    if (finite_any(y)) {
      F s, c;
      sincos_any(y, s, c);
      im = copysign_any((F)0, s * c);
    } else {
      im = copysign_any((F)0, y);
    }
    return;
  }
  if (!finite_any(y)) {                          // no direction at all
    re = x == 0 ? x : y - y;
    im = y - y;
    return;
  }
  if (x != x) {                                  // NaN + i0 keeps the zero
    re = x;
    im = y == 0 ? y : x;
    return;
  }
  F s, c;
  sincos_any(y, s, c);
  if (abs_any(x) > big) {                        // sinh^2 x swamps cos^2 y (and would overflow)
    re = copysign_any((F)1, x);
    im = 4 * s * c * exp_any(-2 * abs_any(x));
  } else {                                       // (sinh x cosh x + i sin y cos y) / (cos^2 y + sinh^2 x)
    F sh, ch;
    sinh_cosh_any(x, sh, ch);
    const F den = c * c + sh * sh;               // a sum of squares: no cancellation
    re = sh * ch / den;
    im = s * c / den;
  }
}

// Inverse sine and cosine of x + iy after Hull, Fairgrieve and Tang (ACM TOMS 23, 1997): with
// r, s the distances of |z| from -1 and +1, a = (r + s) / 2 and b = x / a, the real part is
// asin(b) or acos(b) and the imaginary part log(a + sqrt(a^2 - 1)), each rewritten where it
// would cancel (b near 1, a near 1) and replaced by asymptotic forms where squares would
// overflow or underflow.  Computed for the first quadrant, signs restored at the end.
template <class F> OCN_DEV void asin_acos_complex(F zx, F zy, bool want_acos, F &re, F &im) {
  using L = FloatLimits<F>;
  const F inf = (F)__builtin_inff();
  const F pi = (F)3.14159265358979323846, half_pi = (F)1.57079632679489661923, ln2 = (F)0.69314718055994530942;
  const F x = abs_any(zx), y = abs_any(zy);
  F real, imag;   // of asin (or acos) in the first quadrant
  if (zx != zx || zy != zy) {                    // a NaN part (C, Annex G)
    const F nan = zx + zy;
    if (y == inf) { re = nan; im = want_acos ? -zy : zy; }              // NaN + i Inf: the infinity survives
    else if (x == inf) { re = nan; im = want_acos ? -inf : inf; }       // Inf + i NaN: an infinity of unspecified sign
    else if (zx == 0) { re = want_acos ? half_pi : zx; im = nan; }      // +-0 + i NaN
    else { re = nan; im = nan; }
    return;
  }
  if (x == inf || y == inf) {
    if (x == inf && y == inf) real = (F)0.78539816339744830962;         // pi/4
    else if (x == inf) real = want_acos ? (F)0 : half_pi;
    else real = want_acos ? half_pi : (F)0;
    imag = inf;
  } else if (x < L::safe_max && x > L::safe_min && y < L::safe_max && y > L::safe_min) {
    const F xp1 = x + 1, xm1 = x - 1, yy = y * y;
    const F r = sqrt_any(xp1 * xp1 + yy), s = sqrt_any(xm1 * xm1 + yy);
    const F a = (r + s) * (F)0.5, b = x / a;
    if (b <= (F)0.6417) {
      real = want_acos ? acos_any(b) : asin_any(b);
    } else {                                     // b near 1: through sqrt(a^2 - x^2) without cancellation
      const F apx = a + x;
      F root;                                    // sqrt(a^2 - x^2) (x <= 1), or that over y (x > 1)
      if (x <= 1) root = sqrt_any((F)0.5 * apx * (yy / (r + xp1) + (s - xm1)));
      else root = y * sqrt_any((F)0.5 * (apx / (r + xp1) + apx / (s + xm1)));
      real = want_acos ? atan_any(root / x) : atan_any(x / root);
    }
    if (a <= (F)1.5) {                           // a near 1: a - 1 without cancellation
      F am1;
      if (x < 1) am1 = (F)0.5 * (yy / (r + xp1) + yy / (s - xm1));
      else am1 = (F)0.5 * (yy / (r + xp1) + (s + xm1));
      imag = log1p_any(am1 + sqrt_any(am1 * (a + 1)));
    } else {
      imag = log_any(a + sqrt_any(a * a - 1));
    }
  } else {                                       // a part so large or small that a square would overflow or vanish
    const F xm1 = x - 1, xp1 = x + 1;
    if (y <= L::eps * abs_any(xm1)) {            // y does not reach x - 1
      if (x < 1) {
        real = want_acos ? acos_any(x) : asin_any(x);
        imag = y / sqrt_any(xp1 * (1 - x));
      } else {
        if (L::max / xp1 > xm1) {
          imag = log1p_any(xm1 + sqrt_any(xp1 * xm1));
          real = want_acos ? (y == 0 ? (F)0 : y / sqrt_any(xm1 * xp1)) : half_pi;
        } else {
          imag = ln2 + log_any(x);
          real = want_acos ? y / x : half_pi;
        }
      }
    } else if (y <= L::safe_min) {               // x within y of 1, both differences tiny
      const F t = sqrt_any(y);
      real = want_acos ? t : half_pi - t;
      imag = t;
    } else if (L::eps * y - 1 >= x) {            // x does not reach y
      real = want_acos ? half_pi : x / y;
      imag = ln2 + log_any(y);
    } else if (x > 1) {                          // both large
      real = want_acos ? atan_any(y / x) : atan_any(x / y);
      const F xoy = x / y;
      imag = ln2 + log_any(y) + (F)0.5 * log1p_any(xoy * xoy);
    } else {                                     // x at most 1 (possibly tiny), y beyond the safe range or x below it
      const F a = sqrt_any(1 + y * y);
      real = want_acos ? half_pi : x / a;
      imag = (F)0.5 * log1p_any(2 * y * (y + a));
    }
  }
  if (want_acos) {
    re = __builtin_signbit(zx) ? pi - real : real;
    im = __builtin_signbit(zy) ? imag : -imag;
  } else {
    re = copysign_any(real, zx);
    im = copysign_any(imag, zy);
  }
}

// Inverse hyperbolic tangent of x + iy (the inverse tangent goes through it: atan z =
// -i atanh(iz)): re = log1p(4x / ((1 - x)^2 + y^2)) / 4, im = atan2(2y, (1 - x)(1 + x) - y^2) / 2,
// with the asymptotic forms where a part is so large that the squares would overflow.
template <class F> OCN_DEV void atanh_complex(F x, F y, F &re, F &im) {
  using L = FloatLimits<F>;
  const F inf = (F)__builtin_inff();
  const F half_pi = (F)1.57079632679489661923, ln2 = (F)0.69314718055994530942;
  const F ax = abs_any(x), ay = abs_any(y);
  if (x != x || y != y) {
    if (ay == inf) { re = copysign_any((F)0, x); im = copysign_any(half_pi, y); }   // NaN + i Inf
    else if (ax == inf) { re = copysign_any((F)0, x); im = y; }                     // Inf + i NaN
    else if (x == 0) { re = x; im = y; }                                            // +-0 + i NaN
    else { re = x + y; im = x + y; }
    return;
  }
  if (ax == inf || ay == inf) {
    re = copysign_any((F)0, x);
    im = copysign_any(half_pi, y);
    return;
  }
  const F huge = 16 / L::eps;
  if (ax >= huge || ay >= huge) {                // 1/z to the last bit; the angle has reached +-pi/2
    im = copysign_any(half_pi, y);
    if (ay <= 1) re = 1 / x;
    else if (ax <= 1) re = x / y / y;
    else { const F h = hypot_any(x * (F)0.5, y * (F)0.5); re = x / h / h * (F)0.25; }
    return;
  }
  if (ax == 1 && ay < L::safe_min) {             // next to the poles at +-1: y^2 would vanish
    re = copysign_any((F)0.5, x) * (ln2 - log_any(ay));
  } else {
    const F yy = y * y, d = (1 - ax) * (1 - ax) + yy;
    re = copysign_any((F)0.25 * log1p_any(4 * ax / d), x);
  }
  im = (F)0.5 * atan2_any(2 * y, (1 - ax) * (1 + ax) - y * y);
}

template <int OP, class F> OCN_DEV void elementary_complex(F x, F y, F &re, F &im) {
  if constexpr (OP == U_SINH) {
    sinh_cosh_complex<F>(x, y, true, re, im);
  } else if constexpr (OP == U_COSH) {
    sinh_cosh_complex<F>(x, y, false, re, im);
  } else if constexpr (OP == U_TANH) {
    tanh_complex<F>(x, y, re, im);
  } else if constexpr (OP == U_SIN) {          // -i sinh(iz), iz = -y + ix
    F a, b;
    sinh_cosh_complex<F>(-y, x, true, a, b);
    re = b;
    im = -a;
  } else if constexpr (OP == U_COS) {          // cosh(iz)
    sinh_cosh_complex<F>(-y, x, false, re, im);
  } else if constexpr (OP == U_TAN) {          // -i tanh(iz)
    F a, b;
    tanh_complex<F>(-y, x, a, b);
    re = b;
    im = -a;
  } else if constexpr (OP == U_ASIN) {
    asin_acos_complex<F>(x, y, false, re, im);
  } else if constexpr (OP == U_ACOS) {
    asin_acos_complex<F>(x, y, true, re, im);
  } else if constexpr (OP == U_ATAN) {         // -i atanh(iz)
    F a, b;
    atanh_complex<F>(-y, x, a, b);
    re = b;
    im = -a;
  } else if constexpr (OP == U_EXP) {   // e^x (cos y + i sin y)
    const F half_range = sizeof(F) == 4 ? (F)88 : (F)709;
    const F inf = (F)__builtin_inff();
    if (x == inf && !finite_any(y)) {            // an infinity of unknown direction
      re = inf;
      im = y - y;
      return;
    }
    F s, c;
    sincos_any(y, s, c);
    if (x > half_range) {
      const F h = exp_any(x * (F)0.5);
      re = times_zero_wins(times_zero_wins(h, c), h);
      im = times_zero_wins(times_zero_wins(h, s), h);
    } else {
      const F e = exp_any(x);
      re = times_zero_wins(e, c);
      im = times_zero_wins(e, s);
    }
  } else if constexpr (OP == U_LOG) {   // log |z| + i arg z
    const F h = hypot_any(x, y);
    if (h > (F)0.5 && h < (F)2) {        // near the unit circle: log |z| = log1p(|z|^2 - 1) / 2 without cancellation
      const F ax = abs_any(x);
      re = (F)0.5 * log1p_any((ax - 1) * (ax + 1) + y * y);
    } else {
      re = log_any(h);
    }
    im = atan2_any(y, x);
  } else {                              // U_SQRT, principal branch, signed zeros as in C
    const F inf = (F)__builtin_inff();
    if (x == 0 && y == 0) {
      re = 0;
      im = y;
    } else if (abs_any(y) == inf) {      // an infinite imaginary part wins over everything (as in C)
      re = inf;
      im = y;
    } else if (x == inf) {               // sqrt(+Inf + iy) = +Inf + i0 for finite y
      re = inf;
      im = y == y ? copysign_any((F)0, y) : y;
    } else if (x == -inf) {              // sqrt(-Inf + iy) = 0 + i Inf for finite y
      re = y == y ? (F)0 : y;
      im = copysign_any(inf, y);
    } else {
      // parts in the subnormal range are scaled up first (by an even power of two, taken out of
      // the root again), so that the sum below keeps all its bits; parts near the largest
      // number are scaled down, so that it does not overflow
      const F m = abs_any(x) > abs_any(y) ? abs_any(x) : abs_any(y);
      F up = 1, down = 1;
      if (m < (sizeof(F) == 4 ? (F)0x1p-100f : (F)0x1p-900)) {
        up = sizeof(F) == 4 ? (F)0x1p48f : (F)0x1p108;
        down = sizeof(F) == 4 ? (F)0x1p-24f : (F)0x1p-54;
      } else if (m > (sizeof(F) == 4 ? (F)0x1p125f : (F)0x1p1021)) {
        up = (F)0.0625;
        down = 4;
      }
      x *= up;
      y *= up;
      const F t = sqrt_any((abs_any(x) + hypot_any(x, y)) * (F)0.5);
      if (x >= 0) { re = t * down; im = y / (2 * t) * down; }
      else { re = abs_any(y) / (2 * t) * down; im = copysign_any(t, y) * down; }
    }
  }
}

template <int OP, int T> OCN_DEV reg_t<unary_result_dtype(OP, T)> apply_unary(reg_t<T> a) {
  constexpr int k = dt_kind(T);
  using R = reg_t<T>;
  if constexpr (OP == U_IDENT) return a;
  else if constexpr (OP == U_LNOT) return !a;  // T is bool
  else if constexpr (OP == U_NEG) {
    if constexpr (k == K_SINT || k == K_UINT) { using U = std::make_unsigned_t<R>; return (R)((U)0 - (U)a); }
    else if constexpr (T == DT_F16) return hreg{-a.v};
    else if constexpr (k == K_REAL) return -a;
    else return R{-a.re, -a.im};
  } else if constexpr (OP == U_ABS) {
    if constexpr (k == K_SINT) { using U = std::make_unsigned_t<R>; return a < 0 ? (R)((U)0 - (U)a) : a; }
    else if constexpr (k == K_UINT) return a;
    else if constexpr (T == DT_F16) return hreg{__builtin_fabsf(a.v)};
    else if constexpr (T == DT_F32) return __builtin_fabsf(a);
    else if constexpr (T == DT_F64) return __builtin_fabs(a);
    // the modulus of a complex number: a real value of the same precision, scaled so that it
    // neither overflows nor underflows before the result does
    else if constexpr (T == DT_C16) return hreg{hypotf(a.re, a.im)};
    else if constexpr (T == DT_C32) return hypotf(a.re, a.im);
    else return hypot(a.re, a.im);
  } else if constexpr (OP == U_CONJ) {
    if constexpr (k == K_CPLX) return R{a.re, -a.im};
    else return a;
  } else if constexpr (OP == U_BNOT) {
    if constexpr (k == K_BOOL) return !a;
    else return (R)~a;
  } else if constexpr (OP == U_BSWAP) {  // integer types: reverse the element's bytes
    if constexpr (sizeof(R) == 2) return (R)__builtin_bswap16((uint16_t)a);
    else if constexpr (sizeof(R) == 4) return (R)__builtin_bswap32((uint32_t)a);
    else if constexpr (sizeof(R) == 8) return (R)__builtin_bswap64((uint64_t)a);
    else return a;
  } else if constexpr (OP == U_SQRT && k == K_REAL) {
    if constexpr (T == DT_F16) return hreg{__builtin_sqrtf(a.v)};
    else if constexpr (T == DT_F32) return __builtin_sqrtf(a);
    else return __builtin_sqrt(a);
  } else if constexpr (k == K_REAL) {  // elementary functions: single precision for half and float
    if constexpr (T == DT_F16) return hreg{elementary_real<OP, float>(a.v)};
    else if constexpr (T == DT_F32) return elementary_real<OP, float>(a);
    else return elementary_real<OP, double>(a);
  } else {  // complex elementary functions and the complex square root
    using F = decltype(a.re);
    F re, im;
    elementary_complex<OP, F>(a.re, a.im, re, im);
    return R{re, im};
  }
}

}  // namespace ocn
