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

// floating -> integer: NaN -> 0, truncate toward zero, saturate (infinities saturate)
template <class DI, class F> OCN_DEV DI sat_real(F x) {
  constexpr int bits = (int)sizeof(DI) * 8;
  constexpr DI dmax = std::numeric_limits<DI>::max();
  if (x != x) return 0;
  if constexpr (std::is_signed_v<DI>) {
    constexpr DI dmin = std::numeric_limits<DI>::min();
    const F top = (F)(1ull << (bits - 2)) * (F)2;  // 2^(bits-1), exact
    if (x >= top) return dmax;
    if (x <= -top) return dmin;
    if constexpr (bits <= 32) return (DI)(int32_t)x;
    else return (DI)(int64_t)x;
  } else {
    const F top = (F)(1ull << (bits - 1)) * (F)2;  // 2^bits, exact
    if (x >= top) return dmax;
    if (!(x >= (F)1)) return 0;
    if constexpr (bits <= 32) return (DI)(uint32_t)x;
    else return (DI)(uint64_t)x;
  }
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
template <class F> OCN_DEV F nan_max(F a, F b) {
  if (a != a) return a;
  if (b != b) return b;
  if (a > b) return a;
  if (b > a) return b;
  return __builtin_signbit(a) ? b : a;
}
template <class F> OCN_DEV F nan_min(F a, F b) {
  if (a != a) return a;
  if (b != b) return b;
  if (a < b) return a;
  if (b < a) return b;
  return __builtin_signbit(a) ? a : b;
}

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

template <int OP, class F> OCN_DEV void elementary_complex(F x, F y, F &re, F &im) {
  // Beyond this argument exp, cosh and sinh overflow although their product with a small sine
  // or cosine may not: the exponential is then applied in two halves, (t * e^(u/2)) * e^(u/2).
  const F half_range = sizeof(F) == 4 ? (F)88 : (F)709;
  if constexpr (OP == U_SIN) {          // sin x cosh y + i cos x sinh y
    F s, c;
    sincos_any(x, s, c);
    if (abs_any(y) > half_range) {       // cosh y = |sinh y| = e^|y| / 2 to the last bit
      const F h = exp_any(abs_any(y) * (F)0.5);
      re = times_zero_wins(times_zero_wins(s, h), h * (F)0.5);
      im = times_zero_wins(times_zero_wins(c, h), copysign_any(h * (F)0.5, y));
    } else {
      re = times_zero_wins(s, cosh_any(y));
      im = times_zero_wins(c, sinh_any(y));
    }
  } else if constexpr (OP == U_COS) {   // cos x cosh y - i sin x sinh y
    F s, c;
    sincos_any(x, s, c);
    if (abs_any(y) > half_range) {
      const F h = exp_any(abs_any(y) * (F)0.5);
      re = times_zero_wins(times_zero_wins(c, h), h * (F)0.5);
      im = -times_zero_wins(times_zero_wins(s, h), copysign_any(h * (F)0.5, y));
    } else {
      re = c * cosh_any(y);
      im = -times_zero_wins(s, sinh_any(y));
    }
  } else if constexpr (OP == U_TAN) {   // (sin x cos x + i sinh y cosh y) / (cos^2 x + sinh^2 y)
    const F big = sizeof(F) == 4 ? (F)20 : (F)40;
    F s, c;
    sincos_any(x, s, c);
    if (abs_any(y) > big) {              // sinh^2 y swamps cos^2 x (and would overflow): tan -> +-i
      re = 4 * s * c * exp_any(-2 * abs_any(y));
      im = copysign_any((F)1, y);
    } else {
      const F sh = sinh_any(y), ch = cosh_any(y);
      const F den = c * c + sh * sh;     // a sum of squares: no cancellation
      re = s * c / den;
      im = sh * ch / den;
    }
  } else if constexpr (OP == U_EXP) {   // e^x (cos y + i sin y)
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
      const F t = sqrt_any((abs_any(x) + hypot_any(x, y)) * (F)0.5);
      if (x >= 0) { re = t; im = y / (2 * t); }
      else { re = abs_any(y) / (2 * t); im = copysign_any(t, y); }
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
    else return __builtin_fabs(a);
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
