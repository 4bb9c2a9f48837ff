/*
 * CPU oracle for the strided tensor engine: TEST INFRASTRUCTURE ONLY (see ocn_oracle.h).
 *
 * Everything is evaluated one logical element at a time, straight from the caller's raw
 * descriptors: decode the linear output index into a multi-index, form each operand's byte
 * address as base + offset + sum_d i_d * stride[d] (strides in bytes, section 3.1.3), load,
 * convert to the compute type, apply the operation once, convert to the output type, store.
 * Dimensions are never reordered, merged or flipped here.
 *
 * Build with contraction of a*b+c into fused multiply-adds switched off and no fast-math,
 * so that every floating-point operation below rounds exactly once in its own type.
 *
 * Conventions where the paper is silent are readings made here (listed with the design
 * notes): float->integer casts truncate toward zero, saturate, and map NaN to 0;
 * integer->narrower-integer casts saturate; conversions to floating types round to nearest
 * even in one step; half-precision types (real and complex) compute in single precision
 * and round once when stored; integer arithmetic wraps; min/max propagate NaN and rank +0
 * above -0.
 */
#include "ocn_oracle.h"

#include <complex.h>
#include <math.h>
#include <string.h>

/* ------------------------------------------------------------------------------------ */
/* dtype facts                                                                          */
/* ------------------------------------------------------------------------------------ */

typedef enum { K_BOOL, K_SINT, K_UINT, K_REAL, K_CPLX } kind_t;

static const int k_size[ORC_NUM_DTYPES] = {1, 1, 2, 4, 8, 1, 2, 4, 8, 2, 4, 8, 4, 8, 16};

static int valid_dtype(int dt) { return dt >= 0 && dt < ORC_NUM_DTYPES; }

int orc_dtype_size(int dt) { return valid_dtype(dt) ? k_size[dt] : 0; }

static kind_t kind_of(int dt) {
  if (dt == ORC_BOOL) return K_BOOL;
  if (dt >= ORC_INT8 && dt <= ORC_INT64) return K_SINT;
  if (dt >= ORC_UINT8 && dt <= ORC_UINT64) return K_UINT;
  if (dt >= ORC_HALF && dt <= ORC_DOUBLE) return K_REAL;
  return K_CPLX;
}

/* bits of an integer type (8..64); 0 for others */
static int int_bits(int dt) {
  switch (dt) {
    case ORC_INT8: case ORC_UINT8: return 8;
    case ORC_INT16: case ORC_UINT16: return 16;
    case ORC_INT32: case ORC_UINT32: return 32;
    case ORC_INT64: case ORC_UINT64: return 64;
    default: return 0;
  }
}

/* real component type of a floating dtype: HALF, FLOAT or DOUBLE */
static int real_part_type(int dt) {
  switch (dt) {
    case ORC_CHALF: return ORC_HALF;
    case ORC_CFLOAT: return ORC_FLOAT;
    case ORC_CDOUBLE: return ORC_DOUBLE;
    default: return dt;
  }
}

static int complex_of(int real_dt) {
  switch (real_dt) {
    case ORC_HALF: return ORC_CHALF;
    case ORC_FLOAT: return ORC_CFLOAT;
    default: return ORC_CDOUBLE;
  }
}

/* ------------------------------------------------------------------------------------ */
/* half precision <-> double, written from the IEEE 754 binary16 format definition      */
/* ------------------------------------------------------------------------------------ */

double orc_half_bits_to_double(uint16_t h) {
  int sign = (h >> 15) & 1;
  int e = (h >> 10) & 0x1F;
  int m = h & 0x3FF;
  double v;
  if (e == 0x1F) {
    v = m ? (double)NAN : (double)INFINITY;
  } else if (e == 0) {
    v = ldexp((double)m, -24); /* subnormal: m * 2^-24 */
  } else {
    v = ldexp((double)(1024 + m), e - 25); /* (1 + m/1024) * 2^(e-15) */
  }
  return sign ? -v : v;
}

/* Round to nearest, ties to even, in ONE step from the double value. */
uint16_t orc_double_to_half_bits(double x) {
  uint64_t bits;
  memcpy(&bits, &x, sizeof bits);
  uint16_t sign = (uint16_t)((bits >> 48) & 0x8000u);
  double a = fabs(x);
  if (isnan(x)) return (uint16_t)(sign | 0x7E00u);
  if (a == 0.0) return sign;
  /* 65520 is halfway between the largest finite half (65504) and 2^16: it and everything
   * above rounds to infinity */
  if (a >= 65520.0) return (uint16_t)(sign | 0x7C00u);
  int ex;
  (void)frexp(a, &ex); /* a = f * 2^ex with 0.5 <= f < 1, so floor(log2 a) = ex - 1 */
  int e = ex - 1;
  if (e < -14) e = -14;                  /* subnormal range shares the quantum 2^-24 */
  double n = ldexp(a, 10 - e);           /* exact: a in units of the quantum 2^(e-10) */
  double r = nearbyint(n);               /* default rounding mode: nearest even */
  int64_t ri = (int64_t)r;               /* 0..2048 */
  return (uint16_t)(sign | (uint16_t)(((e + 15) << 10) + (ri - 1024)));
}

static double round_to_half(double x) { return orc_half_bits_to_double(orc_double_to_half_bits(x)); }

/* ------------------------------------------------------------------------------------ */
/* one element, held exactly                                                            */
/* ------------------------------------------------------------------------------------ */

typedef struct {
  kind_t k;
  int64_t i;      /* K_BOOL (0/1), K_SINT */
  uint64_t u;     /* K_UINT */
  double re, im;  /* K_REAL (re), K_CPLX; doubles hold half and float values exactly */
} val_t;

static val_t load_elem(int dt, const unsigned char *p) {
  val_t v;
  memset(&v, 0, sizeof v);
  v.k = kind_of(dt);
  switch (dt) {
    case ORC_BOOL: v.i = (*p != 0); break;
    case ORC_INT8: { int8_t t; memcpy(&t, p, 1); v.i = t; } break;
    case ORC_INT16: { int16_t t; memcpy(&t, p, 2); v.i = t; } break;
    case ORC_INT32: { int32_t t; memcpy(&t, p, 4); v.i = t; } break;
    case ORC_INT64: { int64_t t; memcpy(&t, p, 8); v.i = t; } break;
    case ORC_UINT8: { uint8_t t; memcpy(&t, p, 1); v.u = t; } break;
    case ORC_UINT16: { uint16_t t; memcpy(&t, p, 2); v.u = t; } break;
    case ORC_UINT32: { uint32_t t; memcpy(&t, p, 4); v.u = t; } break;
    case ORC_UINT64: { uint64_t t; memcpy(&t, p, 8); v.u = t; } break;
    case ORC_HALF: { uint16_t t; memcpy(&t, p, 2); v.re = orc_half_bits_to_double(t); } break;
    case ORC_FLOAT: { float t; memcpy(&t, p, 4); v.re = t; } break;
    case ORC_DOUBLE: { double t; memcpy(&t, p, 8); v.re = t; } break;
    case ORC_CHALF: { uint16_t t[2]; memcpy(t, p, 4);
                      v.re = orc_half_bits_to_double(t[0]); v.im = orc_half_bits_to_double(t[1]); } break;
    case ORC_CFLOAT: { float t[2]; memcpy(t, p, 8); v.re = t[0]; v.im = t[1]; } break;
    case ORC_CDOUBLE: { double t[2]; memcpy(t, p, 16); v.re = t[0]; v.im = t[1]; } break;
  }
  return v;
}

/* v must already be of dt's kind and rounded to dt's precision / range */
static void store_elem(int dt, unsigned char *p, val_t v) {
  switch (dt) {
    case ORC_BOOL: { uint8_t t = (uint8_t)(v.i != 0); memcpy(p, &t, 1); } break;
    case ORC_INT8: { int8_t t = (int8_t)v.i; memcpy(p, &t, 1); } break;
    case ORC_INT16: { int16_t t = (int16_t)v.i; memcpy(p, &t, 2); } break;
    case ORC_INT32: { int32_t t = (int32_t)v.i; memcpy(p, &t, 4); } break;
    case ORC_INT64: { int64_t t = v.i; memcpy(p, &t, 8); } break;
    case ORC_UINT8: { uint8_t t = (uint8_t)v.u; memcpy(p, &t, 1); } break;
    case ORC_UINT16: { uint16_t t = (uint16_t)v.u; memcpy(p, &t, 2); } break;
    case ORC_UINT32: { uint32_t t = (uint32_t)v.u; memcpy(p, &t, 4); } break;
    case ORC_UINT64: { uint64_t t = v.u; memcpy(p, &t, 8); } break;
    case ORC_HALF: { uint16_t t = orc_double_to_half_bits(v.re); memcpy(p, &t, 2); } break;
    case ORC_FLOAT: { float t = (float)v.re; memcpy(p, &t, 4); } break;
    case ORC_DOUBLE: { double t = v.re; memcpy(p, &t, 8); } break;
    case ORC_CHALF: { uint16_t t[2] = {orc_double_to_half_bits(v.re), orc_double_to_half_bits(v.im)};
                      memcpy(p, t, 4); } break;
    case ORC_CFLOAT: { float t[2] = {(float)v.re, (float)v.im}; memcpy(p, t, 8); } break;
    case ORC_CDOUBLE: { double t[2] = {v.re, v.im}; memcpy(p, t, 16); } break;
  }
}

/* Elements of a tensor stored in the other byte order (section 3.1.3): the bytes of every
 * scalar - of each component of a complex element - are reversed in memory.  Loading
 * un-reverses them first, storing reverses them last; the value in between is the same. */
static int scalar_bytes(int dt) {
  switch (dt) {
    case ORC_BOOL: case ORC_INT8: case ORC_UINT8: return 1;
    case ORC_INT16: case ORC_UINT16: case ORC_HALF: case ORC_CHALF: return 2;
    case ORC_INT32: case ORC_UINT32: case ORC_FLOAT: case ORC_CFLOAT: return 4;
    default: return 8;
  }
}
static void reverse_scalars(int dt, const unsigned char *src, unsigned char *dst) {
  int sb = scalar_bytes(dt), n = orc_dtype_size(dt);
  for (int s0 = 0; s0 < n; s0 += sb)
    for (int b = 0; b < sb; ++b) dst[s0 + b] = src[s0 + sb - 1 - b];
}
static val_t load_tensor_elem(const orc_tensor *t, const unsigned char *p) {
  if (!t->byteswapped) return load_elem(t->dtype, p);
  unsigned char tmp[16];
  reverse_scalars(t->dtype, p, tmp);
  return load_elem(t->dtype, tmp);
}
static void store_tensor_elem(const orc_tensor *t, unsigned char *p, val_t v) {
  if (!t->byteswapped) { store_elem(t->dtype, p, v); return; }
  unsigned char tmp[16];
  store_elem(t->dtype, tmp, v);
  reverse_scalars(t->dtype, tmp, p);
}

/* ------------------------------------------------------------------------------------ */
/* conversion rules (explicit and implicit type casting, section 3.2.1)                 */
/* ------------------------------------------------------------------------------------ */

static int64_t sint_min(int bits) { return bits == 64 ? INT64_MIN : -((int64_t)1 << (bits - 1)); }
static int64_t sint_max(int bits) { return bits == 64 ? INT64_MAX : ((int64_t)1 << (bits - 1)) - 1; }
static uint64_t uint_max(int bits) { return bits == 64 ? UINT64_MAX : (((uint64_t)1 << bits) - 1); }

/* float -> signed 64: NaN -> 0, truncate toward zero, saturate (+-Inf saturate) */
static int64_t real_to_i64_sat(double x) {
  if (isnan(x)) return 0;
  double t = trunc(x);
  if (t >= 9223372036854775808.0) return INT64_MAX;   /* 2^63 and above */
  if (t <= -9223372036854775808.0) return INT64_MIN;  /* -2^63 and below */
  return (int64_t)t;
}

static uint64_t real_to_u64_sat(double x) {
  if (isnan(x)) return 0;
  double t = trunc(x);
  if (t <= 0.0) return 0; /* negatives and -0 */
  if (t >= 18446744073709551616.0) return UINT64_MAX; /* 2^64 and above */
  return (uint64_t)t;
}

/* round a double to the precision of a real type, nearest even, in one step */
static double round_real(double x, int real_dt) {
  if (real_dt == ORC_HALF) return round_to_half(x);
  if (real_dt == ORC_FLOAT) return (double)(float)x;
  return x;
}

/* integer value -> real type, nearest even in one step.  Casting a 64-bit integer to
 * float or double is a single correctly rounded operation in C on this platform.  For half
 * the detour through double is harmless: any magnitude at or above 65520 becomes infinity
 * either way, and below that the integer is exact in double. */
static double sint_to_real(int64_t i, int real_dt) {
  if (real_dt == ORC_FLOAT) return (double)(float)i;
  if (real_dt == ORC_DOUBLE) return (double)i;
  return round_to_half((double)i);
}
static double uint_to_real(uint64_t u, int real_dt) {
  if (real_dt == ORC_FLOAT) return (double)(float)u;
  if (real_dt == ORC_DOUBLE) return (double)u;
  return round_to_half((double)u);
}

static double to_real_component(val_t v, int real_dt, int imag) {
  switch (v.k) {
    case K_BOOL: case K_SINT: return imag ? 0.0 : sint_to_real(v.i, real_dt);
    case K_UINT: return imag ? 0.0 : uint_to_real(v.u, real_dt);
    case K_REAL: return imag ? 0.0 : round_real(v.re, real_dt);
    default: return round_real(imag ? v.im : v.re, real_dt);
  }
}

static val_t convert(val_t v, int dt) {
  val_t r;
  memset(&r, 0, sizeof r);
  r.k = kind_of(dt);
  switch (r.k) {
    case K_BOOL: /* anything non-zero is true; NaN compares unequal to zero, hence true */
      switch (v.k) {
        case K_BOOL: case K_SINT: r.i = (v.i != 0); break;
        case K_UINT: r.i = (v.u != 0); break;
        case K_REAL: r.i = (v.re != 0.0); break;
        case K_CPLX: r.i = (v.re != 0.0) || (v.im != 0.0); break;
      }
      break;
    case K_SINT: {
      int bits = int_bits(dt);
      int64_t lo = sint_min(bits), hi = sint_max(bits), x = 0;
      switch (v.k) {
        case K_BOOL: case K_SINT: x = v.i; break;
        case K_UINT: x = v.u > (uint64_t)INT64_MAX ? INT64_MAX : (int64_t)v.u; break;
        case K_REAL: case K_CPLX: x = real_to_i64_sat(v.re); break; /* complex: real part */
      }
      r.i = x < lo ? lo : (x > hi ? hi : x);
    } break;
    case K_UINT: {
      int bits = int_bits(dt);
      uint64_t hi = uint_max(bits), x = 0;
      switch (v.k) {
        case K_BOOL: case K_SINT: x = v.i < 0 ? 0 : (uint64_t)v.i; break;
        case K_UINT: x = v.u; break;
        case K_REAL: case K_CPLX: x = real_to_u64_sat(v.re); break;
      }
      r.u = x > hi ? hi : x;
    } break;
    case K_REAL:
      r.re = to_real_component(v, dt, 0); /* complex source: real part */
      break;
    case K_CPLX:
      r.re = to_real_component(v, real_part_type(dt), 0);
      r.im = to_real_component(v, real_part_type(dt), 1); /* +0 for real sources */
      break;
  }
  return r;
}

/* ------------------------------------------------------------------------------------ */
/* implicit-casting result type (section 3.2.1)                                         */
/* ------------------------------------------------------------------------------------ */

/* Exactly representable integer range of a real dtype: [-2^p, 2^p] for a float with p
 * significand bits, the full range for integer types.  Returned as lo = -(2^lo_exp) or 0,
 * hi = 2^hi_exp - (1 or 0); compared through these exponents to avoid 2^64 overflow. */
static int contains(int big, int small) {
  kind_t kb = kind_of(big), ks = kind_of(small);
  if (kb == K_CPLX || ks == K_CPLX) return 0; /* handled by the caller on real parts */
  if (kb == K_REAL) {
    int p = big == ORC_HALF ? 11 : (big == ORC_FLOAT ? 24 : 53);
    if (ks == K_REAL) {
      int q = small == ORC_HALF ? 11 : (small == ORC_FLOAT ? 24 : 53);
      return q <= p;
    }
    if (ks == K_BOOL) return 1;
    /* integers up to magnitude 2^p are exact: intN needs N-1 <= p, uintN needs N <= p */
    return ks == K_SINT ? (int_bits(small) - 1 <= p) : (int_bits(small) <= p);
  }
  if (ks == K_REAL) return 0; /* an integer type cannot keep fractions */
  if (kb == K_BOOL) return ks == K_BOOL;
  if (ks == K_BOOL) return 1;
  if (kb == K_SINT) return ks == K_SINT ? int_bits(small) <= int_bits(big)
                                        : int_bits(small) < int_bits(big);
  /* unsigned keeps only unsigned of at most its width */
  return ks == K_UINT && int_bits(small) <= int_bits(big);
}

static int promote_real(int a, int b) {
  /* candidates from small to large; at equal size integers come before floats */
  static const int cand[] = {ORC_BOOL, ORC_INT8, ORC_UINT8, ORC_INT16, ORC_UINT16, ORC_HALF,
                             ORC_INT32, ORC_UINT32, ORC_FLOAT, ORC_INT64, ORC_UINT64, ORC_DOUBLE};
  for (size_t c = 0; c < sizeof cand / sizeof cand[0]; ++c)
    if (contains(cand[c], a) && contains(cand[c], b)) return cand[c];
  /* nothing keeps both (64-bit integers with floats or with the other signedness):
   * the paper's stated exception is double precision */
  return ORC_DOUBLE;
}

int orc_promote(int a, int b) {
  if (!valid_dtype(a) || !valid_dtype(b)) return ORC_ERR_DTYPE;
  if (kind_of(a) == K_CPLX || kind_of(b) == K_CPLX) {
    int r = promote_real(real_part_type(a), real_part_type(b));
    if (kind_of(r) != K_REAL) r = ORC_HALF; /* cannot happen: a complex part is a float */
    return complex_of(r);
  }
  return promote_real(a, b);
}

/* ------------------------------------------------------------------------------------ */
/* arithmetic in a compute type                                                         */
/* ------------------------------------------------------------------------------------ */

/* wrap a 64-bit pattern to a signed integer of the given width */
static int64_t wrap_s(uint64_t x, int bits) {
  if (bits == 64) return (int64_t)x;
  uint64_t m = ((uint64_t)1 << bits) - 1;
  x &= m;
  if (x >> (bits - 1)) x |= ~m;
  return (int64_t)x;
}
static uint64_t wrap_u(uint64_t x, int bits) { return bits == 64 ? x : (x & (((uint64_t)1 << bits) - 1)); }

/* The arithmetic type of a floating compute type: half-precision types are evaluated in
 * single precision and rounded once when stored. */
typedef enum { A_F32, A_F64 } arith_t;
static arith_t arith_of(int dt) {
  int r = real_part_type(dt);
  return r == ORC_DOUBLE ? A_F64 : A_F32;
}

/* one rounding per operation in the arithmetic type */
static double r_add(arith_t t, double a, double b) { return t == A_F64 ? a + b : (double)((float)a + (float)b); }
static double r_sub(arith_t t, double a, double b) { return t == A_F64 ? a - b : (double)((float)a - (float)b); }
static double r_mul(arith_t t, double a, double b) { return t == A_F64 ? a * b : (double)((float)a * (float)b); }
static double r_div(arith_t t, double a, double b) { return t == A_F64 ? a / b : (double)((float)a / (float)b); }
static double r_sqrt(arith_t t, double a) { return t == A_F64 ? sqrt(a) : (double)sqrtf((float)a); }

/* NaN-propagating min/max; +0 ranks above -0 so the result does not depend on order */
static double real_max(double a, double b) {
  if (isnan(a)) return a;
  if (isnan(b)) return b;
  if (a > b) return a;
  if (b > a) return b;
  return signbit(a) ? b : a; /* equal: prefer the one without a sign bit */
}
static double real_min(double a, double b) {
  if (isnan(a)) return a;
  if (isnan(b)) return b;
  if (a < b) return a;
  if (b < a) return b;
  return signbit(a) ? a : b;
}

static int is_arith_binary(int op) { return op >= ORC_B_ADD && op <= ORC_B_MAX; }
static int is_bitwise_binary(int op) { return op >= ORC_B_BAND && op <= ORC_B_BXOR; }
static int is_logical_binary(int op) { return op >= ORC_B_LAND && op <= ORC_B_LXOR; }
static int is_compare_binary(int op) { return op >= ORC_B_EQ && op <= ORC_B_ABSGT; }

/* is (op, compute type T) defined? */
static int binary_supported(int op, int T) {
  kind_t k = kind_of(T);
  if (is_arith_binary(op)) {
    if (k == K_BOOL) return 0;
    if (k == K_CPLX && (op == ORC_B_MIN || op == ORC_B_MAX)) return 0;
    return 1;
  }
  if (is_bitwise_binary(op)) return k == K_BOOL || k == K_SINT || k == K_UINT;
  if (is_logical_binary(op)) return 1;
  if (op == ORC_B_EQ || op == ORC_B_NE || op == ORC_B_ABSGT) return 1;
  if (op >= ORC_B_LT && op <= ORC_B_GE) return k != K_CPLX;
  return 0;
}

/* a, b already converted to T; returns a value of T's kind (arithmetic/bitwise) or a bool */
static val_t apply_binary(int op, int T, val_t a, val_t b) {
  val_t r;
  memset(&r, 0, sizeof r);
  kind_t k = kind_of(T);
  if (is_logical_binary(op)) { /* T is bool */
    r.k = K_BOOL;
    r.i = op == ORC_B_LAND ? (a.i && b.i) : (op == ORC_B_LOR ? (a.i || b.i) : (a.i != b.i));
    return r;
  }
  if (is_compare_binary(op)) {
    r.k = K_BOOL;
    if (op == ORC_B_ABSGT) {
      switch (k) {
        case K_BOOL: r.i = a.i > b.i; break;
        case K_SINT: { /* |INT_MIN| fits in the unsigned type */
          uint64_t ma = a.i < 0 ? (uint64_t)0 - (uint64_t)a.i : (uint64_t)a.i;
          uint64_t mb = b.i < 0 ? (uint64_t)0 - (uint64_t)b.i : (uint64_t)b.i;
          r.i = ma > mb;
        } break;
        case K_UINT: r.i = a.u > b.u; break;
        case K_REAL: r.i = fabs(a.re) > fabs(b.re); break; /* false when either is NaN */
        case K_CPLX: { /* squared magnitudes in double precision, one rounding per operation */
          double ma = a.re * a.re + a.im * a.im;
          double mb = b.re * b.re + b.im * b.im;
          r.i = ma > mb;
        } break;
      }
      return r;
    }
    int lt = 0, eq = 0, unordered = 0;
    switch (k) {
      case K_BOOL: case K_SINT: lt = a.i < b.i; eq = a.i == b.i; break;
      case K_UINT: lt = a.u < b.u; eq = a.u == b.u; break;
      case K_REAL: unordered = isnan(a.re) || isnan(b.re); lt = a.re < b.re; eq = a.re == b.re; break;
      case K_CPLX: eq = (a.re == b.re) && (a.im == b.im); break; /* only EQ / NE reach here */
    }
    switch (op) {
      case ORC_B_EQ: r.i = eq; break;
      case ORC_B_NE: r.i = !eq; break;
      case ORC_B_LT: r.i = lt; break;
      case ORC_B_LE: r.i = !unordered && (lt || eq); break;
      case ORC_B_GT: r.i = !unordered && !lt && !eq; break;
      case ORC_B_GE: r.i = !unordered && !lt; break;
    }
    return r;
  }
  r.k = k;
  if (is_bitwise_binary(op)) {
    if (k == K_UINT) {
      r.u = op == ORC_B_BAND ? (a.u & b.u) : (op == ORC_B_BOR ? (a.u | b.u) : (a.u ^ b.u));
    } else { /* bool and signed: two's complement patterns; the result stays in range */
      r.i = op == ORC_B_BAND ? (a.i & b.i) : (op == ORC_B_BOR ? (a.i | b.i) : (a.i ^ b.i));
    }
    return r;
  }
  /* arithmetic */
  switch (k) {
    case K_BOOL: break; /* rejected earlier */
    case K_SINT: {
      int bits = int_bits(T);
      uint64_t x = (uint64_t)a.i, y = (uint64_t)b.i;
      switch (op) {
        case ORC_B_ADD: r.i = wrap_s(x + y, bits); break;
        case ORC_B_SUB: r.i = wrap_s(x - y, bits); break;
        case ORC_B_MUL: r.i = wrap_s(x * y, bits); break;
        case ORC_B_DIV: /* truncating; x/0 = 0; the one overflowing quotient wraps */
          if (b.i == 0) r.i = 0;
          else if (b.i == -1) r.i = wrap_s((uint64_t)0 - x, bits);
          else r.i = a.i / b.i;
          break;
        case ORC_B_MIN: r.i = a.i < b.i ? a.i : b.i; break;
        case ORC_B_MAX: r.i = a.i > b.i ? a.i : b.i; break;
      }
    } break;
    case K_UINT: {
      int bits = int_bits(T);
      switch (op) {
        case ORC_B_ADD: r.u = wrap_u(a.u + b.u, bits); break;
        case ORC_B_SUB: r.u = wrap_u(a.u - b.u, bits); break;
        case ORC_B_MUL: r.u = wrap_u(a.u * b.u, bits); break;
        case ORC_B_DIV: r.u = b.u == 0 ? 0 : a.u / b.u; break;
        case ORC_B_MIN: r.u = a.u < b.u ? a.u : b.u; break;
        case ORC_B_MAX: r.u = a.u > b.u ? a.u : b.u; break;
      }
    } break;
    case K_REAL: {
      arith_t t = arith_of(T);
      switch (op) {
        case ORC_B_ADD: r.re = r_add(t, a.re, b.re); break;
        case ORC_B_SUB: r.re = r_sub(t, a.re, b.re); break;
        case ORC_B_MUL: r.re = r_mul(t, a.re, b.re); break;
        case ORC_B_DIV: r.re = r_div(t, a.re, b.re); break;
        case ORC_B_MIN: r.re = real_min(a.re, b.re); break;
        case ORC_B_MAX: r.re = real_max(a.re, b.re); break;
      }
    } break;
    case K_CPLX: {
      arith_t t = arith_of(T);
      switch (op) {
        case ORC_B_ADD: r.re = r_add(t, a.re, b.re); r.im = r_add(t, a.im, b.im); break;
        case ORC_B_SUB: r.re = r_sub(t, a.re, b.re); r.im = r_sub(t, a.im, b.im); break;
        case ORC_B_MUL: /* (a+bi)(c+di) = (ac - bd) + (ad + bc)i, six roundings, no FMA */
          r.re = r_sub(t, r_mul(t, a.re, b.re), r_mul(t, a.im, b.im));
          r.im = r_add(t, r_mul(t, a.re, b.im), r_mul(t, a.im, b.re));
          break;
        case ORC_B_DIV: { /* textbook quotient: numerator times conjugate over |b|^2 */
          double den = r_add(t, r_mul(t, b.re, b.re), r_mul(t, b.im, b.im));
          double nre = r_add(t, r_mul(t, a.re, b.re), r_mul(t, a.im, b.im));
          double nim = r_sub(t, r_mul(t, a.im, b.re), r_mul(t, a.re, b.im));
          r.re = r_div(t, nre, den);
          r.im = r_div(t, nim, den);
        } break;
      }
    } break;
  }
  return r;
}

static int unary_supported(int op, int T) {
  kind_t k = kind_of(T);
  switch (op) {
    case ORC_U_IDENT: case ORC_U_CONJ: case ORC_U_LNOT: return 1;
    case ORC_U_NEG: return k != K_BOOL;
    case ORC_U_ABS: return k != K_BOOL; /* complex: the modulus, a real value (tolerance class) */
    case ORC_U_BNOT: return k == K_BOOL || k == K_SINT || k == K_UINT;
    case ORC_U_BSWAP: return k == K_BOOL || k == K_SINT || k == K_UINT;
    case ORC_U_SQRT: return k == K_REAL || k == K_CPLX;
    case ORC_U_SIN: case ORC_U_COS: case ORC_U_TAN: case ORC_U_EXP: case ORC_U_LOG:
      return k == K_REAL || k == K_CPLX;
    case ORC_U_ASIN: case ORC_U_ACOS: case ORC_U_ATAN: case ORC_U_SINH: case ORC_U_COSH: case ORC_U_TANH:
      return k == K_REAL || k == K_CPLX;
    default: return 0;
  }
}

/* Elementary functions that are not exactly representable (section 3.2: trigonometric
 * operations on all real and complex floating-point types; the paper gives no accuracy).
 * Reading: the value of the C library's double-precision routine (principal branches for the
 * complex ones), rounded once to the arithmetic type of T - single precision for half and
 * float types, double otherwise.  The kernels are held to a few units in the last place of
 * this value, not to its bits. */
static double round_arith(arith_t t, double y) { return t == A_F64 ? y : (double)(float)y; }

static val_t apply_elementary(int op, int T, val_t a) {
  val_t r = a;
  arith_t t = arith_of(T);
  if (kind_of(T) == K_REAL) {
    double y = 0;
    switch (op) {
      case ORC_U_SIN: y = sin(a.re); break;
      case ORC_U_COS: y = cos(a.re); break;
      case ORC_U_TAN: y = tan(a.re); break;
      case ORC_U_EXP: y = exp(a.re); break;
      case ORC_U_LOG: y = log(a.re); break;
      case ORC_U_ASIN: y = asin(a.re); break;
      case ORC_U_ACOS: y = acos(a.re); break;
      case ORC_U_ATAN: y = atan(a.re); break;
      case ORC_U_SINH: y = sinh(a.re); break;
      case ORC_U_COSH: y = cosh(a.re); break;
      case ORC_U_TANH: y = tanh(a.re); break;
    }
    r.re = round_arith(t, y);
  } else {
    double complex z = CMPLX(a.re, a.im), w = z;
    switch (op) {
      case ORC_U_SIN: w = csin(z); break;
      case ORC_U_COS: w = ccos(z); break;
      case ORC_U_TAN: w = ctan(z); break;
      case ORC_U_EXP: w = cexp(z); break;
      case ORC_U_LOG: w = clog(z); break;
      case ORC_U_SQRT: w = csqrt(z); break;
      case ORC_U_ASIN: w = casin(z); break;
      case ORC_U_ACOS: w = cacos(z); break;
      case ORC_U_ATAN: w = catan(z); break;
      case ORC_U_SINH: w = csinh(z); break;
      case ORC_U_COSH: w = ccosh(z); break;
      case ORC_U_TANH: w = ctanh(z); break;
    }
    r.re = round_arith(t, creal(w));
    r.im = round_arith(t, cimag(w));
  }
  return r;
}

static val_t apply_unary(int op, int T, val_t a) {
  val_t r = a;
  kind_t k = kind_of(T);
  int bits = int_bits(T);
  switch (op) {
    case ORC_U_IDENT: break;
    case ORC_U_NEG:
      if (k == K_SINT) r.i = wrap_s((uint64_t)0 - (uint64_t)a.i, bits);
      else if (k == K_UINT) r.u = wrap_u((uint64_t)0 - a.u, bits);
      else { r.re = -a.re; if (k == K_CPLX) r.im = -a.im; }
      break;
    case ORC_U_ABS:
      if (k == K_SINT) r.i = a.i < 0 ? wrap_s((uint64_t)0 - (uint64_t)a.i, bits) : a.i;
      else if (k == K_REAL) r.re = fabs(a.re);
      else if (k == K_CPLX) { /* the modulus: a real value of the same precision, without undue
                                 overflow or underflow (the C library's cabs), rounded once */
        r.k = K_REAL;
        r.re = round_arith(arith_of(T), cabs(CMPLX(a.re, a.im)));
        r.im = 0;
      }
      break;
    case ORC_U_CONJ:
      if (k == K_CPLX) r.im = -a.im;
      break;
    case ORC_U_LNOT: /* T is bool */
      r.i = !a.i;
      break;
    case ORC_U_BNOT:
      if (k == K_BOOL) r.i = !a.i;
      else if (k == K_SINT) r.i = ~a.i; /* stays in range */
      else r.u = wrap_u(~a.u, bits);
      break;
    case ORC_U_BSWAP: { /* section 3.1.3: data in the other byte order; reverse the element's bytes */
      int nbytes = k == K_BOOL ? 1 : bits / 8;
      uint64_t x = k == K_UINT ? a.u : (uint64_t)a.i, y = 0;
      for (int b = 0; b < nbytes; ++b) y |= ((x >> (8 * b)) & 0xff) << (8 * (nbytes - 1 - b));
      if (k == K_UINT) r.u = y;
      else if (k == K_SINT) r.i = wrap_s(y, bits);
      else r.i = a.i;
    } break;
    case ORC_U_SQRT:
      if (k == K_CPLX) return apply_elementary(op, T, a);
      r.re = r_sqrt(arith_of(T), a.re);
      break;
    case ORC_U_SIN: case ORC_U_COS: case ORC_U_TAN: case ORC_U_EXP: case ORC_U_LOG:
    case ORC_U_ASIN: case ORC_U_ACOS: case ORC_U_ATAN: case ORC_U_SINH: case ORC_U_COSH: case ORC_U_TANH:
      return apply_elementary(op, T, a);
  }
  return r;
}

/* ------------------------------------------------------------------------------------ */
/* descriptors                                                                          */
/* ------------------------------------------------------------------------------------ */

static int check_tensor(const orc_tensor *t) {
  if (!t) return ORC_ERR_NULLPTR;
  if (!valid_dtype(t->dtype)) return ORC_ERR_DTYPE;
  if (t->ndim < 0 || t->ndim > ORC_MAX_DIMS) return ORC_ERR_NDIM;
  for (int d = 0; d < t->ndim; ++d)
    if (t->size[d] < 0) return ORC_ERR_SHAPE;
  return ORC_OK;
}

static int64_t numel(const orc_tensor *t) {
  int64_t n = 1;
  for (int d = 0; d < t->ndim; ++d) n *= t->size[d];
  return n;
}

/* input dims, right-aligned against out, must equal out's or be 1 */
static int check_broadcast(const orc_tensor *in, const orc_tensor *out) {
  if (in->ndim > out->ndim) return ORC_ERR_SHAPE;
  int lead = out->ndim - in->ndim;
  for (int d = 0; d < in->ndim; ++d)
    if (in->size[d] != out->size[lead + d] && in->size[d] != 1) return ORC_ERR_SHAPE;
  return ORC_OK;
}

/* multi-index of out (row-major decode of a linear index) */
static void decode(int64_t lin, const orc_tensor *out, int64_t *idx) {
  for (int d = out->ndim - 1; d >= 0; --d) {
    idx[d] = lin % out->size[d];
    lin /= out->size[d];
  }
}

static unsigned char *addr_out(const orc_tensor *t, const int64_t *idx) {
  int64_t off = t->offset;
  for (int d = 0; d < t->ndim; ++d) off += idx[d] * t->stride[d];
  return (unsigned char *)t->base + off;
}

/* address in a broadcast input for out's multi-index */
static const unsigned char *addr_in(const orc_tensor *in, const orc_tensor *out, const int64_t *idx) {
  int lead = out->ndim - in->ndim;
  int64_t off = in->offset;
  for (int d = 0; d < in->ndim; ++d) {
    int64_t i = in->size[d] == 1 ? 0 : idx[lead + d];
    off += i * in->stride[d];
  }
  return (const unsigned char *)in->base + off;
}

/* ------------------------------------------------------------------------------------ */
/* elementwise entry points                                                             */
/* ------------------------------------------------------------------------------------ */

int orc_binary(int op, const orc_tensor *a, const orc_tensor *b, const orc_tensor *out,
               uint32_t flags) {
  int rc;
  if ((rc = check_tensor(a)) || (rc = check_tensor(b)) || (rc = check_tensor(out))) return rc;
  if (op < 0 || op >= ORC_NUM_BINARY) return ORC_ERR_OP;
  if ((rc = check_broadcast(a, out)) || (rc = check_broadcast(b, out))) return rc;
  if ((flags & ORC_STRICT_TYPES) && a->dtype != b->dtype) return ORC_ERR_DTYPE;
  int T;
  if (is_logical_binary(op)) T = ORC_BOOL;
  else if (is_compare_binary(op)) T = orc_promote(a->dtype, b->dtype);
  else {
    /* Section 3.2.1: the operation's type comes from the operands (the smallest type that
       holds both).  A destination that is one of the operands' types (the A += B case) or
       that holds the promoted type takes the operands into its own type; any other
       destination receives the promoted-type result, converted once on store. */
    int P = orc_promote(a->dtype, b->dtype);
    if (out->dtype == a->dtype || out->dtype == b->dtype || orc_promote(P, out->dtype) == out->dtype)
      T = out->dtype;
    else
      T = P;
  }
  if ((flags & ORC_STRICT_TYPES) && !is_compare_binary(op) && !is_logical_binary(op) &&
      a->dtype != out->dtype)
    return ORC_ERR_DTYPE;
  if (!binary_supported(op, T)) return ORC_ERR_DTYPE;
  int64_t n = numel(out);
#pragma omp parallel for schedule(static)
  for (int64_t lin = 0; lin < n; ++lin) {
    int64_t idx[ORC_MAX_DIMS];
    decode(lin, out, idx);
    val_t va = convert(load_tensor_elem(a, addr_in(a, out, idx)), T);
    val_t vb = convert(load_tensor_elem(b, addr_in(b, out, idx)), T);
    val_t r = apply_binary(op, T, va, vb);
    store_tensor_elem(out, addr_out(out, idx), convert(r, out->dtype));
  }
  return ORC_OK;
}

int orc_unary(int op, const orc_tensor *a, const orc_tensor *out, uint32_t flags) {
  int rc;
  if ((rc = check_tensor(a)) || (rc = check_tensor(out))) return rc;
  if (op < 0 || op >= ORC_NUM_UNARY) return ORC_ERR_OP;
  if ((rc = check_broadcast(a, out))) return rc;
  /* compute type: the output's; bool for the logical not; the modulus of a complex tensor is
   * evaluated in that tensor's own type (its result is the real type of the same precision) */
  int T = op == ORC_U_LNOT ? ORC_BOOL : out->dtype;
  if (op == ORC_U_ABS && kind_of(a->dtype) == K_CPLX) T = a->dtype;
  if ((flags & ORC_STRICT_TYPES) && op != ORC_U_LNOT && a->dtype != out->dtype &&
      !(op == ORC_U_ABS && kind_of(a->dtype) == K_CPLX && out->dtype == real_part_type(a->dtype)))
    return ORC_ERR_DTYPE;
  if (!unary_supported(op, T)) return ORC_ERR_DTYPE;
  int64_t n = numel(out);
#pragma omp parallel for schedule(static)
  for (int64_t lin = 0; lin < n; ++lin) {
    int64_t idx[ORC_MAX_DIMS];
    decode(lin, out, idx);
    val_t va = convert(load_tensor_elem(a, addr_in(a, out, idx)), T);
    val_t r = apply_unary(op, T, va);
    store_tensor_elem(out, addr_out(out, idx), convert(r, out->dtype));
  }
  return ORC_OK;
}

int orc_cast_copy(const orc_tensor *src, const orc_tensor *dst) {
  return orc_unary(ORC_U_IDENT, src, dst, 0);
}

/* ------------------------------------------------------------------------------------ */
/* reductions                                                                           */
/* ------------------------------------------------------------------------------------ */

/* compensated (Neumaier) summation state for double-precision inputs */
typedef struct { double s, c; } nsum_t;
static void nsum_add(nsum_t *a, double x) {
  double t = a->s + x;
  if (fabs(a->s) >= fabs(x)) a->c += (a->s - t) + x;
  else a->c += (x - t) + a->s;
  a->s = t;
}
static double nsum_value(const nsum_t *a) { return a->s + a->c; }

static int reduce_supported(int op, int dt) {
  kind_t k = kind_of(dt);
  switch (op) {
    case ORC_R_SUM: case ORC_R_ANY: case ORC_R_ALL: return 1;
    case ORC_R_PROD: case ORC_R_MIN: case ORC_R_MAX: return k != K_CPLX;
    default: return 0;
  }
}

int orc_reduce(int op, const orc_tensor *a, const int32_t *axes, int32_t naxes,
               const orc_tensor *out) {
  int rc;
  if ((rc = check_tensor(a)) || (rc = check_tensor(out))) return rc;
  if (op < 0 || op >= ORC_NUM_REDUCE) return ORC_ERR_OP;
  if (naxes < 0 || naxes > a->ndim) return ORC_ERR_SHAPE;
  if (naxes > 0 && !axes) return ORC_ERR_NULLPTR;
  int reduced[ORC_MAX_DIMS] = {0};
  for (int i = 0; i < naxes; ++i) {
    if (axes[i] < 0 || axes[i] >= a->ndim || reduced[axes[i]]) return ORC_ERR_SHAPE;
    reduced[axes[i]] = 1;
  }
  if (out->ndim != a->ndim - naxes) return ORC_ERR_SHAPE;
  /* kept dims of a, in order, must match out */
  int kept_dim[ORC_MAX_DIMS], red_dim[ORC_MAX_DIMS], nk = 0, nr = 0;
  for (int d = 0; d < a->ndim; ++d) {
    if (reduced[d]) red_dim[nr++] = d; else kept_dim[nk++] = d;
  }
  for (int j = 0; j < nk; ++j)
    if (out->size[j] != a->size[kept_dim[j]]) return ORC_ERR_SHAPE;
  if (!reduce_supported(op, a->dtype)) return ORC_ERR_DTYPE;
  int64_t nred = 1;
  for (int j = 0; j < nr; ++j) nred *= a->size[red_dim[j]];
  int64_t nout = numel(out);
  if ((op == ORC_R_MIN || op == ORC_R_MAX) && nred == 0 && nout > 0) return ORC_ERR_EMPTY;

  kind_t ka = kind_of(a->dtype);
  int in_is_double = real_part_type(a->dtype) == ORC_DOUBLE;

#pragma omp parallel for schedule(static)
  for (int64_t lin = 0; lin < nout; ++lin) {
    int64_t oidx[ORC_MAX_DIMS], aidx[ORC_MAX_DIMS];
    decode(lin, out, oidx);
    for (int j = 0; j < nk; ++j) aidx[kept_dim[j]] = oidx[j];

    /* wide accumulators */
    uint64_t acc_i = (op == ORC_R_PROD) ? 1 : 0;    /* 64-bit wrapping, signed or unsigned */
    double acc_re = (op == ORC_R_PROD) ? 1.0 : 0.0; /* fp64 for half / float inputs */
    double acc_im = 0.0;
    nsum_t ns_re = {0.0, 0.0}, ns_im = {0.0, 0.0};  /* compensated, for double inputs */
    int acc_b = (op == ORC_R_ALL) ? 1 : 0;
    val_t best;
    memset(&best, 0, sizeof best);
    int have_best = 0;

    for (int64_t r = 0; r < nred; ++r) {
      /* row-major decode of the reduced index over the reduced dims, in order */
      int64_t t = r;
      for (int j = nr - 1; j >= 0; --j) {
        aidx[red_dim[j]] = t % a->size[red_dim[j]];
        t /= a->size[red_dim[j]];
      }
      int64_t off = a->offset;
      for (int d = 0; d < a->ndim; ++d) off += aidx[d] * a->stride[d];
      val_t v = load_tensor_elem(a, (const unsigned char *)a->base + off);
      switch (op) {
        case ORC_R_SUM:
          if (ka == K_BOOL || ka == K_SINT) acc_i += (uint64_t)v.i;
          else if (ka == K_UINT) acc_i += v.u;
          else if (in_is_double) { nsum_add(&ns_re, v.re); if (ka == K_CPLX) nsum_add(&ns_im, v.im); }
          else { acc_re += v.re; if (ka == K_CPLX) acc_im += v.im; }
          break;
        case ORC_R_PROD:
          if (ka == K_BOOL || ka == K_SINT) acc_i *= (uint64_t)v.i;
          else if (ka == K_UINT) acc_i *= v.u;
          else acc_re *= v.re;
          break;
        case ORC_R_MIN: case ORC_R_MAX:
          if (!have_best) { best = v; have_best = 1; break; }
          if (ka == K_BOOL || ka == K_SINT) {
            if (op == ORC_R_MIN ? v.i < best.i : v.i > best.i) best = v;
          } else if (ka == K_UINT) {
            if (op == ORC_R_MIN ? v.u < best.u : v.u > best.u) best = v;
          } else {
            best.re = op == ORC_R_MIN ? real_min(best.re, v.re) : real_max(best.re, v.re);
          }
          break;
        case ORC_R_ANY: case ORC_R_ALL: {
          int nz = convert(v, ORC_BOOL).i != 0;
          if (op == ORC_R_ANY) acc_b = acc_b || nz; else acc_b = acc_b && nz;
        } break;
      }
    }

    val_t res;
    memset(&res, 0, sizeof res);
    switch (op) {
      case ORC_R_SUM: case ORC_R_PROD:
        if (ka == K_BOOL || ka == K_SINT) { res.k = K_SINT; res.i = (int64_t)acc_i; }
        else if (ka == K_UINT) { res.k = K_UINT; res.u = acc_i; }
        else {
          res.k = ka;
          if (op == ORC_R_SUM && in_is_double) { res.re = nsum_value(&ns_re); res.im = nsum_value(&ns_im); }
          else { res.re = acc_re; res.im = acc_im; }
        }
        break;
      case ORC_R_MIN: case ORC_R_MAX: res = best; break;
      default: res.k = K_BOOL; res.i = acc_b; break;
    }
    store_tensor_elem(out, addr_out(out, oidx), convert(res, out->dtype));
  }
  return ORC_OK;
}
