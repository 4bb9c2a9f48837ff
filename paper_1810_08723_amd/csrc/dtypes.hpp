// Element-type and operation facts shared by the host planner and the device code: the
// fifteen element types (footnote in section 4 of the paper), which operation is defined for
// which compute type, and the type an operation returns.  No HIP dependency.
#pragma once

#include <stdint.h>

#if defined(__HIPCC__)
#define OCN_HD __host__ __device__ inline
#else
#define OCN_HD inline
#endif

namespace ocn {

enum : int {
  DT_BOOL = 0, DT_I8, DT_I16, DT_I32, DT_I64, DT_U8, DT_U16, DT_U32, DT_U64,
  DT_F16, DT_F32, DT_F64, DT_C16, DT_C32, DT_C64, DT_COUNT
};

enum : int { K_BOOL = 0, K_SINT, K_UINT, K_REAL, K_CPLX };

OCN_HD constexpr int dt_kind(int dt) {
  return dt == DT_BOOL ? K_BOOL : dt <= DT_I64 ? K_SINT : dt <= DT_U64 ? K_UINT : dt <= DT_F64 ? K_REAL : K_CPLX;
}
OCN_HD constexpr int dt_size(int dt) {
  constexpr int s[DT_COUNT] = {1, 1, 2, 4, 8, 1, 2, 4, 8, 2, 4, 8, 4, 8, 16};
  return s[dt];
}
// real component type of a floating dtype
OCN_HD constexpr int dt_real_of(int dt) {
  return dt == DT_C16 ? DT_F16 : dt == DT_C32 ? DT_F32 : dt == DT_C64 ? DT_F64 : dt;
}

enum : int {  // numbering shared with the public header (checked by static_asserts in the API source)
  B_ADD = 0, B_SUB, B_MUL, B_DIV, B_MIN, B_MAX, B_BAND, B_BOR, B_BXOR, B_LAND, B_LOR, B_LXOR,
  B_EQ, B_NE, B_LT, B_LE, B_GT, B_GE, B_ABSGT, B_COUNT
};
enum : int { U_IDENT = 0, U_NEG, U_ABS, U_CONJ, U_LNOT, U_BNOT, U_SQRT, U_SIN, U_COS, U_TAN, U_EXP, U_LOG, U_BSWAP,
              U_ASIN, U_ACOS, U_ATAN, U_SINH, U_COSH, U_TANH, U_COUNT };
enum : int { R_SUM = 0, R_PROD, R_MIN, R_MAX, R_ANY, R_ALL, R_COUNT };

OCN_HD constexpr bool is_arith(int op) { return op >= B_ADD && op <= B_MAX; }
OCN_HD constexpr bool is_bitwise(int op) { return op >= B_BAND && op <= B_BXOR; }
OCN_HD constexpr bool is_logical(int op) { return op >= B_LAND && op <= B_LXOR; }
OCN_HD constexpr bool is_compare(int op) { return op >= B_EQ && op <= B_ABSGT; }

// is (binary op, compute type T) defined?
OCN_HD constexpr bool binary_supported(int op, int T) {
  const int k = dt_kind(T);
  if (is_arith(op)) return k != K_BOOL && !(k == K_CPLX && (op == B_MIN || op == B_MAX));
  if (is_bitwise(op)) return k == K_BOOL || k == K_SINT || k == K_UINT;
  if (is_logical(op)) return true;
  if (op == B_EQ || op == B_NE || op == B_ABSGT) return true;
  if (op >= B_LT && op <= B_GE) return k != K_CPLX;
  return false;
}
OCN_HD constexpr bool unary_supported(int op, int T) {
  const int k = dt_kind(T);
  switch (op) {
    case U_IDENT: case U_CONJ: case U_LNOT: return true;
    case U_NEG: return k != K_BOOL;
    case U_ABS: return k != K_BOOL;   // complex: the modulus, a real value
    case U_BNOT: case U_BSWAP: return k == K_BOOL || k == K_SINT || k == K_UINT;
    case U_SQRT: return k == K_REAL || k == K_CPLX;
    case U_SIN: case U_COS: case U_TAN: case U_EXP: case U_LOG: return k == K_REAL || k == K_CPLX;
    case U_ASIN: case U_ACOS: case U_ATAN: case U_SINH: case U_COSH: case U_TANH: return k == K_REAL || k == K_CPLX;
    default: return false;
  }
}
// result dtype of the operation itself (before conversion to the output type)
OCN_HD constexpr int binary_result_dtype(int op, int T) { return (is_arith(op) || is_bitwise(op)) ? T : DT_BOOL; }
OCN_HD constexpr int unary_result_dtype(int op, int T) {
  return op == U_LNOT ? (int)DT_BOOL : (op == U_ABS && dt_kind(T) == K_CPLX) ? dt_real_of(T) : T;
}


}  // namespace ocn
