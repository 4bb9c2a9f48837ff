// Which (operation, operand dtypes) combinations get a dtype-specialised elementwise kernel,
// and the per-lane vector shape those kernels use.  Everything else runs through the
// generic-dtype kernel, which converts through runtime switches.  Shared by the host planner
// (to report and size launches) and the kernel translation units (to instantiate).
#pragma once

#include "dtypes.hpp"

namespace ocn {


// compute type of a binary operation (section 3.2.1 of the paper and include/ocn.h)
// Logical operations run in bool, comparisons in the operands' promoted type.  Arithmetic and
// bitwise operations run in the destination's type when that is one of the operands' types
// (the A += B case) or holds the promoted type (`widened` = promote(promoted, so)); any other
// destination receives the promoted-type result, converted once on store.
OCN_HD constexpr int binary_compute_dtype(int op, int sa, int sb, int so, int promoted, int widened) {
  if (is_logical(op)) return (int)DT_BOOL;
  if (is_compare(op)) return promoted;
  return (so == sa || so == sb || widened == so) ? so : promoted;
}

// Mixed input types whose +, -, *, / get kernels that convert on load (section 3.2.1: operands
// of different types are converted to a common one): an integer or narrower float with a
// float, either with a double, a real with a complex, in both operand orders, computed in the
// output type.
struct MixedPair { int sa, sb, so; };
constexpr MixedPair kMixedPairs[] = {
    {DT_I32, DT_F32, DT_F32}, {DT_F32, DT_I32, DT_F32}, {DT_F16, DT_F32, DT_F32}, {DT_F32, DT_F16, DT_F32},
    {DT_F32, DT_F64, DT_F64}, {DT_F64, DT_F32, DT_F64}, {DT_I32, DT_F64, DT_F64}, {DT_F64, DT_I32, DT_F64},
    {DT_I64, DT_F64, DT_F64}, {DT_F64, DT_I64, DT_F64}, {DT_F32, DT_C32, DT_C32}, {DT_C32, DT_F32, DT_C32},
    {DT_F64, DT_C64, DT_C64}, {DT_C64, DT_F64, DT_C64}};
constexpr int kNumMixedPairs = (int)(sizeof(kMixedPairs) / sizeof(kMixedPairs[0]));
constexpr int kNumMixedOps = 4;  // B_ADD, B_SUB, B_MUL, B_DIV
static_assert(B_ADD == 0 && B_DIV == 3, "the mixed-type kernels cover the first four binary operations");

OCN_HD constexpr bool mixed_arith_specialised(int op, int sa, int sb, int so) {
  if (op < 0 || op >= kNumMixedOps) return false;
  for (int k = 0; k < kNumMixedPairs; ++k)
    if (kMixedPairs[k].sa == sa && kMixedPairs[k].sb == sb && kMixedPairs[k].so == so) return true;
  return false;
}

OCN_HD constexpr bool binary_specialised(int op, int sa, int sb, int so) {
  if (op < 0 || op >= B_COUNT) return false;
  if (is_arith(op) || is_bitwise(op)) {
    if (!binary_supported(op, so)) return false;
    if (sa == so && sb == so) return true;
    return mixed_arith_specialised(op, sa, sb, so);
  }
  if (is_logical(op)) return sa == DT_BOOL && sb == DT_BOOL && so == DT_BOOL;
  // comparisons: equal input types (so the compute type is that type), bool result
  return sa == sb && so == DT_BOOL && binary_supported(op, sa);
}

// compute type of a unary operation: the output's type; bool for the logical not; the modulus
// of a complex tensor is evaluated in that tensor's own type (and is a real value)
OCN_HD constexpr int unary_compute_dtype(int op, int sa, int so) {
  return op == U_LNOT ? (int)DT_BOOL : (op == U_ABS && dt_kind(sa) == K_CPLX) ? sa : so;
}

OCN_HD constexpr bool unary_specialised(int op, int sa, int so) {
  if (op < 0 || op >= U_COUNT) return false;
  if (op == U_IDENT) return true;  // the full cast matrix
  if (op == U_LNOT) return sa == DT_BOOL && so == DT_BOOL;
  if (op == U_ABS && dt_kind(sa) == K_CPLX) return so == dt_real_of(sa);  // complex -> its real type
  return sa == so && unary_supported(op, so);
}

// Reductions of an elementwise result that get a fused kernel: equal input types; sums of
// a + b, a - b, a * b in that type; sums (counts), any and all of ==, <, >, |a| > |b|.
OCN_HD constexpr bool fused_specialised(int ew_op, int sa, int sb, int mid, int red_op) {
  if (sa != sb || ew_op < 0 || ew_op >= B_COUNT) return false;
  if (ew_op == B_ADD || ew_op == B_SUB || ew_op == B_MUL) {
    if (mid != sa || red_op != R_SUM) return false;
    return sa == DT_I32 || sa == DT_I64 || sa == DT_F16 || sa == DT_F32 || sa == DT_F64 || sa == DT_C32 ||
           sa == DT_C64;
  }
  if (ew_op == B_EQ || ew_op == B_LT || ew_op == B_GT || ew_op == B_ABSGT) {
    if (mid != DT_BOOL || !(red_op == R_SUM || red_op == R_ANY || red_op == R_ALL)) return false;
    if (sa == DT_C32) return ew_op == B_EQ || ew_op == B_ABSGT;
    return sa == DT_I32 || sa == DT_F32 || sa == DT_F64;
  }
  return false;
}

OCN_HD constexpr int imin(int a, int b) { return a < b ? a : b; }
OCN_HD constexpr int imax(int a, int b) { return a > b ? a : b; }

// Elements per lane access of the elementwise kernels: the output moves 16 bytes, so that
// every store instruction of a wavefront writes whole cache lines (a wider output vector
// would be written in several instructions of 16 bytes at a lane stride of the whole vector,
// i.e. in partial lines, which streaming stores do at a fraction of the rate), unless that
// would make the widest input move more than 64 bytes.  Inputs narrower than the output are
// read with accordingly narrower loads.
OCN_HD constexpr int rows_vec(int es_out, int es_max) {
  return imax(1, imin(16 / es_out, 64 / es_max));
}
// Vectors per lane, so that about 64 bytes of the widest operand are in flight per lane.
#ifndef OCN_ROWS_MAXU
#define OCN_ROWS_MAXU 4
#endif
OCN_HD constexpr int rows_unroll(int vec, int es_max) {
  return imax(1, imin(OCN_ROWS_MAXU, 64 / (vec * es_max)));
}

// The rows kernel's own choice.  Every operand moves ONE piece of at most 16 bytes per lane
// and vector, the widest exactly 16, so that the lanes of a wavefront cover whole cache lines
// of every operand with a single instruction each - the access shape that streaming
// (non-temporal) loads and stores need (a double -> int16 cast of 16 Mi elements: 28.8 us with
// 64-byte inputs and 16-byte outputs per lane, 27.1 us with 16-byte inputs and 4-byte outputs).
// A narrow operand still moves at least 4 bytes where the output's 16-byte limit allows it;
// the wide one then takes several pieces and is read without the hint.
OCN_HD constexpr int rows_stream_vec(int es_out, int es_min, int es_max) {
  return imax(1, imin(16 / es_out, imax(16 / es_max, 4 / es_min)));
}
// Vectors per lane: as many as it takes for the narrowest operand to move 16 bytes per lane
// as well (at most four).  Operations on equal widths run fastest with one vector per lane
// and as many workgroups as that takes (int32 x float over 2^26 elements: 88.3 us, against 91.2
// with two and 96 with four); a double -> int16 cast, whose stores are 4 bytes wide, gains
// from four (29.0 us against 29.6 with two and 30.5 with one).
OCN_HD constexpr int rows_stream_unroll(int vec, int es_min) {
  return imax(1, imin(4, 16 / (vec * es_min)));
}

}  // namespace ocn
