/*
 * CPU oracle for the strided tensor engine: TEST INFRASTRUCTURE ONLY.
 *
 * A deliberately plain, slow, per-element evaluation of what the engine computes, written
 * from the tensor model of the Ocean Tensor Package paper (section 3.1.3 "Tensors":
 * data type, at most eight dimensions, general byte strides; section 3.2.1 "Type casting";
 * section 3.2 "Tensor operations": elementwise arithmetic, type casting, reductions along
 * one or more axes; section 4: broadcasting and views through strides).  It never sorts,
 * merges or otherwise rewrites dimensions, and it shares no source, header, table or helper
 * with the GPU library.  Only the tests, the smoke check and the benchmark's CPU-baseline
 * leg may call it; the product never does.
 *
 * All pointers are HOST memory.  Every function returns 0 on success and a negative
 * ORC_ERR_* value otherwise; on error nothing is written.
 *
 * Parity status: the paper prints no numeric results for these operations, so parity with
 * the paper's own implementation is unpinned everywhere; each function below is pinned by
 * the tests under tests/ (marked "not gpu") against closed forms, brute force in exact
 * rational arithmetic, numpy library routines on special cases, and invariants.
 */
#ifndef OCN_ORACLE_H
#define OCN_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ORC_MAX_DIMS 8 /* section 3.1.3: maximum number of tensor dimensions */

/* Element types (footnote of section 4): bool; 8..64-bit signed and unsigned integers;
 * real and complex half, single and double precision. */
enum {
  ORC_BOOL = 0, ORC_INT8, ORC_INT16, ORC_INT32, ORC_INT64,
  ORC_UINT8, ORC_UINT16, ORC_UINT32, ORC_UINT64,
  ORC_HALF, ORC_FLOAT, ORC_DOUBLE,
  ORC_CHALF, ORC_CFLOAT, ORC_CDOUBLE,
  ORC_NUM_DTYPES
};

/* A tensor is a typed, strided view on storage (sections 3.1.2 and 3.1.3).  Element
 * (i0,...,i{n-1}) lives at base + offset + sum_d i_d * stride[d]; strides are in BYTES and
 * may be zero (broadcast) or negative (reversed axis). */
typedef struct {
  void *base;
  int64_t offset;
  int32_t dtype, ndim;
  int64_t size[ORC_MAX_DIMS];
  int64_t stride[ORC_MAX_DIMS];
  int32_t device; /* ignored by the oracle */
  int32_t byteswapped; /* non-zero: the elements are stored in the other byte order (section
                          3.1.3: operations can be applied in either byte order): every scalar -
                          each component of a complex element - has its bytes reversed in memory */
} orc_tensor;

enum { /* unary operations */
  ORC_U_IDENT = 0, ORC_U_NEG, ORC_U_ABS, ORC_U_CONJ, ORC_U_LNOT, ORC_U_BNOT, ORC_U_SQRT,
  ORC_U_SIN, ORC_U_COS, ORC_U_TAN, ORC_U_EXP, ORC_U_LOG, ORC_U_BSWAP,
  ORC_U_ASIN, ORC_U_ACOS, ORC_U_ATAN, ORC_U_SINH, ORC_U_COSH, ORC_U_TANH,
  ORC_NUM_UNARY
};
enum { /* binary operations */
  ORC_B_ADD = 0, ORC_B_SUB, ORC_B_MUL, ORC_B_DIV, ORC_B_MIN, ORC_B_MAX,
  ORC_B_BAND, ORC_B_BOR, ORC_B_BXOR, ORC_B_LAND, ORC_B_LOR, ORC_B_LXOR,
  ORC_B_EQ, ORC_B_NE, ORC_B_LT, ORC_B_LE, ORC_B_GT, ORC_B_GE,
  ORC_B_ABSGT, /* |a| > |b| */
  ORC_NUM_BINARY
};
enum { /* reductions */
  ORC_R_SUM = 0, ORC_R_PROD, ORC_R_MIN, ORC_R_MAX, ORC_R_ANY, ORC_R_ALL,
  ORC_NUM_REDUCE
};

enum {
  ORC_OK = 0,
  ORC_ERR_NULLPTR = -1,
  ORC_ERR_DTYPE = -2,  /* bad dtype, unsupported op/dtype pair, strict-mode mismatch */
  ORC_ERR_NDIM = -3,
  ORC_ERR_SHAPE = -4,
  ORC_ERR_EMPTY = -10, /* min/max over zero elements */
  ORC_ERR_OP = -12
};

#define ORC_STRICT_TYPES 1u /* section 3.2.1: automatic type casting switched off */

/* out[i] = convert_out( f( convert_T( a[i] ) ) ), T chosen as in orc_binary. */
int orc_unary(int op, const orc_tensor *a, const orc_tensor *out, uint32_t flags);

/* out[i] = convert_out( g( convert_T(a[i]), convert_T(b[i]) ) ) for every index i of out.
 * Inputs broadcast against out: an input dimension of size 1 is read at index 0 whatever
 * its stride; inputs of lower rank are padded with leading size-1 dimensions.
 * T = out.dtype for arithmetic and bitwise operations; T = orc_promote(a.dtype, b.dtype)
 * for comparisons and ABSGT; T = bool for the logical operations. */
int orc_binary(int op, const orc_tensor *a, const orc_tensor *b, const orc_tensor *out,
               uint32_t flags);

/* dst[i] = convert(src[i]) (section 3.2.1, explicit type casting on one device). */
int orc_cast_copy(const orc_tensor *src, const orc_tensor *dst);

/* Reduction along the listed axes (section 3.2 lists reductions over one or several axes):
 * out has the kept dimensions of a in their original order. */
int orc_reduce(int op, const orc_tensor *a, const int32_t *axes, int32_t naxes,
               const orc_tensor *out);

/* Implicit-casting result type (section 3.2.1): the smallest type holding both. */
int orc_promote(int dtype_a, int dtype_b);

/* Element size in bytes, or 0 for an invalid dtype. */
int orc_dtype_size(int dtype);

/* Exposed for the tests that pin the half-precision conversions. */
double orc_half_bits_to_double(uint16_t h);
uint16_t orc_double_to_half_bits(double x);

#ifdef __cplusplus
}
#endif
#endif
