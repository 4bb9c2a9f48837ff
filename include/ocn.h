/*
 * ocn - a strided n-dimensional tensor engine for AMD MI355X (gfx950).
 *
 * C ABI of the data-parallel core of the Ocean Tensor Package (van den Berg, arXiv
 * 1810.08723): elementwise unary and binary operations, type-casting copies and reductions
 * along one or more axes, over tensors described the way the paper describes them
 * (section 3.1.3 "Tensors": a data type, at most eight dimensions, sizes, general strides
 * given in bytes; section 3.1.2 "Storage": memory that may be provided by an external
 * source and carry several superimposed tensors of different types).
 *
 * Conventions common to every call
 *  - Every ocn_tensor::base is DEVICE memory owned by the caller.  The library never
 *    allocates, frees or keeps a pointer after a call returns.  Descriptor structs
 *    themselves are HOST memory and are only read during the call.
 *  - Element (i0,...,i{n-1}) of a view lives at base + offset + sum_d i_d * stride[d].
 *    Strides and offset are BYTES; a stride may be zero (broadcast) or negative (reversed
 *    axis).  offset and every stride must be a multiple of the scalar size of the dtype
 *    (for complex types, of its real component), and base + offset must be so aligned.
 *  - Work is enqueued on `stream` (a hipStream_t, or NULL for the default stream) and the
 *    call returns without waiting for it (section 3.1: operations are scheduled
 *    asynchronously on a stream).
 *  - Return value: OCN_OK (0) or a negative OCN_ERR_* code.  On error nothing is launched
 *    and no memory is written.  No exception crosses this boundary.
 *  - An output with zero elements makes the call a successful no-op.
 */
#ifndef OCN_H
#define OCN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define OCN_MAX_DIMS 8 /* section 3.1.3: the maximum number of tensor dimensions is eight */

/* Element types (footnote in section 4): booleans; 8, 16, 32 and 64-bit signed and unsigned
 * integers; real and complex half, single and double precision floating point.  A complex
 * element is the pair (re, im) of its real component type. */
typedef enum {
  OCN_BOOL = 0, OCN_INT8, OCN_INT16, OCN_INT32, OCN_INT64,
  OCN_UINT8, OCN_UINT16, OCN_UINT32, OCN_UINT64,
  OCN_HALF, OCN_FLOAT, OCN_DOUBLE,
  OCN_CHALF, OCN_CFLOAT, OCN_CDOUBLE,
  OCN_NUM_DTYPES
} ocn_dtype;

/* The paper's unified tensor type (sections 2.2 and 3.1.3) reduced to a plain descriptor. */
typedef struct {
  void *base;                    /* device pointer to the start of the storage; borrowed  */
  int64_t offset;                /* bytes from base to element (0,...,0) of this view     */
  int32_t dtype;                 /* ocn_dtype                                             */
  int32_t ndim;                  /* 0 (a scalar) .. OCN_MAX_DIMS                          */
  int64_t size[OCN_MAX_DIMS];    /* extents, >= 0                                         */
  int64_t stride[OCN_MAX_DIMS];  /* bytes; may be 0 or negative                           */
  int32_t device;                /* HIP device ordinal; all operands of a call must agree */
  int32_t byteswapped;           /* non-zero: the elements are stored in the other byte order
                                    (section 3.1.3): every scalar - each component of a complex
                                    element - has its bytes reversed in memory.  The kernels
                                    reverse on load and on store; no extra pass is made.
                                    Honoured by ocn_unary, ocn_binary, ocn_cast_copy,
                                    ocn_reduce and ocn_binary_reduce (and their variants; the
                                    last one then runs as its two calls), and by ocn_gather and
                                    ocn_scatter, which reverse every scalar where the two sides
                                    differ; index arrays, offsets and masks are native data:
                                    OCN_ERR_BYTEORDER otherwise.  The field
                                    takes the place of what used to be padding: zero it */
} ocn_tensor;

typedef enum { /* section 3.2: basic arithmetic; complex types add conjugation (section 4) */
  OCN_U_IDENT = 0, /* out = a (a cast when the types differ)                   */
  OCN_U_NEG,       /* -a; integers wrap                                        */
  OCN_U_ABS,       /* |a|; integers wrap; for a complex input the modulus, evaluated in
                      the input's type: a real value of that precision (a few ulp)  */
  OCN_U_CONJ,      /* complex conjugate; identity on real types                */
  OCN_U_LNOT,      /* !(a != 0)                                                */
  OCN_U_BNOT,      /* ~a for integers, ! for bool                              */
  OCN_U_SQRT,      /* square root: correctly rounded on real floating types;
                      principal branch on complex types (a few ulp, as below) */
  OCN_U_SIN,       /* elementary functions on real and complex floating types  */
  OCN_U_COS,       /* (section 3.2: trigonometric operations): evaluated in    */
  OCN_U_TAN,       /* single precision for half and float types, in double     */
  OCN_U_EXP,       /* otherwise; accurate to a few units in the last place,    */
  OCN_U_LOG,       /* not bit-reproducible against another math library        */
  OCN_U_BSWAP,     /* integer types: the element with its bytes reversed (section
                      3.1.3: data in the other byte order; view floating data as
                      unsigned integers of the scalar size to bring it to native order) */
  OCN_U_ASIN, OCN_U_ACOS, OCN_U_ATAN,   /* inverse trigonometric and hyperbolic functions on */
  OCN_U_SINH, OCN_U_COSH, OCN_U_TANH,   /* real and complex floating types, same accuracy    */
  OCN_NUM_UNARY
} ocn_unary_op;

typedef enum {
  OCN_B_ADD = 0, OCN_B_SUB, OCN_B_MUL, OCN_B_DIV, OCN_B_MIN, OCN_B_MAX, /* arithmetic */
  OCN_B_BAND, OCN_B_BOR, OCN_B_BXOR,                                    /* bitwise    */
  OCN_B_LAND, OCN_B_LOR, OCN_B_LXOR,                                    /* logical    */
  OCN_B_EQ, OCN_B_NE, OCN_B_LT, OCN_B_LE, OCN_B_GT, OCN_B_GE,           /* comparison */
  OCN_B_ABSGT,                                                          /* |a| > |b|  */
  OCN_NUM_BINARY
} ocn_binary_op;

typedef enum { /* section 3.2: tensor reductions along one or more axes */
  OCN_R_SUM = 0, OCN_R_PROD, OCN_R_MIN, OCN_R_MAX, OCN_R_ANY, OCN_R_ALL,
  OCN_NUM_REDUCE
} ocn_reduce_op;

typedef enum {
  OCN_OK = 0,
  OCN_ERR_NULLPTR = -1,     /* a required pointer is NULL                                        */
  OCN_ERR_DTYPE = -2,       /* bad dtype, operation not defined for the type, or a type mismatch
                               with OCN_STRICT_TYPES set                                         */
  OCN_ERR_NDIM = -3,        /* ndim outside 0..OCN_MAX_DIMS                                      */
  OCN_ERR_SHAPE = -4,       /* negative size, input not broadcastable to out, bad axes           */
  OCN_ERR_DEVICE = -5,      /* operands name different devices                                   */
  OCN_ERR_ALIGN = -6,       /* offset/stride/base not a multiple of the scalar size              */
  OCN_ERR_OVERLAP_OUT = -7, /* the output view addresses some byte more than once                */
  OCN_ERR_ALIAS = -8,       /* an input shares bytes with the output without being the same view */
  OCN_ERR_WORKSPACE = -9,   /* reduction workspace missing or too small                          */
  OCN_ERR_EMPTY = -10,      /* min/max over zero elements                                        */
  OCN_ERR_LAUNCH = -11,     /* the HIP runtime reported an error; see ocn_last_hip_error         */
  OCN_ERR_OP = -12,         /* unknown operation code                                            */
  OCN_ERR_BYTEORDER = -13,  /* an operand in the other byte order, in a call that takes native order only */
  OCN_ERR_DOMAIN = -14      /* error mode: an element lies outside the operation's domain         */
} ocn_status;

/* flags */
#define OCN_STRICT_TYPES 1u /* section 3.2.1: automatic type casting switched off; operand
                               types that differ are an error instead of being converted */

/*
 * Elementwise unary operation (sections 3.2 and 3.2.1): for every index i of out,
 *     out[i] = convert_out( f( convert_T( a[i] ) ) ).
 * T is out's dtype (bool for OCN_U_LNOT; a's dtype for OCN_U_ABS of a complex a, whose result
 * is real).  `a` broadcasts against out as in ocn_binary.
 * a may be the identical view as out (in place); any other sharing of bytes between a and
 * out is OCN_ERR_ALIAS (section 4: overlap between tensors must not corrupt results; the
 * paper resolves it with an intermediate tensor, which is the caller's to provide here).
 */
int ocn_unary(int op, const ocn_tensor *a, const ocn_tensor *out, uint32_t flags, void *stream);

/*
 * Elementwise binary operation with implicit type casting and broadcasting (section 3.2.1;
 * section 2.1: type conversions and broadcasting happen before the device function runs -
 * here they are fused into the kernel, no intermediate tensor exists):
 *     out[i] = convert_out( g( convert_T(a[i]), convert_T(b[i]) ) ).
 * Shapes: out fixes the result shape.  Inputs are right-aligned against it; an input
 * dimension must equal out's or be 1, and a size-1 dimension is read at index 0 whatever
 * its stride says (section 4: broadcasting along dimensions).
 * Compute type T, with P = ocn_promote(a.dtype, b.dtype): for arithmetic and bitwise
 * operations out's dtype when that is a.dtype or b.dtype (as in "A += B", where B is coerced
 * to A) or holds P (ocn_promote(P, out.dtype) == out.dtype), otherwise P, and the result is
 * converted to out's dtype once, on store (a narrower destination does not narrow the
 * operands first); P for comparisons and OCN_B_ABSGT; bool for the logical operations.
 * Half-precision types are evaluated in single precision and
 * rounded once when stored.  With OCN_STRICT_TYPES, a.dtype != b.dtype (and, for arithmetic
 * and bitwise operations, a.dtype != out.dtype) is OCN_ERR_DTYPE.
 * Either input may be the identical view as out.
 */
int ocn_binary(int op, const ocn_tensor *a, const ocn_tensor *b, const ocn_tensor *out,
               uint32_t flags, void *stream);

/*
 * Type-casting copy on one device (section 3.2.1, ocean.cast / ocean.ensure): dst[i] =
 * convert(src[i]).  Float to integer truncates toward zero, saturates, NaN gives 0; integer
 * to integer saturates; anything to bool is "!= 0"; to floating types rounds to nearest even
 * in one step; complex to real keeps the real part.  Same as ocn_unary(OCN_U_IDENT, ...).
 */
int ocn_cast_copy(const ocn_tensor *src, const ocn_tensor *dst, void *stream);

/*
 * Reduction along `naxes` distinct axes of a (section 3.2).  out must have
 * a.ndim - naxes dimensions: the kept dimensions of a in their original order.  naxes ==
 * a.ndim is a full reduction to a 0-dimensional out; naxes == 0 is a cast copy.
 * Accumulation: integer and bool sums/products in wrapping 64-bit; half in single, single
 * and double in double precision; min/max exactly in the input type, NaN-propagating, +0
 * above -0; any/all on "!= 0".  The accumulated value is converted once to out's dtype by
 * the ocn_cast_copy rules.  Results of floating sums do not depend on timing (no floating
 * atomics): the same call gives the same bits every time.
 * workspace: DEVICE scratch of at least ocn_reduce_workspace_bytes(...) bytes, 256-byte
 * aligned, caller-owned, used only during the enqueued work (may be NULL when that size is
 * 0).  out must not share bytes with a.  min/max over zero elements: OCN_ERR_EMPTY.
 */
int ocn_reduce(int op, const ocn_tensor *a, const int32_t *axes, int32_t naxes,
               const ocn_tensor *out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * ocn_reduce for callers that cannot allocate device memory and have no workspace to pass:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, kernels, results (bit for bit) and errors as ocn_reduce, except that the partial
 * results of a split reduction live in a fixed array of OCN_REDUCE_SCRATCH_BYTES bytes inside
 * the library's device image (every GPU the library runs on holds its own copy until the
 * process ends).  The call allocates and frees nothing.  OCN_ERR_WORKSPACE if the reduction
 * would need more than that (ocn_reduce_workspace_bytes tells; ocn_reduce takes any size);
 * OCN_ERR_DEVICE unless a->device is the calling thread's current HIP device.  All calls on
 * one GPU share the one array: two calls whose enqueued work may overlap in time (different
 * streams) race on it; calls on one stream are ordered and safe.  Nothing is carried from one
 * call to the next: every partial result that is read was written by the same call.
 */
#define OCN_REDUCE_SCRATCH_BYTES (1u << 20)
int ocn_reduce_scratch(int op, const ocn_tensor *a, const int32_t *axes, int32_t naxes,
                       const ocn_tensor *out, void *stream);

/*
 * Reduction of an elementwise result (sections 3.2 and 5: elementwise functions followed by a
 * reduction along axes, as in inner products and norms): what
 *     ocn_binary(ew_op, a, b, t);  ocn_reduce(red_op, t, axes, naxes, out, ...)
 * gives for a temporary t of type mid_dtype and the broadcast shape of a and b (each pair of
 * sizes equal or 1; missing leading dimensions count as 1), without t ever reaching memory
 * where a fused kernel exists: equal input types with sums of a+b, a-b, a*b in that type
 * (mid_dtype = the input type), or sums / any / all of ==, <, >, |a|>|b| (mid_dtype =
 * OCN_BOOL).  Other combinations run as the two calls above with t at the start of the
 * workspace.  axes index the broadcast shape; out has its kept dimensions.  Floating sums may
 * differ from the two-call result by the order of additions only.  Workspace, alignment,
 * aliasing and error rules as for ocn_reduce; out must not share bytes with a or b.
 */
int ocn_binary_reduce(int ew_op, int red_op, const ocn_tensor *a, const ocn_tensor *b,
                      const int32_t *axes, int32_t naxes, const ocn_tensor *out, int32_t mid_dtype,
                      void *workspace, size_t workspace_bytes, void *stream);

size_t ocn_binary_reduce_workspace_bytes(int ew_op, int red_op, const ocn_tensor *a,
                                         const ocn_tensor *b, const int32_t *axes, int32_t naxes,
                                         const ocn_tensor *out, int32_t mid_dtype);

/*
 * Index binding, gather and scatter (section 3.2.2: index arrays are checked for validity and
 * negative indices converted; boolean masks are counted and converted to explicit indices;
 * bound to a tensor's strides both become relative offsets into its data, after which indexed
 * elements are copied out of, or into, the tensor).  Offsets are int64 byte offsets relative
 * to element (0, ..., 0) of the tensor being indexed, in DEVICE memory.
 *
 * ocn_index_offsets: index and offsets are OCN_INT64 tensors of equal shape (any strides).
 * offsets[k] = i * stride_bytes with i = index[k], or index[k] + dim_size when negative;
 * indices outside [-dim_size, dim_size) give offset 0 and are counted into *invalid_count
 * (DEVICE int64, overwritten).
 */
int ocn_index_offsets(const ocn_tensor *index, int64_t dim_size, int64_t stride_bytes,
                      const ocn_tensor *offsets, void *invalid_count, void *stream);

/*
 * ocn_mask_offsets: mask is an OCN_BOOL tensor (any strides, fewer than 2^31 elements);
 * target_strides (HOST, mask->ndim entries) are the byte strides of the tensor the mask will
 * index.  Writes the offsets sum_d i_d * target_strides[d] of the selected positions, in
 * row-major order of the mask's dimensions, to offsets[0 .. min(count, capacity)) and the
 * number selected to *count (DEVICE int64).  workspace: DEVICE scratch of
 * ocn_mask_offsets_workspace_bytes(mask) bytes, 8-byte aligned.  Three kernel launches.
 */
size_t ocn_mask_offsets_workspace_bytes(const ocn_tensor *mask);
int ocn_mask_offsets(const ocn_tensor *mask, const int64_t *target_strides, void *offsets,
                     int64_t capacity, void *count, void *workspace, size_t workspace_bytes,
                     void *stream);

/*
 * ocn_gather:  out[j, i...] = the element of the indexed tensor at offsets[j] + (inner offset
 * of i...), for j < n.  a_inner describes ONE indexed sub-tensor: its base + offset is
 * element (0, ..., 0) of the indexed tensor, its sizes and strides those of the dimensions that
 * are not indexed (ndim 0 for element-wise selection).  out has shape [n, a_inner sizes...]
 * and the same dtype.  An offset outside [lo, hi] is not followed: that row of out keeps its
 * old contents (pass the smallest and largest offset that stays inside the storage).
 * ocn_scatter: the reverse copy, src[j, i...] into the indexed tensor; offsets that repeat
 * leave one of the written values, which one is not defined.
 * A lane moves one item (an element, or 16 bytes where the rows' fastest dimension is
 * contiguous and 16-byte aligned on both sides); rows of up to 256 items share a workgroup.
 * A copy of 2^32 lanes or more goes out in several launches.
 */
int ocn_gather(const ocn_tensor *a_inner, const void *offsets, int64_t n, int64_t lo, int64_t hi,
               const ocn_tensor *out, void *stream);
int ocn_scatter(const ocn_tensor *src, const void *offsets, int64_t n, int64_t lo, int64_t hi,
                const ocn_tensor *out_inner, void *stream);

/*
 * Domain check of the compute modes (section 3.2.1: the warning, error and complex modes first
 * check the elements against the operator's domain).  *flag (a 0-dimensional OCN_BOOL tensor on
 * the device) := some element of a lies outside the real domain of the unary operation op:
 * negative for OCN_U_SQRT and OCN_U_LOG, of magnitude above one for OCN_U_ASIN and OCN_U_ACOS;
 * every other operation, and complex or bool input, is defined everywhere.  NaN elements do not count.  What to do with the answer - warn, fail, or
 * switch to a complex result type - is the caller's policy.  workspace: DEVICE scratch of
 * ocn_domain_check_workspace_bytes(op, a) bytes (at least 256), 256-byte aligned.
 */
size_t ocn_domain_check_workspace_bytes(int op, const ocn_tensor *a);
int ocn_domain_check(int op, const ocn_tensor *a, const ocn_tensor *flag, void *workspace,
                     size_t workspace_bytes, void *stream);

/*
 * A unary operation in one of the compute modes of section 3.2.1 (parameters added to operators
 * such as the square root and the arccosine, whose domain a real tensor may leave):
 *   OCN_MODE_STANDARD  no check on the elements; NaN where an element is outside the domain.
 *                      Exactly ocn_unary(op, a, out, 0, stream); *outside is set to -1.
 *   OCN_MODE_WARNING   the domain check runs ahead of the operation on the same stream, then
 *                      the operation as in standard mode; *outside tells the caller what to warn about.
 *   OCN_MODE_ERROR     the check runs first; if an element is outside the domain nothing else
 *                      is launched, out is untouched and the call returns OCN_ERR_DOMAIN.
 *   OCN_MODE_COMPLEX   the check decides the result type: outside the domain the operation is
 *                      computed into out_complex (a complex tensor of out's shape; the real
 *                      input converts with a zero imaginary part), otherwise into out.
 * *outside (HOST int, may be NULL): -1 not checked, 0 all elements inside, 1 some outside; in
 * complex mode 1 also means that out_complex was written instead of out.  The domain is that
 * of ocn_domain_check.  Every mode but the standard one reads the check's answer on the host:
 * the call waits for the stream, and cannot be part of a graph capture.  Both result plans
 * are validated before anything is launched.  workspace: DEVICE scratch of
 * ocn_unary_mode_workspace_bytes(op, mode, a) bytes, 256-byte aligned (0 in standard mode).
 */
typedef enum { OCN_MODE_STANDARD = 0, OCN_MODE_WARNING, OCN_MODE_ERROR, OCN_MODE_COMPLEX } ocn_compute_mode;
size_t ocn_unary_mode_workspace_bytes(int op, int mode, const ocn_tensor *a);
int ocn_unary_mode(int op, int mode, const ocn_tensor *a, const ocn_tensor *out, const ocn_tensor *out_complex,
                   void *workspace, size_t workspace_bytes, int *outside, void *stream);

/* Bytes of workspace ocn_reduce needs for these arguments (0 when it runs in one pass).
 * Returns 0 as well when the arguments are invalid; ocn_reduce then reports the error. */
size_t ocn_reduce_workspace_bytes(int op, const ocn_tensor *a, const int32_t *axes,
                                  int32_t naxes, const ocn_tensor *out);

/* Result type of implicit casting (section 3.2.1): the smallest type that can keep both;
 * signed with unsigned 8-bit gives int16; a 64-bit integer with a floating type gives
 * double; a complex operand makes the result complex.  Negative on a bad dtype. */
int ocn_promote(int dtype_a, int dtype_b);

/* Element size in bytes of a dtype, 0 if invalid. */
int ocn_dtype_size(int dtype);

/* Upper bound on the workgroups (of 256 lanes) in one launch: 2^24 - 1 by default and at most,
 * which keeps a launch below 2^32 lanes; 0 restores the default.  Work that needs more runs as
 * a loop inside the kernel (generic-dtype elementwise kernel, generic reductions, index
 * binding) or goes out in several launches (gather, scatter).  Lowering the bound moves that
 * point; results never depend on it.  Process-wide. */
void ocn_set_max_launch_blocks(int64_t blocks);

/* Static description of a status code. */
const char *ocn_error_string(int code);

/* The hipError_t (as int) behind the most recent OCN_ERR_LAUNCH on this host thread. */
int ocn_last_hip_error(void);

/* ---- plan inspection (host only; launches nothing, touches no device memory) -------- */

typedef enum {
  OCN_KERNEL_NONE = 0,     /* zero elements: nothing to launch                              */
  OCN_KERNEL_EW_ROWS,      /* vectorised rows: every operand contiguous (or broadcast)
                              along the innermost canonical dimension                      */
  OCN_KERNEL_EW_TILED,     /* LDS-staged tiles: operands disagree on their fastest axis     */
  OCN_KERNEL_EW_GENERIC,   /* one element per lane, arbitrary strides                       */
  OCN_KERNEL_RED_ROWS,     /* reduced axis is the input's fastest                           */
  OCN_KERNEL_RED_COLS,     /* a kept axis is the input's fastest                            */
  OCN_KERNEL_RED_GENERIC,  /* one output per lane, arbitrary strides                        */
  OCN_KERNEL_EW_INTERLEAVE /* copy from planes into an output whose fastest axis is 2..8 long */
} ocn_kernel_kind;

/* What the host planner decided for a call: the canonical dimension list after dropping
 * size-1 dimensions, flipping, sorting by stride and merging (the optimisation section 4 of
 * the paper names: axes are sorted and consecutive ones merged), slowest dimension first. */
typedef struct {
  int32_t kernel;                     /* ocn_kernel_kind                                    */
  int32_t compute_dtype;              /* T                                                  */
  int32_t ndim;                       /* canonical dimensions (elementwise), or kept dims   */
  int32_t nred;                       /* reductions: canonical reduced dimensions           */
  int64_t size[OCN_MAX_DIMS];
  int64_t stride_out[OCN_MAX_DIMS];   /* bytes                                              */
  int64_t stride_a[OCN_MAX_DIMS];
  int64_t stride_b[OCN_MAX_DIMS];
  int64_t offset_out, offset_a, offset_b; /* bytes from each base, after flips              */
  int64_t red_size[OCN_MAX_DIMS];     /* reductions: reduced dims, slowest first            */
  int64_t red_stride_a[OCN_MAX_DIMS];
  int32_t vec;                        /* elements per lane access along the fastest dim     */
  int32_t tile_log2[OCN_MAX_DIMS];    /* tiled kernel: log2 of the tile extent per dim      */
  int32_t stage_a, stage_b;           /* tiled kernel: operand goes through LDS             */
  int32_t specialised;                /* 1: dtype-specialised kernel; 0: generic-dtype path */
  int32_t passes;                     /* kernel launches the call would make                */
  int64_t grid, block;                /* first launch                                       */
  int64_t split;                      /* reductions: partial results per output (1 = none)  */
  int64_t lds_bytes;
  int64_t unclipped;                  /* tiled kernel: 1 when no tile is clipped and every
                                         access is a whole vector (the leaner kernel form)  */
  int64_t fused;                      /* ocn_binary_reduce: 1 when one fused kernel does the
                                         elementwise step and the reduction                 */
  int64_t tile_group;                 /* tiled kernel: consecutive tiles that share cache
                                         lines of an input and are started on one XCD
                                         (1, 2 or 4)                                        */
} ocn_plan_info;

int ocn_plan_unary(int op, const ocn_tensor *a, const ocn_tensor *out, uint32_t flags,
                   ocn_plan_info *info);
int ocn_plan_binary(int op, const ocn_tensor *a, const ocn_tensor *b, const ocn_tensor *out,
                    uint32_t flags, ocn_plan_info *info);
int ocn_plan_reduce(int op, const ocn_tensor *a, const int32_t *axes, int32_t naxes,
                    const ocn_tensor *out, ocn_plan_info *info);
int ocn_plan_binary_reduce(int ew_op, int red_op, const ocn_tensor *a, const ocn_tensor *b,
                           const int32_t *axes, int32_t naxes, const ocn_tensor *out,
                           int32_t mid_dtype, ocn_plan_info *info);

#ifdef __cplusplus
}
#endif
#endif /* OCN_H */
