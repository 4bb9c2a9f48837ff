// C ABI of the tensor engine (see include/ocn.h): argument checks, planning, launch.
#include <hip/hip_runtime.h>

#include <cstring>
#include <mutex>

#include "../../include/ocn.h"
#include "ew_launch.hpp"
#include "planner.hpp"
#include "red_launch.hpp"

namespace ocn {

// the internal numbering must match the public header
static_assert(DT_BOOL == OCN_BOOL && DT_I64 == OCN_INT64 && DT_U8 == OCN_UINT8 && DT_U64 == OCN_UINT64 &&
              DT_F16 == OCN_HALF && DT_F64 == OCN_DOUBLE && DT_C16 == OCN_CHALF && DT_C64 == OCN_CDOUBLE &&
              DT_COUNT == OCN_NUM_DTYPES, "dtype numbering");
static_assert(B_ADD == OCN_B_ADD && B_MAX == OCN_B_MAX && B_BAND == OCN_B_BAND && B_LAND == OCN_B_LAND &&
              B_EQ == OCN_B_EQ && B_GE == OCN_B_GE && B_ABSGT == OCN_B_ABSGT && B_COUNT == OCN_NUM_BINARY,
              "binary op numbering");
static_assert(U_IDENT == OCN_U_IDENT && U_NEG == OCN_U_NEG && U_ABS == OCN_U_ABS && U_CONJ == OCN_U_CONJ &&
              U_LNOT == OCN_U_LNOT && U_BNOT == OCN_U_BNOT && U_SQRT == OCN_U_SQRT && U_SIN == OCN_U_SIN &&
              U_LOG == OCN_U_LOG && U_BSWAP == OCN_U_BSWAP && U_ASIN == OCN_U_ASIN &&
              U_TANH == OCN_U_TANH && U_COUNT == OCN_NUM_UNARY,
              "unary op numbering");
static_assert(R_SUM == OCN_R_SUM && R_PROD == OCN_R_PROD && R_MIN == OCN_R_MIN && R_MAX == OCN_R_MAX &&
              R_ANY == OCN_R_ANY && R_ALL == OCN_R_ALL && R_COUNT == OCN_NUM_REDUCE, "reduce op numbering");

void register_ew_slice_0(); void register_ew_slice_1(); void register_ew_slice_2(); void register_ew_slice_3();
void register_ew_slice_4(); void register_ew_slice_5(); void register_ew_slice_6(); void register_ew_slice_7();
void register_red_slice_0(); void register_red_slice_1(); void register_red_slice_2(); void register_red_slice_3();
void register_fred_slice_0(); void register_fred_slice_1(); void register_fred_slice_2(); void register_fred_slice_3();

static std::once_flag g_once;
static void ensure_registered() {
  std::call_once(g_once, [] {
    register_ew_slice_0(); register_ew_slice_1(); register_ew_slice_2(); register_ew_slice_3();
    register_ew_slice_4(); register_ew_slice_5(); register_ew_slice_6(); register_ew_slice_7();
    register_red_slice_0(); register_red_slice_1(); register_red_slice_2(); register_red_slice_3();
    register_fred_slice_0(); register_fred_slice_1(); register_fred_slice_2(); register_fred_slice_3();
  });
}

static thread_local int g_last_hip_error = 0;
void record_hip_error(int code) { g_last_hip_error = code; }

static int finish(hipError_t e) {
  if (e == hipSuccess) return OCN_OK;
  g_last_hip_error = (int)e;
  return OCN_ERR_LAUNCH;
}

static int run_elementwise(const EwPlan &p, hipStream_t stream) {
  if (p.kernel == OCN_KERNEL_NONE) return OCN_OK;
  ensure_registered();
  if (p.kernel == OCN_KERNEL_EW_INTERLEAVE) return finish(launch_interleave(p, stream));
  if (!p.specialised) return finish(launch_interp(p, stream));
  EwLauncher f = p.nin == 2 ? g_binary_launchers[p.op][p.a.dtype][p.b.dtype][p.out.dtype]
                            : g_unary_launchers[p.op][p.a.dtype][p.out.dtype];
  if (!f) return finish(launch_interp(p, stream));
  return finish(f(p, stream));
}

// first launch of a (plain or fused) reduction plan, then the fold of its partial results
static int run_reduce(const RedPlan &p, RedLauncher first, char *workspace, hipStream_t stream) {
  if (!first) return OCN_ERR_DTYPE;
  int st = finish(first(p, workspace, stream));
  if (st != OCN_OK || p.split == 1) return st;
  RedPlan q;
  plan_second_pass(p, workspace, &q);
  RedLauncher g = g_reduce_launchers[q.op][q.a_dtype];
  if (!g) return OCN_ERR_DTYPE;
  return finish(g(q, nullptr, stream));
}

}  // namespace ocn

using namespace ocn;

extern "C" {

int ocn_unary(int op, const ocn_tensor *a, const ocn_tensor *out, uint32_t flags, void *stream) {
  EwPlan p;
  const int rc = plan_elementwise(1, op, a, nullptr, out, flags, &p);
  if (rc != OCN_OK) return rc;
  return run_elementwise(p, (hipStream_t)stream);
}

int ocn_binary(int op, const ocn_tensor *a, const ocn_tensor *b, const ocn_tensor *out,
               uint32_t flags, void *stream) {
  EwPlan p;
  const int rc = plan_elementwise(2, op, a, b, out, flags, &p);
  if (rc != OCN_OK) return rc;
  return run_elementwise(p, (hipStream_t)stream);
}

int ocn_cast_copy(const ocn_tensor *src, const ocn_tensor *dst, void *stream) {
  return ocn_unary(OCN_U_IDENT, src, dst, 0, stream);
}

int ocn_reduce(int op, const ocn_tensor *a, const int32_t *axes, int32_t naxes,
               const ocn_tensor *out, void *workspace, size_t workspace_bytes, void *stream) {
  RedPlan p;
  const int rc = plan_reduce(op, a, axes, naxes, out, &p);
  if (rc != OCN_OK) return rc;
  if (p.kernel == OCN_KERNEL_NONE) return OCN_OK;
  if (p.workspace_bytes > 0) {
    if (!workspace || workspace_bytes < p.workspace_bytes) return OCN_ERR_WORKSPACE;
    if ((uintptr_t)workspace % 256 != 0) return OCN_ERR_ALIGN;
  }
  ensure_registered();
  return run_reduce(p, g_reduce_launchers[p.op][p.a_dtype], (char *)workspace, (hipStream_t)stream);
}

int ocn_binary_reduce(int ew_op, int red_op, const ocn_tensor *a, const ocn_tensor *b, const int32_t *axes,
                      int32_t naxes, const ocn_tensor *out, int32_t mid_dtype, void *workspace,
                      size_t workspace_bytes, void *stream) {
  FusedPlan fp;
  const int rc = plan_binary_reduce(ew_op, red_op, a, b, axes, naxes, out, mid_dtype, (char *)workspace, &fp);
  if (rc != OCN_OK) return rc;
  if (fp.workspace_bytes > 0) {
    if (!workspace || workspace_bytes < fp.workspace_bytes) return OCN_ERR_WORKSPACE;
    if ((uintptr_t)workspace % 256 != 0) return OCN_ERR_ALIGN;
  }
  ensure_registered();
  if (fp.unfused) {
    const int st = run_elementwise(fp.ew, (hipStream_t)stream);
    if (st != OCN_OK || fp.red.kernel == OCN_KERNEL_NONE) return st;
    return run_reduce(fp.red, g_reduce_launchers[fp.red.op][fp.red.a_dtype], (char *)workspace + fp.mid_bytes,
                      (hipStream_t)stream);
  }
  if (fp.red.kernel == OCN_KERNEL_NONE) return OCN_OK;
  return run_reduce(fp.red, g_fused_launchers[fp.red.ew_op][fp.red.a_dtype][fp.red.op], (char *)workspace,
                    (hipStream_t)stream);
}

// ---- reduction without a workspace argument ----------------------------------------------
// Partial results of a split reduction go to a fixed array in device memory instead of a
// caller-provided workspace.  In host code the array's name is only a handle: its device
// address is looked up once per device (with that device current) and the kernels are given
// that address.
static __device__ __align__(256) unsigned char scratch[OCN_REDUCE_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static char *g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each device, once known
static std::mutex g_scratch_mutex;

// device address of `scratch` on the CURRENT device (which must be `device`)
static int scratch_address(int device, char **ptr) {
  if (device < 0 || device >= kMaxDevices) return OCN_ERR_DEVICE;
  int current = -1;
  hipError_t e = hipGetDevice(&current);
  if (e != hipSuccess) return finish(e);
  if (current != device) return OCN_ERR_DEVICE;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return finish(e);
    if (!p) return OCN_ERR_LAUNCH;
    g_scratch_ptr[device] = (char *)p;
  }
  *ptr = g_scratch_ptr[device];
  return OCN_OK;
}

int ocn_reduce_scratch(int op, const ocn_tensor *a, const int32_t *axes, int32_t naxes,
                       const ocn_tensor *out, void *stream) {
  RedPlan p;
  const int rc = plan_reduce(op, a, axes, naxes, out, &p);
  if (rc != OCN_OK) return rc;
  if (p.kernel == OCN_KERNEL_NONE) return OCN_OK;
  if (p.workspace_bytes > (size_t)OCN_REDUCE_SCRATCH_BYTES) return OCN_ERR_WORKSPACE;
  char *ws = nullptr;
  if (p.workspace_bytes > 0) {
    // every partial result the second launch reads is written by the first one: nothing in
    // the array has to be cleared between calls
    const int st = scratch_address(a->device, &ws);
    if (st != OCN_OK) return st;
  }
  ensure_registered();
  return run_reduce(p, g_reduce_launchers[p.op][p.a_dtype], ws, (hipStream_t)stream);
}

size_t ocn_binary_reduce_workspace_bytes(int ew_op, int red_op, const ocn_tensor *a, const ocn_tensor *b,
                                         const int32_t *axes, int32_t naxes, const ocn_tensor *out,
                                         int32_t mid_dtype) {
  FusedPlan fp;
  if (plan_binary_reduce(ew_op, red_op, a, b, axes, naxes, out, mid_dtype, nullptr, &fp) != OCN_OK) return 0;
  return fp.workspace_bytes;
}

size_t ocn_reduce_workspace_bytes(int op, const ocn_tensor *a, const int32_t *axes, int32_t naxes,
                                  const ocn_tensor *out) {
  RedPlan p;
  if (plan_reduce(op, a, axes, naxes, out, &p) != OCN_OK) return 0;
  return p.workspace_bytes;
}

int ocn_promote(int dtype_a, int dtype_b) { return promote(dtype_a, dtype_b); }

int ocn_dtype_size(int dtype) { return dtype >= 0 && dtype < DT_COUNT ? dt_size(dtype) : 0; }

const char *ocn_error_string(int code) {
  switch (code) {
    case OCN_OK: return "success";
    case OCN_ERR_NULLPTR: return "a required pointer is null";
    case OCN_ERR_DTYPE: return "invalid dtype, operation not defined for the type, or strict type mismatch";
    case OCN_ERR_NDIM: return "number of dimensions outside 0..8";
    case OCN_ERR_SHAPE: return "shapes are not compatible";
    case OCN_ERR_DEVICE: return "operands are on different devices";
    case OCN_ERR_ALIGN: return "offset, stride or pointer is not aligned to the element's scalar size";
    case OCN_ERR_OVERLAP_OUT: return "the output view overlaps itself";
    case OCN_ERR_ALIAS: return "an input overlaps the output without being the same view";
    case OCN_ERR_WORKSPACE: return "reduction workspace missing or too small";
    case OCN_ERR_EMPTY: return "min/max over zero elements";
    case OCN_ERR_LAUNCH: return "HIP runtime error";
    case OCN_ERR_OP: return "unknown operation";
    case OCN_ERR_BYTEORDER: return "an operand is stored in the other byte order, which this call does not take";
    case OCN_ERR_DOMAIN: return "an element lies outside the domain of the operation";
    default: return "unknown status code";
  }
}

int ocn_last_hip_error(void) { return g_last_hip_error; }

void ocn_set_max_launch_blocks(int64_t blocks) { set_max_launch_blocks(blocks); }

int ocn_plan_unary(int op, const ocn_tensor *a, const ocn_tensor *out, uint32_t flags, ocn_plan_info *info) {
  if (!info) return OCN_ERR_NULLPTR;
  EwPlan p;
  const int rc = plan_elementwise(1, op, a, nullptr, out, flags, &p);
  if (rc != OCN_OK) return rc;
  fill_info(p, info);
  return OCN_OK;
}

int ocn_plan_binary(int op, const ocn_tensor *a, const ocn_tensor *b, const ocn_tensor *out,
                    uint32_t flags, ocn_plan_info *info) {
  if (!info) return OCN_ERR_NULLPTR;
  EwPlan p;
  const int rc = plan_elementwise(2, op, a, b, out, flags, &p);
  if (rc != OCN_OK) return rc;
  fill_info(p, info);
  return OCN_OK;
}

int ocn_plan_reduce(int op, const ocn_tensor *a, const int32_t *axes, int32_t naxes,
                    const ocn_tensor *out, ocn_plan_info *info) {
  if (!info) return OCN_ERR_NULLPTR;
  RedPlan p;
  const int rc = plan_reduce(op, a, axes, naxes, out, &p);
  if (rc != OCN_OK) return rc;
  fill_info(p, info);
  return OCN_OK;
}

// all-zero bytes read as the value 0 of every dtype: the scalar the domain check compares with
static __device__ __align__(16) unsigned char g_zero_scalar[16];
// the value 1 in every dtype (little-endian bytes), one 16-byte slot each, in dtype order
static __device__ __align__(16) unsigned char g_one_scalars[DT_COUNT][16] = {
    {1}, {1}, {1, 0}, {1, 0, 0, 0}, {1, 0, 0, 0, 0, 0, 0, 0},                      // bool, int8..int64
    {1}, {1, 0}, {1, 0, 0, 0}, {1, 0, 0, 0, 0, 0, 0, 0},                           // uint8..uint64
    {0x00, 0x3c}, {0, 0, 0x80, 0x3f}, {0, 0, 0, 0, 0, 0, 0xf0, 0x3f},              // half, float, double
    {0x00, 0x3c, 0, 0}, {0, 0, 0x80, 0x3f, 0, 0, 0, 0},                            // chalf, cfloat
    {0, 0, 0, 0, 0, 0, 0xf0, 0x3f, 0, 0, 0, 0, 0, 0, 0, 0}};                       // cdouble

static int domain_plan(int op, const ocn_tensor *a, const ocn_tensor *flag, char *workspace, FusedPlan *fp, bool *trivial) {
  if (!a || !flag) return OCN_ERR_NULLPTR;
  if (op < 0 || op >= U_COUNT) return OCN_ERR_OP;
  if (flag->dtype != DT_BOOL || flag->ndim != 0) return OCN_ERR_SHAPE;
  const bool negative = op == U_SQRT || op == U_LOG, above_one = op == U_ASIN || op == U_ACOS;
  *trivial = !(negative || above_one);
  if (*trivial) return OCN_OK;
  if (a->dtype < 0 || a->dtype >= DT_COUNT) return OCN_ERR_DTYPE;
  if (dt_kind(a->dtype) == K_CPLX || dt_kind(a->dtype) == K_BOOL) { *trivial = true; return OCN_OK; }
  void *zero = nullptr;
  if (workspace) {  // a real call (not a size query): the device address of the scalar compared with
    const hipError_t e = negative ? hipGetSymbolAddress(&zero, HIP_SYMBOL(g_zero_scalar))
                                  : hipGetSymbolAddress(&zero, HIP_SYMBOL(g_one_scalars));
    if (e != hipSuccess || !zero) return finish(hipGetLastError());
    if (above_one) zero = (char *)zero + 16 * a->dtype;
  } else {
    zero = (void *)((uintptr_t)1 << 60);  // size query: stand-in addresses far from the temporary's
  }
  ocn_tensor z;
  std::memset(&z, 0, sizeof z);
  z.base = zero;
  z.dtype = a->dtype;
  z.ndim = 0;
  z.device = a->device;
  int32_t axes[OCN_MAX_DIMS];
  for (int d = 0; d < a->ndim && d < OCN_MAX_DIMS; ++d) axes[d] = d;
  return plan_binary_reduce(negative ? B_LT : B_ABSGT, R_ANY, a, &z, axes, a->ndim, flag, DT_BOOL, workspace, fp);
}

size_t ocn_domain_check_workspace_bytes(int op, const ocn_tensor *a) {
  ocn_tensor flag;
  std::memset(&flag, 0, sizeof flag);
  flag.base = (void *)(((uintptr_t)1 << 60) + 4096);
  flag.dtype = DT_BOOL;
  if (a) flag.device = a->device;
  FusedPlan fp;
  bool trivial = false;
  if (domain_plan(op, a, &flag, nullptr, &fp, &trivial) != OCN_OK || trivial) return 256;
  return fp.workspace_bytes < 256 ? 256 : fp.workspace_bytes;
}

int ocn_domain_check(int op, const ocn_tensor *a, const ocn_tensor *flag, void *workspace, size_t workspace_bytes,
                     void *stream) {
  if (!workspace || workspace_bytes < 256) return OCN_ERR_WORKSPACE;
  if ((uintptr_t)workspace % 256 != 0) return OCN_ERR_ALIGN;
  FusedPlan fp;
  bool trivial = false;
  int rc = domain_plan(op, a, flag, (char *)workspace, &fp, &trivial);
  if (rc != OCN_OK) return rc;
  if (trivial) {
    // every element is inside the domain: flag := cast(false), through the ordinary cast copy
    // of a zero scalar (no separate fill kernel, nothing a graph capture would mind)
    void *zero = nullptr;
    if (hipGetSymbolAddress(&zero, HIP_SYMBOL(g_zero_scalar)) != hipSuccess || !zero) return finish(hipGetLastError());
    ocn_tensor z;
    std::memset(&z, 0, sizeof z);
    z.base = zero;
    z.dtype = DT_BOOL;
    z.device = flag->device;
    return ocn_cast_copy(&z, flag, stream);
  }
  if (fp.workspace_bytes > workspace_bytes) return OCN_ERR_WORKSPACE;
  ensure_registered();
  if (fp.unfused) {
    const int st = run_elementwise(fp.ew, (hipStream_t)stream);
    if (st != OCN_OK || fp.red.kernel == OCN_KERNEL_NONE) return st;
    return run_reduce(fp.red, g_reduce_launchers[fp.red.op][fp.red.a_dtype], (char *)workspace + fp.mid_bytes,
                      (hipStream_t)stream);
  }
  if (fp.red.kernel == OCN_KERNEL_NONE) return OCN_OK;
  return run_reduce(fp.red, g_fused_launchers[fp.red.ew_op][fp.red.a_dtype][fp.red.op], (char *)workspace,
                    (hipStream_t)stream);
}

// ---- compute modes (section 3.2.1) ---------------------------------------------------------
// The first 256 bytes of the workspace hold the flag the domain check writes; the check's own
// workspace follows.
size_t ocn_unary_mode_workspace_bytes(int op, int mode, const ocn_tensor *a) {
  if (mode == OCN_MODE_STANDARD) return 0;
  return 256 + ocn_domain_check_workspace_bytes(op, a);
}

int ocn_unary_mode(int op, int mode, const ocn_tensor *a, const ocn_tensor *out, const ocn_tensor *out_complex,
                   void *workspace, size_t workspace_bytes, int *outside, void *stream) {
  if (mode < OCN_MODE_STANDARD || mode > OCN_MODE_COMPLEX) return OCN_ERR_OP;
  if (outside) *outside = -1;
  if (mode == OCN_MODE_STANDARD) return ocn_unary(op, a, out, 0, stream);
  // everything that can be refused is refused before the first launch
  EwPlan real_plan, complex_plan;
  int rc = plan_elementwise(1, op, a, nullptr, out, 0, &real_plan);
  if (rc != OCN_OK) return rc;
  if (mode == OCN_MODE_COMPLEX) {
    if (!out_complex) return OCN_ERR_NULLPTR;
    if (out_complex->dtype < 0 || out_complex->dtype >= DT_COUNT || dt_kind(out_complex->dtype) != K_CPLX)
      return OCN_ERR_DTYPE;
    if ((rc = plan_elementwise(1, op, a, nullptr, out_complex, 0, &complex_plan)) != OCN_OK) return rc;
  }
  if (!workspace || workspace_bytes < ocn_unary_mode_workspace_bytes(op, mode, a)) return OCN_ERR_WORKSPACE;
  if ((uintptr_t)workspace % 256 != 0) return OCN_ERR_ALIGN;
  ocn_tensor flag;
  std::memset(&flag, 0, sizeof flag);
  flag.base = workspace;
  flag.dtype = DT_BOOL;
  flag.device = a->device;
  rc = ocn_domain_check(op, a, &flag, (char *)workspace + 256, workspace_bytes - 256, stream);
  if (rc != OCN_OK) return rc;
  unsigned char answer = 0;
  hipError_t e = hipMemcpyAsync(&answer, workspace, 1, hipMemcpyDeviceToHost, (hipStream_t)stream);
  if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);
  if (e != hipSuccess) return finish(e);
  if (outside) *outside = answer ? 1 : 0;
  if (answer && mode == OCN_MODE_ERROR) return OCN_ERR_DOMAIN;
  return run_elementwise(answer && mode == OCN_MODE_COMPLEX ? complex_plan : real_plan, (hipStream_t)stream);
}

int ocn_plan_binary_reduce(int ew_op, int red_op, const ocn_tensor *a, const ocn_tensor *b, const int32_t *axes,
                           int32_t naxes, const ocn_tensor *out, int32_t mid_dtype, ocn_plan_info *info) {
  if (!info) return OCN_ERR_NULLPTR;
  FusedPlan fp;
  const int rc = plan_binary_reduce(ew_op, red_op, a, b, axes, naxes, out, mid_dtype, nullptr, &fp);
  if (rc != OCN_OK) return rc;
  fill_info(fp.red, info);
  info->fused = fp.unfused ? 0 : 1;
  if (fp.unfused && fp.ew.kernel != OCN_KERNEL_NONE) info->passes += 1;
  return OCN_OK;
}

}  // extern "C"
