// Host-side planning for the tensor engine: validation, implicit casting, overlap checks and
// dimension canonicalisation (drop, flip, sort, merge), then kernel selection.
//
// This is the device-independent "module interface" work of the paper's section 2.1
// (parameter checks, compatibility of dimensions, type resolution, broadcasting) plus the
// one optimisation the paper names in section 4: sorting of axes and merging of consecutive
// axes to increase memory locality and reduce the overhead of iterating over dimensions.
// Plain C++ with no HIP dependency, so it can be built and sanitised on the host alone.
#pragma once

#include <stddef.h>
#include <stdint.h>

#include "../../include/ocn.h"

namespace ocn {

constexpr int kMaxDims = OCN_MAX_DIMS;
constexpr int kBlock = 256;        // threads per workgroup of every kernel (4 wavefronts)
constexpr int kWave = 64;
constexpr int64_t kNumCUs = 256;          // MI355X: 8 XCDs x 32 compute units
constexpr uint32_t kXcds = 8;
constexpr int64_t kLdsPerCu = 160 * 1024;  // bytes of LDS per compute unit
// Operands of this many bytes or more are streamed: stores bypass the caches (an ordinary store
// leaves the lines dirty in the 256 MB Infinity Cache and the next kernel pays for the
// write-back), loads carry the non-temporal hint.
constexpr int64_t kStreamBytes = (int64_t)32 << 20;
#ifndef OCN_MAX_BLOCKS_PER_CU
#define OCN_MAX_BLOCKS_PER_CU 8
#endif
constexpr int64_t kMaxBlocksPerCu = OCN_MAX_BLOCKS_PER_CU;  // resident 256-lane workgroups per CU worth launching

// unsigned division by an invariant: q = (mulhi(n, m) + n) >> s, valid for n < 2^31
struct FastDiv {
  uint32_t d, m, s;
};
FastDiv make_fastdiv(uint32_t d);
inline uint32_t fastdiv_host(uint32_t n, const FastDiv &f) {
  return (uint32_t)((((uint64_t)n * f.m) >> 32) + n) >> f.s;
}

struct Operand {
  char *ptr;                    // base + offset, after flips
  int64_t stride[kMaxDims];     // bytes, canonical order (slowest first)
  int32_t dtype;
};

struct EwPlan {
  int kernel = OCN_KERNEL_NONE;
  int op = 0;
  int nin = 0;                  // 1 unary, 2 binary
  int T = 0;                    // compute dtype
  int ndim = 0;
  int64_t size[kMaxDims] = {0};
  Operand out{}, a{}, b{};
  int64_t off_out = 0, off_a = 0, off_b = 0;  // offsets relative to the caller's base
  int64_t numel = 0;
  // rows kernel
  int vec = 1;                  // elements per lane access
  int unroll = 1;               // vectors per lane
  bool a_inner_bcast = false, b_inner_bcast = false;
  // tiled kernel
  int tile_log2[kMaxDims] = {0};
  int tile_bits = 0;            // log2 of the elements of one tile
  bool stage_a = false, stage_b = false;
  int vecw_o = 0, vecw_a = 0, vecw_b = 0;  // log2 vector length of each enumeration order
  int nord = 0;                 // dims with a tile extent > 1
  int8_t ord_o[kMaxDims] = {0}, ord_a[kMaxDims] = {0}, ord_b[kMaxDims] = {0};
  int64_t ntiles[kMaxDims] = {0};
  int64_t total_tiles = 0;
  bool specialised = false;     // a dtype-specialised kernel exists for this signature
  bool fast_tiled = false;      // tiled kernel: the unclipped all-vector form applies
  bool nt_store = false;        // the output is too large to stay cached: stream it past the caches
  bool nt_a = false, nt_b = false;  // rows kernel: that input is read with streaming loads
  int swap = 0;                 // operands stored in the other byte order: bit 0 a, bit 1 b, bit 2 out
  int64_t grid = 0;
  int64_t lds_bytes = 0;
  int pair_dim = -1;            // all-vector tiled form: tiles that are neighbours along this dim share
  int pair_log2 = 0;            // cache lines of an input, in groups of 1 << pair_log2 tiles
};

struct RedPlan {
  int kernel = OCN_KERNEL_NONE;
  int op = 0;
  int nkept = 0, nred = 0;
  int64_t ksize[kMaxDims] = {0}, kstride_a[kMaxDims] = {0}, kstride_o[kMaxDims] = {0};
  int64_t rsize[kMaxDims] = {0}, rstride_a[kMaxDims] = {0};
  int64_t off_a = 0, off_out = 0;
  char *a_ptr = nullptr, *out_ptr = nullptr;
  int a_dtype = 0, out_dtype = 0;
  int64_t nout = 0, nredtot = 0;
  int vec = 1;
  int group = kBlock;           // lanes cooperating on one output (rows kernel): a power of two up to 64, or 256
  int block = kBlock;           // threads per workgroup (the cols kernel may use 1024)
  bool short_rows = false;      // rows kernel: every row fits one vector per lane of its group (loop-free kernel)
  int cpw = kWave;              // cols kernel: lanes per row of columns (power of two, at most a wavefront)
  bool nt_load = false;         // the input is far larger than the caches: stream it (non-temporal vector loads)
  bool lean = false;            // rows kernel: the common 2-D shape, run by the lean form of the kernel
  bool fold = false;            // second launch over [split][output] partial results: one output per lane
  bool swap_a = false, swap_o = false;  // the input / the output is stored in the other byte order
  int64_t split = 1;            // partial results per output
  int64_t chunk = 0;            // reduction elements (rows: vectors) per split
  int64_t grid = 0;
  int acc_dtype = 0;            // dtype the partial results are stored in
  size_t workspace_bytes = 0;
  int passes = 1;
  // reduction of an elementwise result (second input b; zero strides where it is broadcast)
  bool fused = false;
  int ew_op = 0, b_dtype = 0, mid_dtype = 0;
  char *b_ptr = nullptr;
  int64_t off_b = 0;
  int64_t kstride_b[kMaxDims] = {0}, rstride_b[kMaxDims] = {0};
  bool a_fast_bcast = false, b_fast_bcast = false;  // broadcast along the vectorised dim
};

// out = reduce(red_op, binary(ew_op, a, b) held as mid_dtype, axes), planned either as one fused
// kernel (plan->fused) or, when no fused kernel exists for the types, as the elementwise
// operation into a temporary followed by the reduction: then *unfused is set, `mid` describes
// the temporary (row-major, at the start of the workspace) and both sub-plans are filled in.
struct FusedPlan {
  RedPlan red;
  bool unfused = false;
  ocn_tensor mid{};
  EwPlan ew;
  size_t mid_bytes = 0;            // bytes of the temporary, rounded up to 256
  size_t workspace_bytes = 0;      // temporary + reduction workspace
};
int plan_binary_reduce(int ew_op, int red_op, const ocn_tensor *a, const ocn_tensor *b,
                       const int32_t *axes, int32_t naxes, const ocn_tensor *out, int mid_dtype,
                       char *workspace, FusedPlan *plan);

int plan_elementwise(int nin, int op, const ocn_tensor *a, const ocn_tensor *b,
                     const ocn_tensor *out, uint32_t flags, EwPlan *plan);
int plan_reduce(int op, const ocn_tensor *a, const int32_t *axes, int32_t naxes,
                const ocn_tensor *out, RedPlan *plan);
// plan for folding `split` partial results per output, stored as [nout][split] (rows) or
// [split][nout] (cols) of acc_dtype in the workspace, into the final output
void plan_second_pass(const RedPlan &first, char *workspace, RedPlan *second);

int promote(int a, int b);
int reduce_acc_dtype(int op, int in_dtype);
bool reduce_supported(int op, int in_dtype);

// Most workgroups one launch may have (2^24 - 1 of 256 lanes keeps a launch below 2^32 lanes;
// ocn_set_max_launch_blocks lowers it).  Kernels whose grid would be larger loop over their
// work with the capped grid, or their work goes out in several launches.
int64_t max_launch_blocks();
void set_max_launch_blocks(int64_t blocks);

// remembers a failed HIP call for ocn_last_hip_error (per host thread)
void record_hip_error(int code);

void fill_info(const EwPlan &p, ocn_plan_info *info);
void fill_info(const RedPlan &p, ocn_plan_info *info);

}  // namespace ocn
