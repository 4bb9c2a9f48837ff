// Copy into an output whose fastest axis is only a few elements long while the input's fastest
// axis is the output's next one - planes to interleaved, e.g. channel-first to channel-last
// with three channels.  (Section 4 of the paper: strided tensors are handled by sorting and
// merging axes; this is the layout that leaves a short innermost axis behind.)
//
// A lane takes V = 16 / ES consecutive positions of the long axis: it loads one 16-byte vector
// from each of the C planes (neighbouring lanes read neighbouring vectors of a plane), deals
// the V * C elements out in the output's order in registers, and parks its 16 * C bytes in LDS.
// The wavefront then stores what it parked as C runs of 64 consecutive 16-byte pieces - whole
// cache lines, as streaming stores need them - where a lane storing its own C pieces would
// write every third piece of a line.  The general tiled kernel reads and writes this layout
// one element at a time (a fp32 copy of [64, 3, 512, 512] took 198 us).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>

#include "ew_launch.hpp"

namespace ocn {
namespace {

struct InterleaveArgs {
  char *out;
  const char *a;
  int32_t nouter;                       // dims above the long axis
  FastDiv odiv[kMaxDims];               // their sizes, fastest first
  int64_t so[kMaxDims], sa[kMaxDims];   // their byte strides, same order
  FastDiv mvec_div;                     // vectors along the long axis
  int64_t plane;                        // byte stride of the short axis in the input
  uint32_t nvec;                        // vectors in total
  int32_t nt_store, nt_load;
};

using Q = uint32_t __attribute__((ext_vector_type(4)));

template <int ES, int C> __global__ __launch_bounds__(kBlock) void ew_interleave_kernel(const InterleaveArgs p) {
  constexpr int V = 16 / ES;
  struct alignas(ES) Elem { unsigned char b[ES]; };
  __shared__ Q parked[kBlock * C];
  const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const uint32_t g = blockIdx.x * kBlock + tid;
  const bool valid = g < p.nvec;
  int64_t off_o = 0;
  if (valid) {
    uint32_t row = fastdiv(g, p.mvec_div);
    const uint32_t col = g - row * p.mvec_div.d;
    int64_t off_a = (int64_t)col * 16;
    off_o = (int64_t)col * (16 * C);
#pragma unroll
    for (int k = 0; k < kMaxDims; ++k) {
      if (k < p.nouter) {
        const uint32_t q = (k == p.nouter - 1) ? 0u : fastdiv(row, p.odiv[k]);
        const uint32_t i = row - q * p.odiv[k].d;
        row = q;
        off_o += (int64_t)i * p.so[k];
        off_a += (int64_t)i * p.sa[k];
      }
    }
    union { Q q; Elem e[V]; } in[C];
#pragma unroll
    for (int c = 0; c < C; ++c) {
      const Q *src = reinterpret_cast<const Q *>(p.a + off_a + (int64_t)c * p.plane);
      if (p.nt_load) {
        OCN_KEEP_BRANCH();
        in[c].q = __builtin_nontemporal_load(src);
        OCN_KEEP_BRANCH();
      } else {
        in[c].q = *src;
      }
    }
    union { Q q[C]; Elem e[V * C]; } o;
#pragma unroll
    for (int j = 0; j < V * C; ++j) o.e[j] = in[j % C].e[j / C];
#pragma unroll
    for (int c = 0; c < C; ++c) parked[(wave * kWave + lane) * C + c] = o.q[c];
  }
  __syncthreads();
  // piece k * 64 + lane of the wavefront's 64 * C pieces belongs to source lane (piece / C)
#pragma unroll
  for (int k = 0; k < C; ++k) {
    const uint32_t piece = (uint32_t)k * kWave + lane;
    const uint32_t from = piece / C, part = piece - from * C;
    const uint32_t lo = (uint32_t)__shfl((int)(uint32_t)off_o, (int)from, kWave);
    const uint32_t hi = (uint32_t)__shfl((int)(uint32_t)((uint64_t)off_o >> 32), (int)from, kWave);
    const int ok = __shfl(valid ? 1 : 0, (int)from, kWave);
    if (ok) {
      Q *dst = reinterpret_cast<Q *>(p.out + (int64_t)(((uint64_t)hi << 32) | lo) + (int64_t)part * 16);
      const Q v = parked[wave * kWave * C + piece];
      if (p.nt_store) {
        OCN_KEEP_BRANCH();
        __builtin_nontemporal_store(v, dst);
        OCN_KEEP_BRANCH();
      } else {
        *dst = v;
      }
    }
  }
}

template <int ES> hipError_t launch_es(int c, unsigned grid, hipStream_t s, const InterleaveArgs &a) {
  switch (c) {
#define OCN_CASE(CC) \
  case CC: hipLaunchKernelGGL((ew_interleave_kernel<ES, CC>), dim3(grid), dim3(kBlock), 0, s, a); break;
    OCN_CASE(2) OCN_CASE(3) OCN_CASE(4) OCN_CASE(5) OCN_CASE(6) OCN_CASE(7) OCN_CASE(8)
#undef OCN_CASE
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace

// plan: canonical dims [outer ..., M, C]; out contiguous over (M, C), input contiguous along M
hipError_t launch_interleave(const EwPlan &p, hipStream_t stream) {
  InterleaveArgs a;
  std::memset(&a, 0, sizeof a);
  const int n = p.ndim, es = dt_size(p.out.dtype), v = 16 / es;
  const int64_t c = p.size[n - 1], mvec = p.size[n - 2] / v;
  a.out = p.out.ptr;
  a.a = p.a.ptr;
  a.nouter = n - 2;
  int64_t rows = 1;
  for (int k = 0; k < n - 2; ++k) {   // fastest outer dim first
    const int d = n - 3 - k;
    a.odiv[k] = make_fastdiv((uint32_t)p.size[d]);
    a.so[k] = p.out.stride[d];
    a.sa[k] = p.a.stride[d];
    rows *= p.size[d];
  }
  a.mvec_div = make_fastdiv((uint32_t)mvec);
  a.plane = p.a.stride[n - 1];
  a.nvec = (uint32_t)(rows * mvec);
  a.nt_store = p.nt_store;
  a.nt_load = p.nt_a;
  const unsigned grid = (unsigned)p.grid;
  switch (es) {
    case 1: return launch_es<1>((int)c, grid, stream, a);
    case 2: return launch_es<2>((int)c, grid, stream, a);
    case 4: return launch_es<4>((int)c, grid, stream, a);
    case 8: return launch_es<8>((int)c, grid, stream, a);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace ocn
