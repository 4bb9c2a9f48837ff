// Index binding, gather and scatter for gfx950 (section 3.2.2 of the paper: index arrays are
// checked and negative indices converted; boolean masks are counted and converted to explicit
// indices; bound to strides both become relative offsets into the data buffer, after which the
// indexed elements are copied out of, or into, the tensor).
//
//   ocn_index_offsets  one lane per index: wrap, range check, multiply by the stride; invalid
//                      indices are counted (one integer atomic per wavefront that saw any)
//   ocn_mask_offsets   stream compaction in the mask's row-major order, three launches and no
//                      waiting between workgroups: per-workgroup counts, an exclusive scan of
//                      the counts by one workgroup (through LDS, coalesced both ways), then every workgroup writes the offsets of
//                      its selected elements behind its prefix (staged in LDS so that the
//                      stores are coalesced).  Lanes own 16 consecutive mask bytes (one 128-bit
//                      load when the mask is contiguous).
//   ocn_gather/scatter one lane per copied item (an element, or 16 bytes where the rows' fastest
//                      dimension is contiguous and aligned), rows of `inner` elements per offset;
//                      short rows share a workgroup, long ones take several.  Offsets outside the stated range are skipped, never followed.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>

#include "../../include/ocn.h"
#include "dtypes.hpp"
#include "dev_types.hpp"
#include "planner.hpp"

namespace ocn {
namespace {

constexpr int kMaskPerLane = 16;                       // mask elements per lane
constexpr int kMaskChunk = kBlock * kMaskPerLane;      // per workgroup
constexpr int kScanBlock = 1024;

__device__ __forceinline__ uint32_t fdiv(uint32_t n, const FastDiv &f) { return (__umulhi(n, f.m) + n) >> f.s; }

// ---------------------------------------------------------------------------------------
// index arrays
// ---------------------------------------------------------------------------------------

struct IndexArgs {
  const char *idx;
  char *off;
  int32_t ndim;
  int64_t size[kMaxDims], si[kMaxDims], so[kMaxDims];  // row-major: last dim fastest
  int64_t n, dim_size, stride;
  unsigned long long *invalid;
};

__global__ void fill_u64_kernel(unsigned long long *p, unsigned long long v) { *p = v; }

__global__ __launch_bounds__(kBlock) void index_offsets_kernel(const IndexArgs p) {
  // the grid is capped (a launch cannot have 2^32 lanes): longer index arrays loop; every lane
  // of a wavefront makes the same number of trips, so that the vote below stays whole
  const int64_t step = (int64_t)gridDim.x * kBlock;
  for (int64_t e0 = (int64_t)blockIdx.x * kBlock; e0 < p.n; e0 += step) {
  const int64_t e = e0 + threadIdx.x;
  bool bad = false;
  if (e < p.n) {
    int64_t rem = e, oi = 0, oo = 0;
#pragma unroll
    for (int d = kMaxDims - 1; d >= 0; --d) {
      if (d < p.ndim) {
        const int64_t q = rem / p.size[d];
        const int64_t i = rem - q * p.size[d];
        rem = q;
        oi += i * p.si[d];
        oo += i * p.so[d];
      }
    }
    int64_t i = *reinterpret_cast<const int64_t *>(p.idx + oi);
    if (i < 0) i += p.dim_size;
    bad = i < 0 || i >= p.dim_size;
    *reinterpret_cast<int64_t *>(p.off + oo) = bad ? 0 : i * p.stride;
  }
  const unsigned long long votes = __ballot(bad);
  if (votes != 0 && (threadIdx.x & (kWave - 1)) == 0) atomicAdd(p.invalid, (unsigned long long)__popcll(votes));
  }
}

// Both tensors contiguous (and 16-byte aligned): two indices per lane, one 16-byte load and one
// 16-byte store each, streamed when the arrays are too large to stay cached; no index
// decomposition (the kernel above divides 64-bit numbers once per dim and element: 2^26
// indices 264 us).
__global__ __launch_bounds__(kBlock) void index_offsets_flat_kernel(const IndexArgs p, int nt) {
  using L2 = long long __attribute__((ext_vector_type(2)));
  const int64_t npair = (p.n + 1) / 2;
  const int64_t step = (int64_t)gridDim.x * kBlock;
  for (int64_t e0 = (int64_t)blockIdx.x * kBlock; e0 < npair; e0 += step) {
    const int64_t e = e0 + threadIdx.x;
    int nbad = 0;
    if (e < npair) {
      const bool both = 2 * e + 1 < p.n;
      L2 v;
      if (both) {
        if (nt) { asm volatile(""); v = __builtin_nontemporal_load(reinterpret_cast<const L2 *>(p.idx) + e); asm volatile(""); }
        else v = reinterpret_cast<const L2 *>(p.idx)[e];
      } else {
        v.x = reinterpret_cast<const long long *>(p.idx)[2 * e];
        v.y = 0;
      }
      long long i0 = v.x < 0 ? v.x + p.dim_size : v.x, i1 = v.y < 0 ? v.y + p.dim_size : v.y;
      const bool bad0 = i0 < 0 || i0 >= p.dim_size, bad1 = both && (i1 < 0 || i1 >= p.dim_size);
      nbad = (bad0 ? 1 : 0) + (bad1 ? 1 : 0);
      L2 r;
      r.x = bad0 ? 0 : i0 * p.stride;
      r.y = bad1 ? 0 : i1 * p.stride;
      if (both) {
        if (nt) { asm volatile(""); __builtin_nontemporal_store(r, reinterpret_cast<L2 *>(p.off) + e); asm volatile(""); }
        else reinterpret_cast<L2 *>(p.off)[e] = r;
      } else {
        reinterpret_cast<long long *>(p.off)[2 * e] = r.x;
      }
    }
    // every lane of a wavefront makes the same number of trips, so the shuffles stay whole
#pragma unroll
    for (int d = kWave / 2; d >= 1; d >>= 1) nbad += __shfl_xor(nbad, d, kWave);
    if (nbad != 0 && (threadIdx.x & (kWave - 1)) == 0) atomicAdd(p.invalid, (unsigned long long)nbad);
  }
}

// ---------------------------------------------------------------------------------------
// boolean masks
// ---------------------------------------------------------------------------------------

struct MaskArgs {
  const char *mask;
  int32_t ndim;                       // canonical dims, row-major: last fastest
  FastDiv div[kMaxDims];
  int64_t sm[kMaxDims], st[kMaxDims]; // mask / target byte strides
  uint32_t n;                         // mask elements (< 2^31)
  int32_t contig;                     // the mask is one contiguous, 16-byte aligned run
  int64_t *block_counts;              // [nblocks]; after the scan: exclusive prefixes
  uint32_t nblocks;
  int64_t *offsets;
  int64_t capacity;
  int64_t *count;
  int32_t nt_store;                   // large result: streaming stores
};

__device__ __forceinline__ void mask_decode(const MaskArgs &p, uint32_t e, int64_t &om, int64_t &ot) {
  om = 0;
  ot = 0;
#pragma unroll
  for (int d = kMaxDims - 1; d >= 0; --d) {
    if (d < p.ndim) {
      const uint32_t q = d == 0 ? 0u : fdiv(e, p.div[d]);
      const uint32_t i = e - q * p.div[d].d;
      e = q;
      om += (int64_t)i * p.sm[d];
      ot += (int64_t)i * p.st[d];
    }
  }
}

// bit k set: element e0 + k is selected
__device__ __forceinline__ uint32_t mask_flags(const MaskArgs &p, uint32_t e0) {
  uint32_t flags = 0;
  if (e0 >= p.n) return 0;
  if (p.contig && e0 + kMaskPerLane <= p.n) {
    const uint4 v = *reinterpret_cast<const uint4 *>(p.mask + e0);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int k = 0; k < kMaskPerLane; ++k)
      if ((w[k >> 2] >> (8 * (k & 3))) & 0xffu) flags |= 1u << k;
    return flags;
  }
#pragma unroll 4
  for (int k = 0; k < kMaskPerLane; ++k) {
    const uint32_t e = e0 + (uint32_t)k;
    if (e < p.n) {
      int64_t om, ot;
      mask_decode(p, e, om, ot);
      if (*reinterpret_cast<const uint8_t *>(p.mask + om) != 0) flags |= 1u << k;
    }
  }
  return flags;
}

// exclusive prefix of `v` over the workgroup's lanes; total in `sum` (all lanes)
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t *lds, uint32_t &sum) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  uint32_t inc = v;
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    const uint32_t up = (uint32_t)__shfl_up((int)inc, d, kWave);
    if (lane >= d) inc += up;
  }
  if (lane == kWave - 1) lds[wave] = inc;
  __syncthreads();
  uint32_t before = 0, total = 0;
#pragma unroll
  for (int w = 0; w < kBlock / kWave; ++w) {
    if (w < wave) before += lds[w];
    total += lds[w];
  }
  sum = total;
  return before + inc - v;
}

__global__ __launch_bounds__(kBlock) void mask_count_kernel(const MaskArgs p) {
  __shared__ uint32_t lds[kBlock / kWave];
  const uint32_t e0 = (blockIdx.x * kBlock + threadIdx.x) * kMaskPerLane;
  const uint32_t c = (uint32_t)__popc(mask_flags(p, e0));
  uint32_t sum;
  (void)block_exclusive_scan(c, lds, sum);
  if (threadIdx.x == 0) p.block_counts[blockIdx.x] = (int64_t)sum;
}

// The same counts for a contiguous mask: a wavefront per chunk of kMaskChunk bytes, every lane
// with four 16-byte loads in flight (the loads of a wavefront cover 1 KiB each), no LDS and no
// barrier; four chunks per workgroup.  (One load per lane and a workgroup per chunk read a
// 64 MB mask at 3 TB/s.)
__global__ __launch_bounds__(kBlock) void mask_count_contig_kernel(const MaskArgs p) {
  const uint32_t lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const uint32_t chunk = blockIdx.x * (kBlock / kWave) + wave;
  if (chunk >= p.nblocks) return;     // whole wavefronts leave together
  const uint32_t base = chunk * (uint32_t)kMaskChunk;
  uint32_t c = 0;
  constexpr int kPieces = kMaskChunk / (kWave * 16);
  uint4 v[kPieces];
#pragma unroll
  for (int k = 0; k < kPieces; ++k) {
    const uint32_t e = base + (uint32_t)k * (kWave * 16) + lane * 16u;
    v[k] = make_uint4(0u, 0u, 0u, 0u);
    if (e + 16u <= p.n) {
      v[k] = *reinterpret_cast<const uint4 *>(p.mask + e);
    } else if (e < p.n) {               // the ragged end of the mask, byte by byte
      uint32_t w[4] = {0u, 0u, 0u, 0u};
      for (uint32_t i = 0; e + i < p.n; ++i)
        w[i >> 2] |= (uint32_t) * reinterpret_cast<const uint8_t *>(p.mask + e + i) << (8 * (i & 3));
      v[k] = make_uint4(w[0], w[1], w[2], w[3]);
    }
  }
  // bytes that are not zero: bit 7 of each byte of ((w & 0x7f..) + 0x7f..) | w
  auto nonzero_bytes = [](uint32_t w) { return (uint32_t)__popc((((w & 0x7f7f7f7fu) + 0x7f7f7f7fu) | w) & 0x80808080u); };
#pragma unroll
  for (int k = 0; k < kPieces; ++k)
    c += nonzero_bytes(v[k].x) + nonzero_bytes(v[k].y) + nonzero_bytes(v[k].z) + nonzero_bytes(v[k].w);
#pragma unroll
  for (int d = kWave / 2; d >= 1; d >>= 1) c += (uint32_t)__shfl_xor((int)c, d, kWave);
  if (lane == 0) p.block_counts[chunk] = (int64_t)c;
}

// one workgroup: block_counts[i] := sum of block_counts[0 .. i), *count := total.  Rounds of
// 1024 x 16 counts: read coalesced into LDS, each lane adds up 16 consecutive ones, the lane
// sums are scanned with wavefront shuffles, and the prefixes go back through LDS so that the
// stores are coalesced too.  Counts are at most kMaskChunk and a round's total stays below
// 2^26, so LDS holds 32-bit values; the carry between rounds is 64-bit.
__global__ __launch_bounds__(kScanBlock) void mask_scan_kernel(const MaskArgs p) {
  constexpr int kPer = 16, kRound = kScanBlock * kPer, kWaves = kScanBlock / kWave;
  __shared__ uint32_t tile[kRound + kRound / kPer];   // one pad word per lane segment: no bank conflicts
  __shared__ uint32_t wave_sum[kWaves];
  const int t = threadIdx.x, lane = t & (kWave - 1), wave = t / kWave;
  int64_t carry = 0;
  for (int64_t base = 0; base < (int64_t)p.nblocks; base += kRound) {
#pragma unroll
    for (int k = 0; k < kPer; ++k) {
      const int64_t i = base + k * kScanBlock + t;
      const int j = k * kScanBlock + t;
      tile[j + j / kPer] = i < (int64_t)p.nblocks ? (uint32_t)p.block_counts[i] : 0u;
    }
    __syncthreads();
    uint32_t own[kPer], s = 0;
#pragma unroll
    for (int k = 0; k < kPer; ++k) {
      own[k] = tile[t * (kPer + 1) + k];
      s += own[k];
    }
    uint32_t inc = s;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
      const uint32_t up = (uint32_t)__shfl_up((int)inc, d, kWave);
      if (lane >= d) inc += up;
    }
    if (lane == kWave - 1) wave_sum[wave] = inc;
    __syncthreads();
    uint32_t before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      if (w < wave) before += wave_sum[w];
      total += wave_sum[w];
    }
    uint32_t run = before + inc - s;
#pragma unroll
    for (int k = 0; k < kPer; ++k) {
      tile[t * (kPer + 1) + k] = run;
      run += own[k];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kPer; ++k) {
      const int64_t i = base + k * kScanBlock + t;
      const int j = k * kScanBlock + t;
      if (i < (int64_t)p.nblocks) p.block_counts[i] = carry + (int64_t)tile[j + j / kPer];
    }
    carry += (int64_t)total;
    __syncthreads();   // the next round overwrites tile and wave_sum
  }
  if (t == 0) *p.count = carry;
}

__global__ __launch_bounds__(kBlock) void mask_write_kernel(const MaskArgs p) {
  __shared__ uint32_t lds[kBlock / kWave];
  // the positions (inside this workgroup's chunk) of its selected elements, in order: 8 KiB,
  // where the offsets themselves would take 32 KiB and leave room for five workgroups per CU
  __shared__ uint16_t staged[kMaskChunk];
  static_assert(kMaskChunk <= 65536, "positions inside a chunk are staged as 16-bit values");
  const uint32_t chunk0 = blockIdx.x * (uint32_t)kMaskChunk;
  const uint32_t e0 = chunk0 + threadIdx.x * kMaskPerLane;
  const uint32_t flags = mask_flags(p, e0);
  uint32_t sum;
  uint32_t slot = block_exclusive_scan((uint32_t)__popc(flags), lds, sum);
  uint32_t f = flags;
  while (f) {
    const int k = __ffs((int)f) - 1;
    f &= f - 1;
    staged[slot++] = (uint16_t)(threadIdx.x * kMaskPerLane + (uint32_t)k);
  }
  __syncthreads();
  // coalesced stores behind this workgroup's prefix; a position becomes its offset on the way out
  const int64_t base = p.block_counts[blockIdx.x];
  for (uint32_t i = threadIdx.x; i < sum; i += kBlock)
    if (base + i < p.capacity) {
      int64_t om, ot;
      mask_decode(p, chunk0 + (uint32_t)staged[i], om, ot);
      if (p.nt_store) {  // (the empty asm keeps the compiler from merging the two stores and dropping the hint)
        asm volatile("");
        __builtin_nontemporal_store(ot, p.offsets + base + i);
        asm volatile("");
      } else {
        p.offsets[base + i] = ot;
      }
    }
}

// ---------------------------------------------------------------------------------------
// gather / scatter
// ---------------------------------------------------------------------------------------

struct GatherArgs {
  const char *src;                    // gather: the indexed tensor; scatter: the rows
  char *dst;
  const int64_t *offsets;
  int64_t n, lo, hi;
  int32_t ndim;                       // canonical inner dims, last fastest
  FastDiv div[kMaxDims];
  int64_t ss[kMaxDims], sd[kMaxDims]; // inner byte strides on the source / destination side
  int64_t row_stride;                 // bytes between rows on the side that is not indexed
  uint32_t inner;                     // elements per row
  uint32_t vec;                       // elements a lane copies at once (1, or 16 bytes' worth)
  uint32_t items;                     // lane items per row: inner / vec
  int32_t items_log2;                 // >= 0: rows of at most 256 items, padded to 1 << items_log2 lanes,
                                      // 256 >> items_log2 rows per workgroup; -1: workgroups per row below
  FastDiv chunks_div;                 // workgroups per row
  int32_t nt_rows;                    // gather of single elements: stream the (large) result past the caches
  int32_t swap_sc;                    // the two sides are stored in different byte orders: bytes of one scalar (0: same order)
};

// reverses every scalar of `sc` bytes in a piece that is moved between byte orders
template <class P> __device__ __forceinline__ void reorder(P &v, int sc) {
  if (sc == 0) return;
  if constexpr (sizeof(P) >= 2) { if (sc == 2) reverse_scalars<2>(v); }
  if constexpr (sizeof(P) >= 4) { if (sc == 4) reverse_scalars<4>(v); }
  if constexpr (sizeof(P) >= 8) { if (sc == 8) reverse_scalars<8>(v); }
}

template <int ES> struct Bytes { unsigned char b[ES]; };
template <> struct alignas(2) Bytes<2> { unsigned char b[2]; };
template <> struct alignas(4) Bytes<4> { unsigned char b[4]; };
template <> struct alignas(8) Bytes<8> { unsigned char b[8]; };
template <> struct alignas(16) Bytes<16> { unsigned char b[16]; };

// SCATTER = false: dst[j, i] = src[offsets[j] + i];  true: dst[offsets[j] + i] = src[j, i]
// A lane copies one item: an element, or 16 bytes of the rows' fastest dim when that dim is
// contiguous and aligned on both sides (an offset that is not a multiple of 16 falls back to
// element copies for its row).  Short rows share a workgroup.
template <int ES, bool SCATTER> __global__ __launch_bounds__(kBlock) void gather_kernel(const GatherArgs p) {
  constexpr int V = 16 / ES;
  int64_t j;
  uint32_t item;
  if (p.items_log2 >= 0) {
    j = (int64_t)blockIdx.x * (kBlock >> p.items_log2) + (threadIdx.x >> p.items_log2);
    item = threadIdx.x & ((1u << p.items_log2) - 1u);
    if (j >= p.n) return;
  } else {
    const uint32_t row = fdiv(blockIdx.x, p.chunks_div);
    j = row;
    item = (blockIdx.x - row * p.chunks_div.d) * kBlock + threadIdx.x;
  }
  if (item >= p.items) return;
  const int64_t off = p.offsets[j];
  if (off < p.lo || off > p.hi) return;
  int64_t os = 0, od = 0;
  uint32_t rem = item * p.vec;
#pragma unroll
  for (int d = kMaxDims - 1; d >= 0; --d) {
    if (d < p.ndim) {
      const uint32_t q = d == 0 ? 0u : fdiv(rem, p.div[d]);
      const uint32_t k = rem - q * p.div[d].d;
      rem = q;
      os += (int64_t)k * p.ss[d];
      od += (int64_t)k * p.sd[d];
    }
  }
  if (SCATTER) { os += j * p.row_stride; od += off; }
  else { os += off; od += j * p.row_stride; }
  if (V > 1 && p.vec > 1) {
    if ((off & 15) == 0) {
      Bytes<16> v = *reinterpret_cast<const Bytes<16> *>(p.src + os);
      reorder(v, p.swap_sc);
      *reinterpret_cast<Bytes<16> *>(p.dst + od) = v;
    } else {
#pragma unroll
      for (int e = 0; e < V; ++e) {
        Bytes<ES> v = *reinterpret_cast<const Bytes<ES> *>(p.src + os + e * ES);
        reorder(v, p.swap_sc);
        *reinterpret_cast<Bytes<ES> *>(p.dst + od + e * ES) = v;
      }
    }
  } else {
    Bytes<ES> v = *reinterpret_cast<const Bytes<ES> *>(p.src + os);
    reorder(v, p.swap_sc);
    *reinterpret_cast<Bytes<ES> *>(p.dst + od) = v;
  }
}

// Single elements per offset, the rows side contiguous (a[mask], a[index array] on a flat list):
// a lane takes four consecutive offsets (two 16-byte loads), moves the four elements, and
// handles the rows side as one piece of 4 * ES bytes - four times the bytes in flight per lane
// of the kernel above, whose lanes each wait on one offset and then on one element.  An
// offset outside [lo, hi] still skips its element alone.
template <int ES, bool SCATTER> __global__ __launch_bounds__(kBlock) void gather_scalar4_kernel(const GatherArgs p) {
  using E = Bytes<ES>;
  struct alignas(4 * ES) E4 { E e[4]; };
  using L2 = long long __attribute__((ext_vector_type(2)));
  const int64_t j0 = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * 4;
  if (j0 >= p.n) return;
  char *dst = p.dst;
  const char *src = p.src;
  if (j0 + 4 <= p.n) {
    const L2 o01 = *reinterpret_cast<const L2 *>(p.offsets + j0), o23 = *reinterpret_cast<const L2 *>(p.offsets + j0 + 2);
    const int64_t off[4] = {o01.x, o01.y, o23.x, o23.y};
    bool ok[4], all = true;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      ok[i] = off[i] >= p.lo && off[i] <= p.hi;
      all = all && ok[i];
    }
    if (SCATTER) {
      E4 v = *reinterpret_cast<const E4 *>(src + j0 * ES);
      reorder(v, p.swap_sc);
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (ok[i]) *reinterpret_cast<E *>(dst + off[i]) = v.e[i];
    } else {
      E4 v;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (ok[i]) v.e[i] = *reinterpret_cast<const E *>(src + off[i]);
      reorder(v, p.swap_sc);
      if (all) {
        if (ES == 4 && p.nt_rows) {   // (16 bytes per lane: a wavefront's store covers whole lines)
          using Q = uint32_t __attribute__((ext_vector_type(4)));
          Q q;
          __builtin_memcpy(&q, &v, 16);
          asm volatile("");
          __builtin_nontemporal_store(q, reinterpret_cast<Q *>(dst + j0 * ES));
          asm volatile("");
        } else {
          *reinterpret_cast<E4 *>(dst + j0 * ES) = v;
        }
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (ok[i]) *reinterpret_cast<E *>(dst + (j0 + i) * ES) = v.e[i];
      }
    }
  } else {
    for (int64_t j = j0; j < p.n; ++j) {
      const int64_t off = p.offsets[j];
      if (off < p.lo || off > p.hi) continue;
      E v = SCATTER ? *reinterpret_cast<const E *>(src + j * ES) : *reinterpret_cast<const E *>(src + off);
      reorder(v, p.swap_sc);
      if (SCATTER) *reinterpret_cast<E *>(dst + off) = v;
      else *reinterpret_cast<E *>(dst + j * ES) = v;
    }
  }
}

int done(hipError_t e) {
  if (e == hipSuccess) return OCN_OK;
  record_hip_error((int)e);
  return OCN_ERR_LAUNCH;
}

// the indexing kernels take tensors in native byte order only (one-byte scalars have no order)
bool other_byte_order(const ocn_tensor *t) {
  return t && t->byteswapped && t->dtype >= 0 && t->dtype < DT_COUNT && dt_size(dt_real_of(t->dtype)) > 1;
}

bool bad_tensor(const ocn_tensor *t) {
  if (!t || t->ndim < 0 || t->ndim > kMaxDims || t->dtype < 0 || t->dtype >= DT_COUNT) return true;
  for (int d = 0; d < t->ndim; ++d)
    if (t->size[d] < 0) return true;
  return false;
}
int64_t numel_of(const ocn_tensor *t) {
  int64_t n = 1;
  for (int d = 0; d < t->ndim; ++d) n *= t->size[d];
  return n;
}

int plan_mask(const ocn_tensor *mask, const int64_t *target_strides, MaskArgs *m) {
  if (bad_tensor(mask)) return mask ? OCN_ERR_SHAPE : OCN_ERR_NULLPTR;
  if (mask->dtype != DT_BOOL) return OCN_ERR_DTYPE;
  if (mask->ndim > 0 && !target_strides) return OCN_ERR_NULLPTR;
  const int64_t n = numel_of(mask);
  if (n >= ((int64_t)1 << 31)) return OCN_ERR_SHAPE;
  std::memset(m, 0, sizeof *m);
  m->n = (uint32_t)n;
  m->mask = (const char *)mask->base + mask->offset;
  // canonical dims in the mask's own (row-major) order: drop size 1, merge neighbours that both
  // the mask and the target walk as one longer dim
  int nd = 0;
  int64_t size[kMaxDims];
  for (int d = 0; d < mask->ndim; ++d) {
    if (mask->size[d] == 1) continue;
    const int64_t sz = mask->size[d], sm = mask->stride[d], st = target_strides[d];
    if (nd > 0 && m->sm[nd - 1] == sm * sz && m->st[nd - 1] == st * sz) {
      size[nd - 1] *= sz;
      m->sm[nd - 1] = sm;
      m->st[nd - 1] = st;
    } else {
      size[nd] = sz; m->sm[nd] = sm; m->st[nd] = st;
      ++nd;
    }
  }
  m->ndim = nd;
  for (int d = 0; d < nd; ++d) m->div[d] = make_fastdiv((uint32_t)size[d]);
  m->contig = (nd == 0 || (nd == 1 && m->sm[0] == 1)) && ((uintptr_t)m->mask % 16 == 0);
  m->nblocks = (uint32_t)((n + kMaskChunk - 1) / kMaskChunk);
  return OCN_OK;
}

}  // namespace
}  // namespace ocn

using namespace ocn;

extern "C" {

int ocn_index_offsets(const ocn_tensor *index, int64_t dim_size, int64_t stride_bytes, const ocn_tensor *offsets,
                      void *invalid_count, void *stream) {
  if (bad_tensor(index) || bad_tensor(offsets)) return (!index || !offsets) ? OCN_ERR_NULLPTR : OCN_ERR_SHAPE;
  if (other_byte_order(index) || other_byte_order(offsets)) return OCN_ERR_BYTEORDER;
  if (!invalid_count) return OCN_ERR_NULLPTR;
  if (index->dtype != DT_I64 || offsets->dtype != DT_I64) return OCN_ERR_DTYPE;
  if (index->ndim != offsets->ndim || dim_size < 0) return OCN_ERR_SHAPE;
  if (index->device != offsets->device) return OCN_ERR_DEVICE;
  IndexArgs a;
  std::memset(&a, 0, sizeof a);
  a.n = 1;
  for (int d = 0; d < index->ndim; ++d) {
    if (index->size[d] != offsets->size[d]) return OCN_ERR_SHAPE;
    a.size[d] = index->size[d];
    a.si[d] = index->stride[d];
    a.so[d] = offsets->stride[d];
    a.n *= index->size[d];
  }
  if (((intptr_t)index->base + index->offset) % 8 || ((intptr_t)offsets->base + offsets->offset) % 8) return OCN_ERR_ALIGN;
  for (int d = 0; d < index->ndim; ++d)
    if (index->size[d] > 1 && (a.si[d] % 8 || a.so[d] % 8)) return OCN_ERR_ALIGN;
  a.ndim = index->ndim;
  a.idx = (const char *)index->base + index->offset;
  a.off = (char *)offsets->base + offsets->offset;
  a.dim_size = dim_size;
  a.stride = stride_bytes;
  a.invalid = (unsigned long long *)invalid_count;
  // every check comes before the first launch: on error nothing has been enqueued or written
  const int64_t grid = std::min<int64_t>((a.n + kBlock - 1) / kBlock, max_launch_blocks());   // the kernel loops beyond that
  if (a.n > 0 && (!index->base || !offsets->base)) return OCN_ERR_NULLPTR;
  hipStream_t s = (hipStream_t)stream;
  hipLaunchKernelGGL(fill_u64_kernel, dim3(1), dim3(1), 0, s, a.invalid, 0ull);
  // both tensors contiguous in row-major order and 16-byte aligned: the flat kernel
  bool flat = ((uintptr_t)a.idx % 16) == 0 && ((uintptr_t)a.off % 16) == 0;
  int64_t expect = 8;
  for (int d = index->ndim - 1; d >= 0 && flat; --d) {
    if (a.size[d] != 1 && (a.si[d] != expect || a.so[d] != expect)) flat = false;
    expect *= a.size[d];
  }
  if (a.n > 0 && flat) {
    const int64_t npair = (a.n + 1) / 2;
    const int64_t fgrid = std::min<int64_t>((npair + kBlock - 1) / kBlock, max_launch_blocks());
    hipLaunchKernelGGL(index_offsets_flat_kernel, dim3((unsigned)fgrid), dim3(kBlock), 0, s, a, a.n * 8 >= ((int64_t)32 << 20) ? 1 : 0);
  } else if (a.n > 0) {
    hipLaunchKernelGGL(index_offsets_kernel, dim3((unsigned)grid), dim3(kBlock), 0, s, a);
  }
  return done(hipGetLastError());
}

size_t ocn_mask_offsets_workspace_bytes(const ocn_tensor *mask) {
  if (bad_tensor(mask)) return 0;
  const int64_t n = numel_of(mask);
  return (size_t)((n + kMaskChunk - 1) / kMaskChunk + 1) * sizeof(int64_t);
}

int ocn_mask_offsets(const ocn_tensor *mask, const int64_t *target_strides, void *offsets, int64_t capacity,
                     void *count, void *workspace, size_t workspace_bytes, void *stream) {
  MaskArgs m;
  const int rc = plan_mask(mask, target_strides, &m);
  if (rc != OCN_OK) return rc;
  if (!count || capacity < 0 || (capacity > 0 && !offsets)) return OCN_ERR_NULLPTR;
  if (((uintptr_t)offsets % 8) || ((uintptr_t)count % 8)) return OCN_ERR_ALIGN;
  hipStream_t s = (hipStream_t)stream;
  if (m.n == 0) {
    hipLaunchKernelGGL(fill_u64_kernel, dim3(1), dim3(1), 0, s, (unsigned long long *)count, 0ull);
    return done(hipGetLastError());
  }
  if (!mask->base) return OCN_ERR_NULLPTR;
  if (!workspace || workspace_bytes < ocn_mask_offsets_workspace_bytes(mask)) return OCN_ERR_WORKSPACE;
  if ((uintptr_t)workspace % 8) return OCN_ERR_ALIGN;
  m.block_counts = (int64_t *)workspace;
  m.offsets = (int64_t *)offsets;
  m.capacity = capacity;
  m.count = (int64_t *)count;
  m.nt_store = std::min<int64_t>(capacity, m.n) * 8 >= ((int64_t)32 << 20);  // too large to stay cached
  if (m.contig)
    hipLaunchKernelGGL(mask_count_contig_kernel, dim3((m.nblocks + kBlock / kWave - 1) / (kBlock / kWave)), dim3(kBlock),
                       0, s, m);
  else
    hipLaunchKernelGGL(mask_count_kernel, dim3(m.nblocks), dim3(kBlock), 0, s, m);
  hipLaunchKernelGGL(mask_scan_kernel, dim3(1), dim3(kScanBlock), 0, s, m);
  hipLaunchKernelGGL(mask_write_kernel, dim3(m.nblocks), dim3(kBlock), 0, s, m);
  return done(hipGetLastError());
}

// shared by gather and scatter: `rows` has shape [n, inner...], `inner` describes one indexed
// sub-tensor of the tensor the offsets point into
static int run_gather(bool scatter, const ocn_tensor *inner, const void *offsets, int64_t n, int64_t lo, int64_t hi,
                      const ocn_tensor *rows, void *stream) {
  if (bad_tensor(inner) || bad_tensor(rows)) return (!inner || !rows) ? OCN_ERR_NULLPTR : OCN_ERR_SHAPE;
  if (inner->dtype != rows->dtype) return OCN_ERR_DTYPE;
  // a copy of elements between two tensors of the same byte order needs no reversal; between
  // different orders every scalar is reversed on the way (section 3.1.3)
  const bool reorder_scalars = other_byte_order(inner) != other_byte_order(rows);
  if (inner->device != rows->device) return OCN_ERR_DEVICE;
  if (n < 0 || rows->ndim != inner->ndim + 1 || rows->size[0] != n) return OCN_ERR_SHAPE;
  for (int d = 0; d < inner->ndim; ++d)
    if (rows->size[d + 1] != inner->size[d]) return OCN_ERR_SHAPE;
  const int es = dt_size(inner->dtype);
  const int sc = dt_size(dt_real_of(inner->dtype));
  GatherArgs g;
  std::memset(&g, 0, sizeof g);
  const int64_t inner_elems = numel_of(inner);
  if (n == 0 || inner_elems == 0) return OCN_OK;
  if (!offsets || !inner->base || !rows->base) return OCN_ERR_NULLPTR;
  if ((uintptr_t)offsets % 8) return OCN_ERR_ALIGN;
  if (((intptr_t)inner->base + inner->offset) % sc || ((intptr_t)rows->base + rows->offset) % sc || rows->stride[0] % sc)
    return OCN_ERR_ALIGN;
  if (inner_elems >= ((int64_t)1 << 31)) return OCN_ERR_SHAPE;
  // canonical inner dims: drop size 1, order by the stride on the rows side (slowest first), merge
  struct D { int64_t size, si, sr; } d[kMaxDims];
  int nd = 0;
  for (int k = 0; k < inner->ndim; ++k) {
    if (inner->size[k] == 1) continue;
    if (inner->stride[k] % sc || rows->stride[k + 1] % sc) return OCN_ERR_ALIGN;
    d[nd++] = D{inner->size[k], inner->stride[k], rows->stride[k + 1]};
  }
  auto mag = [](int64_t v) { return v < 0 ? -v : v; };
  for (int a = 1; a < nd; ++a)
    for (int b = a; b > 0 && mag(d[b].sr) > mag(d[b - 1].sr); --b) std::swap(d[b], d[b - 1]);
  int m = 0;
  for (int k = 0; k < nd; ++k) {
    if (m > 0 && d[m - 1].si == d[k].si * d[k].size && d[m - 1].sr == d[k].sr * d[k].size) {
      d[m - 1].size *= d[k].size; d[m - 1].si = d[k].si; d[m - 1].sr = d[k].sr;
    } else {
      d[m++] = d[k];
    }
  }
  g.ndim = m;
  for (int k = 0; k < m; ++k) {
    g.div[k] = make_fastdiv((uint32_t)d[k].size);
    g.ss[k] = scatter ? d[k].sr : d[k].si;
    g.sd[k] = scatter ? d[k].si : d[k].sr;
  }
  g.src = scatter ? (const char *)rows->base + rows->offset : (const char *)inner->base + inner->offset;
  g.dst = scatter ? (char *)inner->base + inner->offset : (char *)rows->base + rows->offset;
  g.offsets = (const int64_t *)offsets;
  g.n = n;
  g.lo = lo;
  g.hi = hi;
  g.row_stride = rows->stride[0];
  g.swap_sc = reorder_scalars ? sc : 0;
  g.inner = (uint32_t)inner_elems;
  // 16-byte items along the rows' fastest dim when it is contiguous and everything else keeps
  // such items aligned (the offsets themselves are checked row by row in the kernel)
  const int vfull = 16 / es;
  g.vec = 1;
  if (vfull > 1 && m > 0 && d[m - 1].si == es && d[m - 1].sr == es && d[m - 1].size % vfull == 0 &&
      ((intptr_t)inner->base + inner->offset) % 16 == 0 && ((intptr_t)rows->base + rows->offset) % 16 == 0 &&
      rows->stride[0] % 16 == 0) {
    bool ok = true;
    for (int k = 0; k + 1 < m; ++k) ok = ok && d[k].si % 16 == 0 && d[k].sr % 16 == 0;
    if (ok) g.vec = (uint32_t)vfull;
  }
  g.items = (uint32_t)(inner_elems / g.vec);
  int64_t grid;
  if (g.items <= (uint32_t)kBlock) {   // short rows share a workgroup
    g.items_log2 = 0;
    while ((1u << g.items_log2) < g.items) ++g.items_log2;
    const int64_t rows_per_block = kBlock >> g.items_log2;
    grid = (n + rows_per_block - 1) / rows_per_block;
    g.chunks_div = make_fastdiv(1);
  } else {
    g.items_log2 = -1;
    const int64_t chunks = ((int64_t)g.items + kBlock - 1) / kBlock;
    g.chunks_div = make_fastdiv((uint32_t)chunks);
    grid = n * chunks;
  }
  const int64_t max_blocks = max_launch_blocks();
  hipStream_t s = (hipStream_t)stream;
  // single elements, the rows side contiguous and aligned for pieces of four: four offsets per lane
  if (inner_elems == 1 && es <= 8 && rows->stride[0] == es && (uintptr_t)offsets % 16 == 0 &&
      ((intptr_t)rows->base + rows->offset) % (4 * es) == 0) {
    const int64_t per_launch = max_blocks * kBlock * 4;   // a multiple of four offsets: later launches stay aligned
    for (int64_t j0 = 0; j0 < n; j0 += per_launch) {
      GatherArgs q = g;
      q.nt_rows = !scatter && n * es >= ((int64_t)32 << 20);
      q.n = std::min<int64_t>(per_launch, n - j0);
      q.offsets = g.offsets + j0;
      if (scatter) q.src = g.src + j0 * es;
      else q.dst = g.dst + j0 * es;
      const int64_t launch_grid = (q.n + 4 * kBlock - 1) / (4 * kBlock);
#define OCN_LAUNCH4(ES)                                                                                                  \
  if (scatter) hipLaunchKernelGGL((gather_scalar4_kernel<ES, true>), dim3((unsigned)launch_grid), dim3(kBlock), 0, s, q); \
  else hipLaunchKernelGGL((gather_scalar4_kernel<ES, false>), dim3((unsigned)launch_grid), dim3(kBlock), 0, s, q);
      switch (es) {
        case 1: OCN_LAUNCH4(1) break;
        case 2: OCN_LAUNCH4(2) break;
        case 4: OCN_LAUNCH4(4) break;
        default: OCN_LAUNCH4(8) break;
      }
#undef OCN_LAUNCH4
    }
    return done(hipGetLastError());
  }
  // A launch may not exceed 2^32 lanes: longer lists of offsets go out in several launches,
  // each over a contiguous run of rows (the kernels are independent of one another).
  const int64_t blocks_per_row_num = g.items_log2 >= 0 ? 1 : (int64_t)g.chunks_div.d;      // blocks per row ...
  const int64_t rows_per_block = g.items_log2 >= 0 ? (kBlock >> g.items_log2) : 1;          // ... or rows per block
  if (blocks_per_row_num > max_blocks) return OCN_ERR_SHAPE;   // a single row of 2^40 items: not a gather any more
  const int64_t rows_per_launch = g.items_log2 >= 0 ? max_blocks * rows_per_block : max_blocks / blocks_per_row_num;
  (void)grid;
  const GatherArgs all = g;
  for (int64_t j0 = 0; j0 < n; j0 += rows_per_launch) {
    g = all;
    g.n = std::min<int64_t>(rows_per_launch, n - j0);
    g.offsets = all.offsets + j0;
    if (scatter) g.src = all.src + j0 * all.row_stride;
    else g.dst = all.dst + j0 * all.row_stride;
    const int64_t launch_grid = g.items_log2 >= 0 ? (g.n + rows_per_block - 1) / rows_per_block : g.n * blocks_per_row_num;
#define OCN_LAUNCH(ES)                                                                                               \
  if (scatter) hipLaunchKernelGGL((gather_kernel<ES, true>), dim3((unsigned)launch_grid), dim3(kBlock), 0, s, g);   \
  else hipLaunchKernelGGL((gather_kernel<ES, false>), dim3((unsigned)launch_grid), dim3(kBlock), 0, s, g);
    switch (es) {
      case 1: OCN_LAUNCH(1) break;
      case 2: OCN_LAUNCH(2) break;
      case 4: OCN_LAUNCH(4) break;
      case 8: OCN_LAUNCH(8) break;
      default: OCN_LAUNCH(16) break;
    }
  }
#undef OCN_LAUNCH
  return done(hipGetLastError());
}

int ocn_gather(const ocn_tensor *a_inner, const void *offsets, int64_t n, int64_t lo, int64_t hi,
               const ocn_tensor *out, void *stream) {
  return run_gather(false, a_inner, offsets, n, lo, hi, out, stream);
}

int ocn_scatter(const ocn_tensor *src, const void *offsets, int64_t n, int64_t lo, int64_t hi,
                const ocn_tensor *out_inner, void *stream) {
  return run_gather(true, out_inner, offsets, n, lo, hi, src, stream);
}

}  // extern "C"
