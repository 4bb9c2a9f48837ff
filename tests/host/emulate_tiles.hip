// Host-side emulation of the tiled elementwise kernel's index arithmetic (no GPU needed).
//
// For randomly shaped and strided operands it replays, on the CPU, exactly the address and
// LDS-slot computations every lane of ew_tiled_kernel performs (using the kernel's own
// helper functions and the host-built argument tables) and checks that
//   * every global access stays inside its operand's byte range,
//   * every output element is written exactly once,
//   * every LDS read in the compute phase returns the element that belongs to that output
//     position (so staging order, slot numbering and swizzle agree), inside the LDS budget.
// Plans that qualify for the unclipped all-vector form of the kernel are replayed a second
// time through that form's argument tables (32-bit offsets, XOR-composed LDS addresses).
// Exit code 0 when every case passes.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../paper_1810_08723_amd/csrc/ew_launch.hpp"

using namespace ocn;

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd() {
  rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
  return (uint32_t)(rng_state >> 33);
}
static int rnd_in(int lo, int hi) { return lo + (int)(rnd() % (uint32_t)(hi - lo + 1)); }

struct HostTensor {
  ocn_tensor t;
  int64_t lo, hi;  // byte range relative to base
};

// a view with permuted dims over a dense buffer, optionally stepped along one axis
static HostTensor make_view(int dt, int ndim, const int64_t *sizes, char *base, bool allow_step) {
  HostTensor h;
  std::memset(&h, 0, sizeof h);
  int perm[8];
  for (int i = 0; i < ndim; ++i) perm[i] = i;
  for (int i = ndim - 1; i > 0; --i) std::swap(perm[i], perm[rnd() % (uint32_t)(i + 1)]);
  int step_axis = allow_step && ndim > 0 && (rnd() % 3 == 0) ? rnd_in(0, ndim - 1) : -1;
  const int es = dt_size(dt);
  int64_t acc = es;
  int64_t stride[8];
  for (int k = ndim - 1; k >= 0; --k) {  // perm[k] is the k-th slowest buffer axis
    const int ax = perm[k];
    const int64_t step = ax == step_axis ? 2 : 1;
    stride[ax] = acc * step;
    acc *= sizes[ax] * step;
  }
  h.t.base = base;
  h.t.dtype = dt;
  h.t.ndim = ndim;
  h.t.offset = 0;
  for (int i = 0; i < ndim; ++i) { h.t.size[i] = sizes[i]; h.t.stride[i] = stride[i]; }
  h.lo = 0;
  h.hi = acc;
  return h;
}

static int g_stats[8];  // tiled-or-generic, staged a, staged b, vector compute, vector staging, edge tiles, fast form, paired tiles

// Replay of ew_tiled_fast_kernel: returns 0 when every output element is written once, from the
// right input elements, with every access in range and aligned.
static int check_fast(const EwPlan &p, const HostTensor &a, const HostTensor &b, const HostTensor &o, int es,
                      int case_no) {
  const FastTiledArgs f = make_fast_tiled_args(p, es);
  const int VA = std::max(1, 16 / es), VC = 1 << p.vecw_o;
  const int64_t out_elems = (o.hi - o.lo) / es;
  std::vector<uint8_t> written(out_elems, 0);
  const int64_t lds_bytes = p.lds_bytes;
  std::vector<int64_t> lds(lds_bytes / es);  // global byte offset held by each LDS element, per area
  auto in_range = [&](const HostTensor &h, const char *ptr, int bytes) {
    const int64_t off = ptr - (char *)h.t.base;
    return off >= h.lo && off + bytes <= h.hi;
  };
  auto expect = [&](int64_t out_off, int64_t &ea, int64_t &eb) {
    ea = p.off_a; eb = p.off_b;
    int64_t rem = out_off - p.off_out;
    for (int d = 0; d < p.ndim; ++d) {
      const int64_t c = rem / p.out.stride[d];
      rem -= c * p.out.stride[d];
      ea += c * p.a.stride[d];
      eb += c * p.b.stride[d];
    }
    return rem == 0;
  };
#define FAIL(msg) do { std::printf("case %d (fast form): %s\n", case_no, msg); return 1; } while (0)
  for (int64_t blk = 0; blk < p.total_tiles; ++blk) {
    uint32_t t = (uint32_t)blk;
    if (f.pair_log2) {   // the kernel's workgroup -> tile map
      const uint32_t lg = (uint32_t)f.pair_log2, r = t & 7u, h = (t >> 3) & ((1u << lg) - 1u), q = t >> (3 + lg);
      t = (q << (3 + lg)) | (r << lg) | h;
    }
    int64_t bo = 0, ba = 0, bb = 0;
    for (int j = 0; j < f.ntd; ++j) {
      const uint32_t q = fastdiv(t, f.ntdiv[j]);
      const uint32_t tc = t - q * f.ntdiv[j].d;
      t = q;
      bo += (int64_t)tc * f.step[0][j]; ba += (int64_t)tc * f.step[1][j]; bb += (int64_t)tc * f.step[2][j];
    }
    if (t != 0) FAIL("tile index not exhausted");
    std::fill(lds.begin(), lds.end(), INT64_MIN);
    for (int y = 0; y < 2; ++y) {
      if (!(y == 0 ? f.stage_a : f.stage_b)) continue;
      const FastOrder &g = f.ord[y + 1];
      const HostTensor &h = y == 0 ? a : b;
      const char *gbase = y == 0 ? f.a + ba : f.b + bb;
      for (uint32_t tid = 0; tid < (uint32_t)kBlock; ++tid) {
        uint32_t off[3], slot;
        if (y == 0) fast_lane<2>(g, tid, off, slot); else fast_lane<4>(g, tid, off, slot);
        const uint32_t l = (swizzle(slot, f.swz[y]) << f.es_log2[y]) | f.lds_base[y];
        for (int jj = 0; jj < g.niter; ++jj) {
          const char *src = gbase + g.hi_off[y + 1][jj] + off[y + 1];
          if ((uintptr_t)src % 16 != 0) FAIL("misaligned staging load");
          if (!in_range(h, src, 16)) FAIL("staging load out of range");
          for (int i = 0; i < VA; ++i) {
            const uint32_t addr = l ^ (f.st_hi[y][jj] ^ f.st_el[y][i]);
            if (addr % es != 0 || (int64_t)addr + es > lds_bytes) FAIL("LDS write out of range");
            if (lds[addr / es] != INT64_MIN) FAIL("LDS element written twice");
            lds[addr / es] = (src + (int64_t)i * es) - (char *)h.t.base;
          }
        }
      }
    }
    const FastOrder &g = f.ord[0];
    const int EP = std::min(std::max(1, 16 / es), VC);
    for (uint32_t tid = 0; tid < (uint32_t)kBlock; ++tid) {
      uint32_t off[3], slot;
      fast_lane<7>(g, tid, off, slot);
      const uint32_t lane_slot = tid << f.vc_log2;
      uint32_t r[2];
      for (int y = 0; y < 2; ++y) r[y] = (swizzle(lane_slot, f.swz[y]) << f.es_log2[y]) | f.lds_base[y];
      for (int jj = 0; jj < g.niter; ++jj) {
        char *po = f.out + bo + g.hi_off[0][jj] + off[0];
        if ((uintptr_t)po % ((size_t)VC * es) != 0) FAIL("misaligned vector store");
        if (!in_range(o, po, VC * es)) FAIL("store out of range");
        for (int i = 0; i < VC; ++i) {
          char *pe = po + (int64_t)i * es;
          const int64_t oidx = (pe - (char *)o.t.base) / es;
          if (written[oidx]++) FAIL("output element written twice");
          int64_t ea, eb, got[2];
          if (!expect(pe - (char *)o.t.base, ea, eb)) FAIL("store between elements");
          for (int y = 0; y < 2; ++y) {
            if (y == 0 ? f.stage_a : f.stage_b) {
              const uint32_t addr = (r[y] ^ (f.rd_hi[y][jj] ^ f.rd_ch[y][i / EP])) + (uint32_t)(i % EP) * es;
              if ((r[y] ^ (f.rd_hi[y][jj] ^ f.rd_ch[y][i / EP])) % ((uint32_t)EP * es) != 0) FAIL("misaligned LDS read");
              if ((int64_t)addr + es > lds_bytes) FAIL("LDS read out of range");
              got[y] = lds[addr / es];
            } else {
              const HostTensor &h = y == 0 ? a : b;
              const char *src = (y == 0 ? f.a + ba : f.b + bb) + g.hi_off[y + 1][jj] + off[y + 1];
              if ((uintptr_t)src % ((size_t)VC * es) != 0) FAIL("misaligned direct load");
              if (!in_range(h, src, VC * es)) FAIL("direct load out of range");
              got[y] = (src + (int64_t)i * es) - (char *)h.t.base;
            }
          }
          if (got[0] != ea || got[1] != eb) {
            std::printf("case %d (fast form): wrong element: a %ld want %ld, b %ld want %ld (tile %ld tid %u pass %d i %d)\n",
                        case_no, (long)got[0], (long)ea, (long)got[1], (long)eb, (long)blk, tid, jj, i);
            return 1;
          }
        }
      }
    }
  }
#undef FAIL
  int64_t count = 0;
  for (auto w : written) count += w;
  if (count != p.numel) { std::printf("case %d (fast form): %ld of %ld output elements written\n", case_no, (long)count, (long)p.numel); return 1; }
  return 0;
}

static int check_case(int dt, int ndim, const int64_t *sizes, int case_no) {
  const int es = dt_size(dt);
  // fake, well separated and aligned base addresses (never dereferenced)
  char *base_a = (char *)0x100000000ull, *base_b = (char *)0x200000000ull, *base_o = (char *)0x300000000ull;
  HostTensor a = make_view(dt, ndim, sizes, base_a, true);
  HostTensor b = make_view(dt, ndim, sizes, base_b, true);
  HostTensor o = make_view(dt, ndim, sizes, base_o, false);
  EwPlan p;
  int rc = plan_elementwise(2, B_ADD, &a.t, &b.t, &o.t, 0, &p);
  if (rc != OCN_OK) { std::printf("case %d: plan rc=%d\n", case_no, rc); return 1; }
  if (p.kernel != OCN_KERNEL_EW_TILED && p.kernel != OCN_KERNEL_EW_GENERIC) return 0;  // rows: not this test
  if (!p.specialised) return 0;
  const TiledArgs t = make_tiled_args(p, es);
  g_stats[0]++; g_stats[1] += t.stage_a; g_stats[2] += t.stage_b; g_stats[3] += p.vecw_o > 0;
  g_stats[4] += (p.vecw_a > 0) + (p.vecw_b > 0);
  const uint32_t tile_elems = 1u << t.tile_bits;
  if (p.lds_bytes > 64 * 1024) { std::printf("case %d: LDS %ld\n", case_no, (long)p.lds_bytes); return 1; }
  const int64_t out_elems = (o.hi - o.lo) / es;
  std::vector<uint8_t> written(out_elems, 0);
  std::vector<int64_t> lds_a(tile_elems), lds_b(tile_elems);
  const int VA = std::max(1, 16 / es), VC = rows_vec(es, es);

  auto in_range = [&](const HostTensor &h, const char *ptr, int bytes) {
    const int64_t off = ptr - (char *)h.t.base;
    return off >= h.lo && off + bytes <= h.hi;
  };
  // expected input offsets of an output element, from its output byte offset
  auto expect = [&](int64_t out_off, int64_t &ea, int64_t &eb) {
    ea = p.off_a; eb = p.off_b;
    int64_t rem = out_off - p.off_out;
    for (int d = 0; d < p.ndim; ++d) {
      const int64_t c = rem / p.out.stride[d];
      rem -= c * p.out.stride[d];
      ea += c * p.a.stride[d];
      eb += c * p.b.stride[d];
    }
    return rem == 0;
  };

  for (int64_t blk = 0; blk < p.total_tiles; ++blk) {
    uint32_t tt = (uint32_t)blk;
    int64_t base_off_o = 0, base_off_a = 0, base_off_b = 0;
    uint32_t lim_dim[kMaxDims];
    bool full = true;
    for (int d = kMaxDims - 1; d >= 0; --d) {
      lim_dim[d] = 1;
      if (d < t.ndim) {
        const uint32_t q = d == 0 ? 0u : fastdiv(tt, t.ntdiv[d]);
        const uint32_t tc = tt - q * t.ntdiv[d].d;
        tt = q;
        const int64_t i0 = (int64_t)tc << t.tl[d], ext = (int64_t)1 << t.tl[d], rem = t.size[d] - i0;
        lim_dim[d] = (uint32_t)(rem < ext ? rem : ext);
        full = full && rem >= ext;
        if (rem < ext && blk == p.total_tiles - 1) g_stats[5]++;
        base_off_o += i0 * t.so[d]; base_off_a += i0 * t.sa[d]; base_off_b += i0 * t.sb[d];
      }
    }
    std::fill(lds_a.begin(), lds_a.end(), INT64_MIN);
    std::fill(lds_b.begin(), lds_b.end(), INT64_MIN);
    // staging
    for (int which = 1; which <= 2; ++which) {
      if (!(which == 1 ? t.stage_a : t.stage_b)) continue;
      const TileOrder &od = t.ord[which];
      const int V = od.vecw ? VA : 1;
      if (od.vecw && (1 << od.vecw) != VA) { std::printf("case %d: vecw mismatch\n", case_no); return 1; }
      const uint32_t nvec = tile_elems >> od.vecw;
      const char *gbase = (which == 1 ? t.a + base_off_a : t.b + base_off_b);
      const HostTensor &h = which == 1 ? a : b;
      std::vector<int64_t> &lds = which == 1 ? lds_a : lds_b;
      const TileSwizzle &z = t.swz[which - 1];
      for (uint32_t tid = 0; tid < (uint32_t)kBlock; ++tid) {
        const LanePos lo = lane_pos(od, tid);
        const uint32_t step = 1u << od.lds_shift[0];
        for (int jj = 0; jj < od.niter; ++jj) {
          const uint32_t e = tid + (uint32_t)jj * kBlock;
          int nn = e < nvec ? V : 0;
          if (!full && nn) nn = vec_inside(od, e, lim_dim);
          const char *src = gbase + lo.off[which] + od.hi_off[which][jj];
          const uint32_t slot = lo.slot + od.hi_slot[jj];
          if (nn == V && V > 1 && ((uintptr_t)src % 16) != 0) { std::printf("case %d: misaligned vector load\n", case_no); return 1; }
          for (int i = 0; i < nn; ++i) {
            if (!in_range(h, src + (int64_t)i * es, es)) { std::printf("case %d: staging read out of range\n", case_no); return 1; }
            const uint32_t ph = swizzle(slot + (uint32_t)i * step, z);
            if (ph >= tile_elems) { std::printf("case %d: LDS slot %u out of range\n", case_no, ph); return 1; }
            if (lds[ph] != INT64_MIN) { std::printf("case %d: LDS slot written twice\n", case_no); return 1; }
            lds[ph] = (src + (int64_t)i * es) - (char *)h.t.base;
          }
        }
      }
    }
    // compute
    const TileOrder &oo = t.ord[0];
    const int V = oo.vecw ? VC : 1;
    if (oo.vecw && (1 << oo.vecw) != VC) { std::printf("case %d: compute vecw mismatch\n", case_no); return 1; }
    const uint32_t nvec = tile_elems >> oo.vecw;
    for (uint32_t tid = 0; tid < (uint32_t)kBlock; ++tid) {
      const LanePos lo = lane_pos(oo, tid);
      for (int jj = 0; jj < oo.niter; ++jj) {
        const uint32_t e = tid + (uint32_t)jj * kBlock;
        int nn = e < nvec ? V : 0;
        if (!full && nn) nn = vec_inside(oo, e, lim_dim);
        char *po = t.out + base_off_o + lo.off[0] + oo.hi_off[0][jj];
        if (nn == V && V > 1 && ((uintptr_t)po % ((size_t)V * es)) != 0) { std::printf("case %d: misaligned vector store\n", case_no); return 1; }
        const uint32_t slot0 = e * (uint32_t)V;
        for (int i = 0; i < nn; ++i) {
          char *pe = po + (int64_t)i * es;
          if (!in_range(o, pe, es)) { std::printf("case %d: store out of range\n", case_no); return 1; }
          const int64_t oidx = (pe - (char *)o.t.base) / es;
          if (written[oidx]++) { std::printf("case %d: output element written twice\n", case_no); return 1; }
          int64_t ea, eb;
          if (!expect(pe - (char *)o.t.base, ea, eb)) { std::printf("case %d: store between elements\n", case_no); return 1; }
          // a
          int64_t got_a, got_b;
          if (t.stage_a) {
            const int EPC = std::min(std::max(1, 16 / es), V);
            const uint32_t ph = swizzle(slot0 + (uint32_t)(i / EPC * EPC), t.swz[0]) + (uint32_t)(i % EPC);
            if (ph >= tile_elems) { std::printf("case %d: LDS read out of range\n", case_no); return 1; }
            got_a = lds_a[ph];
          } else {
            const char *src = t.a + base_off_a + lo.off[1] + oo.hi_off[1][jj] + (int64_t)i * oo.stride[1][0];
            if (!in_range(a, src, es)) { std::printf("case %d: direct a read out of range\n", case_no); return 1; }
            if (nn == V && V > 1 && oo.stride[1][0] == es && i == 0 && ((uintptr_t)src % ((size_t)V * es)) != 0) { std::printf("case %d: misaligned direct a\n", case_no); return 1; }
            got_a = src - (char *)a.t.base;
          }
          if (t.stage_b) {
            const int EPC = std::min(std::max(1, 16 / es), V);
            const uint32_t ph = swizzle(slot0 + (uint32_t)(i / EPC * EPC), t.swz[1]) + (uint32_t)(i % EPC);
            if (ph >= tile_elems) { std::printf("case %d: LDS read out of range\n", case_no); return 1; }
            got_b = lds_b[ph];
          } else {
            const char *src = t.b + base_off_b + lo.off[2] + oo.hi_off[2][jj] + (int64_t)i * oo.stride[2][0];
            if (!in_range(b, src, es)) { std::printf("case %d: direct b read out of range\n", case_no); return 1; }
            if (nn == V && V > 1 && oo.stride[2][0] == es && i == 0 && ((uintptr_t)src % ((size_t)V * es)) != 0) { std::printf("case %d: misaligned direct b\n", case_no); return 1; }
            got_b = src - (char *)b.t.base;
          }
          if (got_a != ea || got_b != eb) {
            std::printf("case %d: wrong element: a %ld want %ld, b %ld want %ld (tile %ld tid %u pass %d i %d stage %d,%d vec %d,%d,%d)\n",
                        case_no, (long)got_a, (long)ea, (long)got_b, (long)eb, (long)blk, tid, jj, i, t.stage_a, t.stage_b,
                        p.vecw_o, p.vecw_a, p.vecw_b);
            return 1;
          }
        }
      }
    }
  }
  int64_t numel = 1;
  for (int i = 0; i < ndim; ++i) numel *= sizes[i];
  int64_t count = 0;
  for (auto w : written) count += w;
  if (count != numel) { std::printf("case %d: %ld of %ld output elements written\n", case_no, (long)count, (long)numel); return 1; }
  if (p.fast_tiled) {
    g_stats[6]++;
    if (p.pair_dim >= 0) g_stats[7]++;
    return check_fast(p, a, b, o, es, case_no);
  }
  return 0;
}

int main(int argc, char **argv) {
  const int ncases = argc > 1 ? std::atoi(argv[1]) : 400;
  const int dts[5] = {DT_U8, DT_I16, DT_F32, DT_F64, DT_C64};
  int tiled = 0;
  for (int c = 0; c < ncases; ++c) {
    // every sixth case: three to five small power-of-two extents (short runs of every operand:
    // the shapes whose neighbouring tiles share cache lines)
    const int ndim = c % 6 == 0 ? rnd_in(3, 5) : rnd_in(1, 5);
    int64_t sizes[8];
    int64_t total = 1;
    for (int i = 0; i < ndim; ++i) {
      const int kind = rnd_in(0, 3);
      sizes[i] = kind == 0 ? rnd_in(1, 4) : kind == 1 ? rnd_in(5, 20) : kind == 2 ? (1 << rnd_in(2, 6)) : rnd_in(21, 70);
      if (c % 3 == 0) sizes[i] = 1 << rnd_in(1, c % 6 == 0 ? 4 : 6);  // every third case: power-of-two extents (no clipped tiles)
      if (total * sizes[i] > 300000) sizes[i] = 2;
      total *= sizes[i];
    }
    const int dt = dts[rnd() % 5];
    if (check_case(dt, ndim, sizes, c)) {
      std::printf("FAILED case %d: dt=%d ndim=%d sizes=", c, dt, ndim);
      for (int i = 0; i < ndim; ++i) std::printf("%ld ", (long)sizes[i]);
      std::printf("\n");
      return 1;
    }
    ++tiled;
  }
  std::printf("ok: %d cases; %d used the tiled kernel (staged a %d, staged b %d, vector compute %d, "
              "vector staging %d, clipped tile dims %d, all-vector form %d, with grouped tiles %d)\n", tiled, g_stats[0],
              g_stats[1], g_stats[2], g_stats[3], g_stats[4], g_stats[5], g_stats[6], g_stats[7]);
  return 0;
}
