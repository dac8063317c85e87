// Pieces shared by the bf16 MFMA grouped-GEMM kernels (expert computation, ScMoE paper
// Eq. (1)): vector types, the LDS swizzle, the argument block, the epilogue's GELU forms and
// the persistent tile schedule.
#pragma once
#include "common.hpp"

#include <type_traits>

namespace scmoe {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

#define SCMOE_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define SCMOE_GLB_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

// XOR swizzle of the 16-byte chunk index inside an LDS row.  A 64-lane ds_read_b128 is
// served in four passes of 16 lanes, and on gfx950 the passes are NOT runs of consecutive
// lanes (measured with a pairwise timing probe): {0-3, 12-15, 20-27}, {4-11, 16-19, 28-31}
// and the same two sets + 32.  A fragment read of the 16x16x32 MFMA has lane l on row l % 16
// and chunk l / 16, so one pass covers rows 0-3 and 12-15 with one chunk and rows 4-11 with
// the next; the 16 accesses must fall into 16 distinct 16-byte bank groups of the 256-byte
// bank window.  With 128-byte rows (two rows per window) chunk ^ (row/2 % 8) does that; with
// 64-byte rows (four per window) chunk ^ (-(row/4) % 4).  (Checked by enumeration.)
template <int CPR>
__host__ __device__ constexpr int swz(int r) {
  return CPR == 8 ? ((r >> 1) & 7) : ((0 - (r >> 2)) & 3);
}


struct GemmArgs {
  const unsigned char* A;   // activations, bf16 [rows, Kd]
  int64_t lda;              // row stride of A in elements
  const int32_t* gather;    // row r of the packed order reads A[gather[r]]; nullptr = identity
  const int32_t* offsets;   // [E + 1] segment starts, device
  const unsigned char* W;   // bf16 [E, N, Kd], row stride ldw
  int64_t ldw;              // row stride of W in elements (>= Kd)
  const float* bias;        // [E, N] or nullptr
  unsigned char* C;         // bf16 [rows, N], row stride ldc
  int64_t ldc;
  int E, N, Kd;
  int nt;                   // column tiles
  int gelu_mode;
  int stream_out;           // store C with the streaming (non-temporal) hint
  // Fused output decode (optional; scatter == nullptr stores C[r, :] as is).  Packed row r
  // is written to row t = scatter[r] of C as  addend[t, :] + row_scale[t] * (sum + bias).
  const int32_t* scatter;
  const float* row_scale;
  const unsigned char* addend;   // bf16 [*, N], row stride ldadd; may be C itself
  int64_t ldadd;
  // Split-K of the last, partly filled round of tiles (optional; splitk_part == nullptr: off).
  float* splitk_part;            // SPLITK_PARTS partial tiles of BM x BN floats
  int* splitk_count;             // SPLITK_PARTS arrival counters, zero between launches
  // Optional dense extra segment with operands of its own (xrows == 0: none): xC[r, :] =
  // act(xA[r, :] . xW^T + xbias) for r < xrows, same N and Kd.  Its tiles come first in the
  // tile order and it has the segment id E.  (The shared expert riding in the launch of the
  // routed experts' first GEMM.)  Not combined with scatter.
  int xrows;
  const unsigned char* xA;
  int64_t xlda;
  const unsigned char* xW;       // bf16 [N, Kd], row stride xldw
  int64_t xldw;
  const float* xbias;            // [N] or nullptr
  unsigned char* xC;
  int64_t xldc;
};

// Scratch of the split-K tail: per XCD as many partial tiles as workgroups are resident
// there (64 at most on a 256-CU device: 32 CUs x 2 workgroups), 256 KiB each at most.
constexpr int SPLITK_PARTS = 8 * 64;
constexpr size_t SPLITK_TILE_BYTES = 256 * 256 * 4;
constexpr size_t SPLITK_COUNT_BYTES = SPLITK_PARTS * sizeof(int);
constexpr size_t SPLITK_WS_BYTES = SPLITK_COUNT_BYTES + 8 * 32 * SPLITK_TILE_BYTES;
constexpr int SPLITK_MAX = 8;    // most parts one tile is cut into
// Tiles are cut along K only from this K on.  Writing a part's partial sums and reading them
// back costs about as much as 20 k-tiles of 64, whatever K is (all workgroups do it at the same
// time, so it is memory traffic, not latency); below K = 2048 a tile is done sooner than that.
// (Measured, layer step: small 0.129 -> 0.119 ms, medium 0.659 -> 0.647 ms with the limit.)
constexpr int SPLITK_MIN_K = 2048;

// erf-form GELU for the bf16 epilogue: erf(v / sqrt 2) ~ v * P(v^2) on |v| <= 3 sqrt 2,
// saturated outside (degree-8 minimax fit; |error of GELU| < 6e-5, far below the bf16
// rounding of the stored value).  13 VALU operations, no transcendental.
__device__ __forceinline__ float gelu_erf_fast(float v) {
  const float vc = __builtin_amdgcn_fmed3f(v, -4.2426405f, 4.2426405f);
  const float u = vc * vc;
  float p = 1.1253472459449299e-10f;
  p = fmaf(p, u, -1.0743693046322278e-08f);
  p = fmaf(p, u, 4.5365794676399673e-07f);
  p = fmaf(p, u, -1.1292409908492118e-05f);
  p = fmaf(p, u, 0.0001871810673037544f);
  p = fmaf(p, u, -0.002218799665570259f);
  p = fmaf(p, u, 0.019636236131191254f);
  p = fmaf(p, u, -0.1326938420534134f);
  p = fmaf(p, u, 0.7978062629699707f);
  const float e = p * vc;
  const float h = 0.5f * v;
  return fmaf(h, e, h);
}

__device__ __forceinline__ float gelu_tanh_fast(float v) {
  // 0.5 v (1 + tanh u) == v / (1 + exp(-2u))
  const float u2 = -1.5957691216057308f * (v + 0.044715f * v * v * v);
  return v * __frcp_rn(1.0f + __expf(u2));
}

__device__ __forceinline__ uint32_t cvt_pk_bf16(float a, float b) {
  f32x2_t f = {a, b};
  bf16x2_t h = __builtin_convertvector(f, bf16x2_t);
  return __builtin_bit_cast(uint32_t, h);
}

// Sum of two pairs of bf16 in fp32, rounded once.
__device__ __forceinline__ uint32_t add_bf16x2(uint32_t a, uint32_t b) {
  const float lo = __uint_as_float(a << 16) + __uint_as_float(b << 16);
  const float hi = __uint_as_float(a & 0xffff0000u) + __uint_as_float(b & 0xffff0000u);
  return cvt_pk_bf16(lo, hi);
}

// A precaution between the last matrix instruction and instructions written out in asm that
// read its results: the compiler inserts the wait states an MFMA result needs ahead of the
// instructions it schedules itself, and is not known to do so ahead of these.
__device__ __forceinline__ void mfma_results_settle() {
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
}

// 16-byte store / loads at device scope (sc1: past the caches that are not shared by the whole
// device), for data handed from one workgroup to another inside a kernel.  The store is not
// waited for here (follow it with a vmcnt(0) wait before publishing); the load reads four
// pieces 1 KiB apart and returns when they have arrived.
__device__ __forceinline__ void store16_device_scope(float* p, f32x4_t v) {
  // (the wait state after it: a store of more than 8 bytes per lane still reads its data
  // registers when the next instruction issues, and the compiler, which keeps that hazard for
  // its own stores, does not know that this is one)
  asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void load4x16_device_scope(const float* p, f32x4_t& a, f32x4_t& b, f32x4_t& c, f32x4_t& d) {
  asm volatile(
      "global_load_dwordx4 %0, %4, off sc1\n\t"
      "global_load_dwordx4 %1, %4, off offset:1024 sc1\n\t"
      "global_load_dwordx4 %2, %4, off offset:2048 sc1\n\t"
      "global_load_dwordx4 %3, %4, off offset:3072 sc1\n\t"
      "s_waitcnt vmcnt(0)"
      : "=&v"(a), "=&v"(b), "=&v"(c), "=&v"(d)
      : "v"(p)
      : "memory");
}

// Sixteen such loads in flight at once: four pieces 1 KiB apart from each of four bases.  (The
// reader of split-K partial sums has nothing to overlap a round trip to memory with: what
// counts is how few round trips it makes.)
__device__ __forceinline__ void load16x16_device_scope(const float* p0, const float* p1, const float* p2,
                                                       const float* p3, f32x4_t (&t)[16]) {
  asm volatile(
      "global_load_dwordx4 %0, %16, off sc1\n\t"
      "global_load_dwordx4 %1, %16, off offset:1024 sc1\n\t"
      "global_load_dwordx4 %2, %16, off offset:2048 sc1\n\t"
      "global_load_dwordx4 %3, %16, off offset:3072 sc1\n\t"
      "global_load_dwordx4 %4, %17, off sc1\n\t"
      "global_load_dwordx4 %5, %17, off offset:1024 sc1\n\t"
      "global_load_dwordx4 %6, %17, off offset:2048 sc1\n\t"
      "global_load_dwordx4 %7, %17, off offset:3072 sc1\n\t"
      "global_load_dwordx4 %8, %18, off sc1\n\t"
      "global_load_dwordx4 %9, %18, off offset:1024 sc1\n\t"
      "global_load_dwordx4 %10, %18, off offset:2048 sc1\n\t"
      "global_load_dwordx4 %11, %18, off offset:3072 sc1\n\t"
      "global_load_dwordx4 %12, %19, off sc1\n\t"
      "global_load_dwordx4 %13, %19, off offset:1024 sc1\n\t"
      "global_load_dwordx4 %14, %19, off offset:2048 sc1\n\t"
      "global_load_dwordx4 %15, %19, off offset:3072 sc1\n\t"
      "s_waitcnt vmcnt(0)"
      : "=&v"(t[0]), "=&v"(t[1]), "=&v"(t[2]), "=&v"(t[3]), "=&v"(t[4]), "=&v"(t[5]), "=&v"(t[6]), "=&v"(t[7]),
        "=&v"(t[8]), "=&v"(t[9]), "=&v"(t[10]), "=&v"(t[11]), "=&v"(t[12]), "=&v"(t[13]), "=&v"(t[14]), "=&v"(t[15])
      : "v"(p0), "v"(p1), "v"(p2), "v"(p3)
      : "memory");
}

// f(integral_constant<int, I>) for I = B .. N-1, unrolled at compile time.
template <int B, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (B < N) {
    f(std::integral_constant<int, B>{});
    static_for<B + 1, N>(f);
  }
}

// Workgroup barrier of the main loops.  __syncthreads() carries workgroup-scope fences, for
// which the compiler drains the vector-memory counter (s_waitcnt vmcnt(0)): that would wait
// for every global -> LDS copy in flight, including the ones requested for later k-tiles, and
// undo the multi-stage pipeline.  The kernels wait for exactly the copies they need with an
// explicit vmcnt before the barrier; this barrier only orders the LDS traffic.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Persistent tile schedule.  Row tiles are counted from offsets[] on the device (no host
// round trip).  Workgroup ids congruent mod 8 run on one XCD.  The tiles form up to two
// ranges: the dense extra segment (if any) and the E segments of offsets[], segment after
// segment, each segment in the raster order "a group of up to GM row tiles x all column
// tiles" (so a group never mixes two experts' weights).  XCD x owns the x-th eighth of the
// extra segment's range; the other range is dealt to the XCDs in chunks of RR tiles, XCD
// after XCD, and only the rest that does not fill a round of chunks is cut into eighths (so
// every XCD gets the same amount of both kinds of work, and at any time all XCDs read the
// weights of the same one or two experts, which the memory-side cache then serves).  The
// workgroups of an XCD take the tiles of its share round-robin, so the tiles in flight on one
// XCD are neighbours and share A and W panels in its L2.
template <int BM, int BN, int GM>
struct TileSchedule {
  int mt_seg, nt, E, xt, xrows;   // row tiles of the offsets[] segments / of the extra segment
  const int32_t* offsets;
  int nslots;
  int a0, na, rr, b0;             // this XCD's share: tiles a0 .. a0+na-1 of the extra segment's
                                  // range; of the other range rr tiles out of the dealt chunks,
                                  // then tiles from b0 on of the undealt rest
  static constexpr int RR = 32;
  // Work items of this XCD.  Its `full` tiles fill whole rounds of nslots workgroups; the `rem`
  // tiles of the last, partly filled round are each cut along K into S parts (S > 1 only with
  // scratch for the partial sums), so that the round keeps (nearly) all workgroups busy.
  // Item order: first the rem * S parts (part w % S of local tile full + w / S), then the full
  // tiles (local tile = item - parts), then rem * FS finish items, one per FS-th of a cut tile,
  // which add the parts up and write the result.  A workgroup takes items slot, slot + nslots,
  // ...: a part is always the first item of its workgroup, a finish item the last, so the
  // partial sums are long written when they are read (the kernel still checks the arrival count).
  int full, rem, S, npart, ngemm, nfin, xcd;
  int cur_e = 0, cur_base = 0;    // where the last search through offsets[] ended (see locate)

  __device__ __forceinline__ TileSchedule(const GemmArgs& p, int nk, bool can_split, int FS)
      : mt_seg(0), nt(p.nt), E(p.E), xt((p.xrows + BM - 1) / BM), xrows(p.xrows), offsets(p.offsets) {
    for (int q = 0; q < E; ++q) mt_seg += (offsets[q + 1] - offsets[q] + BM - 1) / BM;
    xcd = blockIdx.x & 7;
    nslots = gridDim.x >> 3;
    auto share = [&](int total, int& first) {
      const int chunk = (total + 7) >> 3;
      first = xcd * chunk;
      const int last = (xcd + 1) * chunk < total ? (xcd + 1) * chunk : total;
      return last > first ? last - first : 0;
    };
    na = share(xt * nt, a0);
    const int routed = mt_seg * nt;
    rr = (routed / (8 * RR)) * RR;
    int n = share(routed - 8 * rr, b0);
    b0 += 8 * rr;
    n += na + rr;
    full = (n / nslots) * nslots;
    rem = n - full;
    S = 1;
    if (can_split && rem > 0) {
      S = nslots / rem;
      if (S > SPLITK_MAX) S = SPLITK_MAX;
      if (S > nk) S = nk;
      if (S < 1) S = 1;
    }
    npart = S > 1 ? rem * S : 0;
    ngemm = S > 1 ? npart + full : n;
    nfin = S > 1 ? rem * FS : 0;
  }
  // GEMM item (it < ngemm) -> local tile index and part (part < 0: the whole tile)
  __device__ __forceinline__ void item(int it, int& l, int& part) const {
    if (it < npart) {
      l = full + it / S;
      part = it - (it / S) * S;
    } else {
      l = it - npart;
      part = -1;
    }
  }
  // raster order inside a range of mt row tiles: tile l -> row tile, first column
  // (the fewest groups of at most GM row tiles, of sizes that differ by one at most: the first
  // `big` groups have one row tile more than the others)
  __device__ __forceinline__ void raster(int l, int mt, int& m, int& n0) const {
    const int ng = (mt + GM - 1) / GM;
    const int base = mt / ng, big = mt - base * ng;
    const int lbig = big * (base + 1) * nt;          // tiles in the larger groups
    int grows, first, r;
    if (l < lbig) {
      grows = base + 1;
      const int g = l / (grows * nt);
      first = g * grows;
      r = l - g * grows * nt;
    } else {
      grows = base;
      const int g = (l - lbig) / (grows * nt);
      first = big * (base + 1) + g * grows;
      r = (l - lbig) - g * grows * nt;
    }
    m = first + r % grows;
    n0 = (r / grows) * BN;
  }
  // local tile l -> expert e (E: the dense extra segment), packed rows [row0, row_end)
  // (row0 + BM may exceed row_end), column n0
  // The tiles of a workgroup come in ascending order, so the search through offsets[] goes on
  // from the expert of the previous tile (cur_e, with cur_base tiles in the experts before
  // it) instead of from expert 0: a dependent scalar load per expert passed, 2 us per tile
  // at 16 experts when started from 0 every time.
  __device__ __forceinline__ void locate(int l, int& e, int& row0, int& row_end, int& n0) {
    int mt;
    if (l < na) {
      raster(a0 + l, xt, mt, n0);
      e = E;
      row0 = mt * BM;
      row_end = xrows;
      return;
    }
    // Segment after segment, each in its own raster order: a raster group never holds rows
    // of two experts, so the workgroups that run side by side share one expert's weights.
    int t = l - na;
    t = (t < rr) ? ((t / RR) * 8 + xcd) * RR + t % RR : b0 + t - rr;
    row0 = 0;
    row_end = 1;
    n0 = 0;
    if (t < cur_base) {        // not expected; start over
      cur_e = 0;
      cur_base = 0;
    }
    int base = cur_base;
    for (e = cur_e; e < E; ++e) {
      const int s = offsets[e];
      const int c = offsets[e + 1] - s;
      const int ntile = (c + BM - 1) / BM;
      if (t - base < ntile * nt) {
        raster(t - base, ntile, mt, n0);
        row0 = s + mt * BM;
        row_end = s + c;
        cur_e = e;
        cur_base = base;
        break;
      }
      base += ntile * nt;
    }
    if (e == E) e = E - 1;   // not reachable for a tile of this XCD's share
  }
};

// Grouped GEMM for calls of very few rows (ffn_skinny.hip): true if a call with this upper
// bound on its packed rows is one for it.
bool gemm_skinny_fits(int max_rows, int E);
int launch_gemm_skinny(const GemmArgs& a, bool act, int max_rows, void* scratch, size_t scratch_bytes,
                       hipStream_t stream);

}  // namespace scmoe
