// Expert computation (ScMoE paper Eq. (1); experts are two-layer MLPs, Sec. 2.1) in bf16
// on the CDNA4 matrix cores: a grouped GEMM over variable-length expert segments.
//
//   C[r, n] = act( sum_k A[row(r), k] * W[e, n, k] + bias[e, n] ),  r in segment e
//
// Both operands are K-contiguous ([rows, K] activations, [N, K] weights), which is the
// layout v_mfma_f32_16x16x32_bf16 wants: each lane feeds 8 consecutive k of one row.
//
// Design (gfx950):
//  * Persistent workgroups; each takes BM x BN output tiles (one expert per tile) from a
//    schedule derived on the device from offsets[] (no host round trip), and requests the
//    first k-tiles of its next tile before it runs the epilogue of the current one.  The
//    tiles of the last, partly filled round are cut along K (see the split-K block below).
//  * Global -> LDS copies use the direct-to-LDS form of the global load (16 bytes per
//    lane, no VGPR staging).  Such a load writes 1 KiB of consecutive LDS per wave, so the
//    bank-conflict swizzle is applied on the global side: the lane that fills LDS slot
//    (row, c) fetches k-chunk  c ^ swz(row)  of that row.
//  * N LDS stages and double-buffered register fragments: global loads run N-1 k-tiles
//    ahead, LDS reads one half-step (16 MFMAs) ahead, issued one behind each MFMA; one
//    workgroup barrier per k-tile, which orders LDS traffic only (lds_barrier).
//  * The MFMA is issued with the weight fragment as its first operand, so a lane ends up
//    holding 4 consecutive output columns of one row; the epilogue re-assembles rows in a
//    small per-wave LDS patch and stores whole 128-byte lines.
//  * Workgroup ids congruent mod 8 land on one XCD and share its L2: the tiles in flight on
//    an XCD are neighbours inside one expert (they share A and W panels), and the XCDs are
//    dealt neighbouring chunks, so that all of them read the same experts' weights at a time
//    (TileSchedule).
//  * Rows can be gathered on load through an index array (the dispatch permutation, paper
//    Sec. 2.2 "input encode"), and the second GEMM can scatter, scale and add on store
//    ("output decode"), which lets the layer skip both permuted copies.
#include "mfma_common.hpp"
#include <atomic>

namespace scmoe {

template <int BM_, int BN_, int BK_, int WM_, int WN_, int NS_>
struct TileCfg {
  static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_, NS = NS_;   // NS: LDS stages
  static constexpr int WAVES = WM * WN, THREADS = 64 * WAVES;
  static constexpr int TM = BM / WM, TN = BN / WN;       // wave tile
  static constexpr int MI = TM / 16, NJ = TN / 16;       // 16x16 MFMA tiles per wave
  static constexpr int RB = BK * 2;                      // bytes of one LDS row
  static constexpr int CPR = RB / 16;                    // 16-byte chunks per row
  static constexpr int RPL = 64 / CPR;                   // rows filled by one wave-wide load
  static constexpr int A_BYTES = BM * RB, B_BYTES = BN * RB, STAGE = A_BYTES + B_BYTES;
  static constexpr int A_PER_WAVE = BM / RPL / WAVES, B_PER_WAVE = BN / RPL / WAVES;
  static constexpr int STG_ROW = TN * 2;                  // bytes of one row of a wave's epilogue staging patch
  static constexpr int STG_ROWS = (WAVES == 8) ? 32 : 16; // rows staged at a time (LDS budget)
  static constexpr int STG_BYTES = STG_ROWS * STG_ROW;
  static constexpr int LDS_BYTES = NS * STAGE + WAVES * STG_BYTES;
  // workgroups of this shape that fit one CU (512 VGPRs per SIMD lane, 160 KiB LDS)
  static constexpr int WG_PER_CU = (160 * 1024 / LDS_BYTES) < (8 / WAVES) ? (160 * 1024 / LDS_BYTES) : (8 / WAVES);
  // Row tiles per raster group.  A first GEMM (N = F) has many column tiles and an XCD's 32
  // tiles in flight are best a 6 x 5 patch of a group; a second GEMM (N = d) has few (8 at
  // d = 2048), and groups of 4 x 8 tiles coincide with the chunks the XCDs are dealt.
  static constexpr int GM_FIRST = 6, GM_SECOND = 4;
  static_assert(BM % (RPL * WAVES) == 0 && BN % (RPL * WAVES) == 0, "loads must divide evenly");
  static_assert((TM == 128 || TM == 64) && TN == 64 && (BK == 32 || BK == 64) && NS >= 2 && NS <= 4, "tile shape");
  static_assert(LDS_BYTES * WG_PER_CU <= 160 * 1024 && WG_PER_CU >= 1, "LDS budget");
};

// DEC: output decode in the epilogue of a second GEMM.  0: none.  1: row r of the packed
// output goes to token scatter[r]: C[scatter[r]] = addend[scatter[r]] + row_scale[scatter[r]] * row
// (addend may be null: nothing is added).
// 2: rows stay where they are: C[r] = addend[r] + row_scale[2 r] * row (row_scale: pairs of
// coefficients per row, the first one is used; either pointer may be null).
template <class CFG, bool ACT, bool OFF32, int DEC>
__global__ __launch_bounds__(CFG::THREADS, CFG::WG_PER_CU * CFG::WAVES / 4) void gemm_bf16_kernel(const GemmArgs p) {
  constexpr int BM = CFG::BM, BN = CFG::BN, BK = CFG::BK, RB = CFG::RB, CPR = CFG::CPR;
  constexpr int MI = CFG::MI, NJ = CFG::NJ, STAGE = CFG::STAGE, A_BYTES = CFG::A_BYTES;
  constexpr int NS = CFG::NS;
  constexpr int KS32 = BK / 32;                                 // 32-k MFMA steps per k-tile
  constexpr int HS = 2 * KS32;                                  // half-steps per k-tile
  constexpr int LPW = CFG::A_PER_WAVE + CFG::B_PER_WAVE;        // direct loads per wave and k-tile
  constexpr bool XSEG = ACT, DECODE = DEC != 0;
  static_assert(!(ACT && DEC != 0) && DEC >= 0 && DEC <= 2, "the output decode belongs to second GEMMs");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

  // ---- tile schedule ------------------------------------------------------------------------
  const int nk_all = p.Kd / BK;
  TileSchedule<BM, BN, ACT ? CFG::GM_FIRST : CFG::GM_SECOND> sched(p, nk_all, p.splitk_part != nullptr && p.Kd >= SPLITK_MIN_K, CFG::WAVES);
  const int nslots = sched.nslots;
  int it = blockIdx.x >> 3;                // work item: a tile, one K-part of a tile of the last round, or a finish item
  if (it >= sched.ngemm + sched.nfin) return;
  int nk = nk_all;                         // k-tiles of the current item

  // ---- per-lane source addresses of the direct-to-LDS loads -------------------------------
  // OFF32 (both operands span less than 4 GiB, checked on the host): an address is a
  // wave-uniform 64-bit base plus a 32-bit per-lane offset, which the load takes as scalar
  // base + vector offset: one register per load and no vector address arithmetic between
  // the barrier of a k-tile and its next MFMA.  Otherwise full 64-bit per-lane pointers.
  const unsigned char* aptr[OFF32 ? 1 : CFG::A_PER_WAVE];
  const unsigned char* bptr[OFF32 ? 1 : CFG::B_PER_WAVE];
  uint32_t aoff[OFF32 ? CFG::A_PER_WAVE : 1], boff[OFF32 ? CFG::B_PER_WAVE : 1];
  const unsigned char* abase = nullptr;     // OFF32: p.A / the expert's W, advanced to the item's first k-tile
  const unsigned char* wbase = nullptr;
  auto set_ptrs = [&](int e, int row0, int row_end, int n0, int kb) {   // kb: first k-tile of the item
    // The dense extra segment (operands of its own) exists for first GEMMs only, the fused
    // output decode for second GEMMs only and in an instantiation of its own: no kernel
    // carries code it does not run (the register allocation of the k loop feels every
    // scalar that is live across it).
    const bool xs = XSEG && e == p.E;
    const int64_t lda = xs ? p.xlda : p.lda, ldw = xs ? p.xldw : p.ldw;
    const int32_t* gather = xs ? nullptr : p.gather;
    const unsigned char* We = (xs ? p.xW : p.W + static_cast<int64_t>(e) * p.N * ldw * 2) + static_cast<int64_t>(kb) * RB;
    abase = (xs ? p.xA : p.A) + static_cast<int64_t>(kb) * RB;
    wbase = We;
#pragma unroll
    for (int i = 0; i < CFG::A_PER_WAVE; ++i) {
      const int row = (wave * CFG::A_PER_WAVE + i) * CFG::RPL + lane / CPR;
      const int kc = (lane % CPR) ^ swz<CPR>(row);
      int m = row0 + row;
      if (m > row_end - 1) m = row_end - 1;      // rows past the segment re-read its last row
      const int64_t src = gather ? gather[m] : m;
      if constexpr (OFF32) aoff[i] = static_cast<uint32_t>(src * lda * 2 + kc * 16);
      else aptr[i] = abase + src * lda * 2 + kc * 16;
    }
#pragma unroll
    for (int i = 0; i < CFG::B_PER_WAVE; ++i) {
      const int row = (wave * CFG::B_PER_WAVE + i) * CFG::RPL + lane / CPR;
      const int kc = (lane % CPR) ^ swz<CPR>(row);
      int n = n0 + row;
      if (n > p.N - 1) n = p.N - 1;
      if constexpr (OFF32) boff[i] = static_cast<uint32_t>(static_cast<int64_t>(n) * ldw * 2 + kc * 16);
      else bptr[i] = We + static_cast<int64_t>(n) * ldw * 2 + kc * 16;
    }
  };
  auto issue_loads = [&](int kt, int stage) {
    unsigned char* sa = smem + stage * STAGE + wave * CFG::A_PER_WAVE * 1024;
    unsigned char* sb = smem + stage * STAGE + A_BYTES + wave * CFG::B_PER_WAVE * 1024;
    const unsigned char* ak = abase + static_cast<int64_t>(kt) * RB;
    const unsigned char* wk = wbase + static_cast<int64_t>(kt) * RB;
    if constexpr (OFF32) asm volatile("" : "+s"(ak), "+s"(wk));   // the scalar sums stay scalar
#pragma unroll
    for (int i = 0; i < CFG::A_PER_WAVE; ++i) {
      if constexpr (OFF32) {
        asm volatile("" : "+v"(aoff[i]));   // keeps the offset a 32-bit register of its own
        __builtin_amdgcn_global_load_lds(SCMOE_GLB_PTR(ak + aoff[i]), SCMOE_LDS_PTR(sa + i * 1024), 16, 0, 0);
      } else {
        __builtin_amdgcn_global_load_lds(SCMOE_GLB_PTR(aptr[i] + static_cast<int64_t>(kt) * RB),
                                         SCMOE_LDS_PTR(sa + i * 1024), 16, 0, 0);
      }
    }
#pragma unroll
    for (int i = 0; i < CFG::B_PER_WAVE; ++i) {
      if constexpr (OFF32) {
        asm volatile("" : "+v"(boff[i]));
        __builtin_amdgcn_global_load_lds(SCMOE_GLB_PTR(wk + boff[i]), SCMOE_LDS_PTR(sb + i * 1024), 16, 0, 0);
      } else {
        __builtin_amdgcn_global_load_lds(SCMOE_GLB_PTR(bptr[i] + static_cast<int64_t>(kt) * RB),
                                         SCMOE_LDS_PTR(sb + i * 1024), 16, 0, 0);
      }
    }
  };
  auto issue_prologue = [&]() {
#pragma unroll
    for (int t = 0; t < NS; ++t)
      if (t < nk) issue_loads(t, t);
  };
  // wait until at most `tiles` of the newest k-tiles are still in flight (loads complete in
  // issue order, LPW loads per k-tile and wave)
  auto wait_vm = [&](auto n_c) {
    constexpr int n = decltype(n_c)::value;
    static_assert(n < 64, "vmcnt field");
    __builtin_amdgcn_s_waitcnt((n & 15) | ((n >> 4) << 14) | 0x0F70);
  };
  auto wait_tiles = [&](int tiles) {
    if (tiles >= 2) wait_vm(std::integral_constant<int, 2 * LPW>{});
    else if (tiles == 1) wait_vm(std::integral_constant<int, LPW>{});
    else wait_vm(std::integral_constant<int, 0>{});
  };

  // ---- fragment reads (the same for every tile) ---------------------------------------------
  // v_mfma_f32_16x16x32_bf16: an operand fragment is 16 rows x 32 k, lane l holding the 8
  // consecutive k of chunk l / 16 of row l % 16.  (Per flop it moves half the accumulator
  // data of the 32x32x16 form; with random operands a register-only loop of it sustains
  // 2.09 PFLOP/s at 2.05 GHz against 1.78 PFLOP/s at 1.78 GHz: the chip is power-limited.)
  // A wave's 128 x 64 tile is 8 x 4 such products per 32 k; it is walked in half-steps of
  // 16 MFMAs: the 4 weight fragments of the 32 k against row-subtiles 0-3, then against 4-7.
  const int wave_m = wave / CFG::WN, wave_n = wave % CFG::WN;
  const int l16 = lane & 15, lq = lane >> 4;
  // LDS byte address of (row l16, chunk lq) for each 32-k step of stage 0, swizzled (the
  // swizzle depends on row % 16 only).  Plain integers on top of an opaque base, so that the
  // address of any (stage, step, subtile) is one loop-invariant register plus an immediate.
  unsigned lds0 = static_cast<unsigned>(reinterpret_cast<uintptr_t>(SCMOE_LDS_PTR(smem)));
  asm volatile("" : "+s"(lds0));
  unsigned xb[KS32], wb[KS32];
#pragma unroll
  for (int ks = 0; ks < KS32; ++ks) {
    const unsigned cs = static_cast<unsigned>(((ks * 4 + lq) ^ swz<CPR>(l16)) << 4);
    xb[ks] = lds0 + (wave_m * CFG::TM + l16) * RB + cs;
    wb[ks] = lds0 + A_BYTES + (wave_n * CFG::TN + l16) * RB + cs;
  }
  typedef const __attribute__((address_space(3))) bf16x8_t* lds_frag_ptr;

  f32x4_t acc[MI][NJ];          // MI = 8 row-subtiles, NJ = 4 column-subtiles of 16
  bf16x8_t wf[2][NJ];           // weight fragments of a 32-k step, double-buffered: step q of stage R
                                // uses buffer (R * KS32 + q) % 2, consecutive steps alternate
  bf16x8_t xf[2][MI / 2];       // activation fragments of a half-step, one buffer per half
  static_assert((NS * KS32) % 2 == 0, "the weight-fragment buffers alternate over the unrolled k loop");
  // Reads for half-step hs of stage R.  Read order = order of first use.
  auto load_frags = [&](int R, int hs) {
    const int ks = hs >> 1, half = hs & 1, st = R * STAGE, wbuf = (R * KS32 + ks) & 1;
    if (half == 0) {
#pragma unroll
      for (int t = 0; t < (MI / 2 > NJ ? MI / 2 : NJ); ++t) {
        if (t < NJ) wf[wbuf][t] = *reinterpret_cast<lds_frag_ptr>(static_cast<uintptr_t>(wb[ks] + st + t * 16 * RB));
        if (t < MI / 2) xf[0][t] = *reinterpret_cast<lds_frag_ptr>(static_cast<uintptr_t>(xb[ks] + st + t * 16 * RB));
      }
    } else {
#pragma unroll
      for (int t = 0; t < MI / 2; ++t)
        xf[1][t] = *reinterpret_cast<lds_frag_ptr>(static_cast<uintptr_t>(xb[ks] + st + (MI / 2 + t) * 16 * RB));
    }
  };
  auto mfma_step = [&](int R, int hs) {
    const int ks = hs >> 1, half = hs & 1, wbuf = (R * KS32 + ks) & 1;
#pragma unroll
    for (int i = 0; i < MI / 2; ++i)
#pragma unroll
      for (int j = 0; j < NJ; ++j)
        acc[half * (MI / 2) + i][j] =
            __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[wbuf][j], xf[half][i], acc[half * (MI / 2) + i][j], 0, 0, 0);
  };
  // issue order of one half-step: MFMA, ds_read, MFMA, ds_read, ... (the reads feed the NEXT one)
  auto interleave = [&](auto next_hs_c) {
    constexpr int reads = (decltype(next_hs_c)::value & 1) ? MI / 2 : MI / 2 + NJ;
#pragma unroll
    for (int q = 0; q < reads; ++q) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, (MI / 2) * NJ - reads, 0);
  };

  int e, row0, row_end, n0, part;
  auto setup = [&](int item) {
    int l;
    sched.item(item, l, part);
    sched.locate(l, e, row0, row_end, n0);
    int kb = 0;
    nk = nk_all;
    if (part >= 0) {
      kb = part * nk_all / sched.S;
      nk = (part + 1) * nk_all / sched.S - kb;
    }
    set_ptrs(e, row0, row_end, n0, kb);
  };
  if (it < sched.ngemm) {
  setup(it);
  issue_prologue();
  for (;;) {
    // The accumulators start from the bias (lane: columns 16 j + 4 lq ... of its column block;
    // for a split-K item only in part 0).  Loading it here and not in the epilogue matters:
    // a load in the epilogue would wait behind the next tile's first k-tiles, which are
    // requested before the epilogue and complete in issue order.
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int n = n0 + wave_n * CFG::TN + j * 16 + 4 * lq;
      f32x4_t b = {0.0f, 0.0f, 0.0f, 0.0f};
      const bool xseg = XSEG && e == p.E;
      const float* bias = xseg ? p.xbias : p.bias + static_cast<int64_t>(e) * p.N;
      if ((xseg ? p.xbias : p.bias) != nullptr && part <= 0 && n < p.N)
        b = *reinterpret_cast<const f32x4_t*>(bias + n);
#pragma unroll
      for (int i = 0; i < MI; ++i) acc[i][j] = b;
    }

    // ---- main loop ---------------------------------------------------------------------------
    // Global -> LDS runs NS-1 k-tiles ahead; LDS -> registers runs one half-step ahead, each
    // ds_read slotted behind an MFMA; one workgroup barrier per k-tile.  After an epilogue
    // the stores of the previous tile share the counter with the loads, so everything is
    // waited for (the prologue loads had the whole epilogue to land).
    wait_vm(std::integral_constant<int, 0>{});
    lds_barrier();
    load_frags(0, 0);   // (stage 0, half-step 0)
    // One k-tile with its LDS stage known at compile time (the k loop is unrolled NS-fold),
    // so every LDS address is a loop-invariant register plus an immediate and no address
    // arithmetic has to share registers with fragments that are still in flight.
    auto k_tile = [&](auto stage_c, auto steady_c, int kt) {
      constexpr int stage = decltype(stage_c)::value;
      constexpr bool steady = decltype(steady_c)::value;   // k-tiles kt+1 .. kt+NS all exist
      constexpr int next = (stage + 1 == NS) ? 0 : stage + 1;
      static_for<0, HS - 1>([&](auto hs_c) {
        constexpr int hs = decltype(hs_c)::value;
        __builtin_amdgcn_sched_barrier(0);
        load_frags(stage, hs + 1);
        mfma_step(stage, hs);
        interleave(std::integral_constant<int, hs + 1>{});
      });
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (steady) {
        // No branches here: the compiler's counter bookkeeping merges conservatively at every
        // join, and a full LDS wait ahead of the last step would idle the MFMA pipe while all
        // waves fetch the next stage's first fragments at once.
        wait_tiles(NS - 2);
        lds_barrier();
        issue_loads(kt + NS, stage);
        __builtin_amdgcn_sched_barrier(0);
        load_frags(next, 0);
        mfma_step(stage, HS - 1);
        interleave(std::integral_constant<int, 0>{});
      } else {
        if (kt + 1 < nk) {
          // k-tiles kt+1 .. min(kt+NS-1, nk-1) are in flight; k-tile kt+1 must have landed.
          // After the barrier it has for every wave, and every wave holds its last fragments
          // of k-tile kt in registers, so this stage can be refilled with k-tile kt+NS.
          const int later = nk - kt - 2;
          wait_tiles(later < NS - 2 ? later : NS - 2);
          lds_barrier();
          if (kt + NS < nk) issue_loads(kt + NS, stage);
          load_frags(next, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        mfma_step(stage, HS - 1);
      }
    };
    using std::integral_constant;
    using std::bool_constant;
    int kt = 0;
    for (; kt + 2 * NS <= nk; kt += NS) {       // steady state: every load and read exists
      k_tile(integral_constant<int, 0>{}, bool_constant<true>{}, kt);
      k_tile(integral_constant<int, 1>{}, bool_constant<true>{}, kt + 1);
      if constexpr (NS > 2) k_tile(integral_constant<int, 2>{}, bool_constant<true>{}, kt + 2);
      if constexpr (NS > 3) k_tile(integral_constant<int, 3>{}, bool_constant<true>{}, kt + 3);
    }
    for (; kt < nk; kt += NS) {                 // the last k-tiles (fewer than 2 NS), guarded
      k_tile(integral_constant<int, 0>{}, bool_constant<false>{}, kt);
      if (kt + 1 < nk) k_tile(integral_constant<int, 1>{}, bool_constant<false>{}, kt + 1);
      if constexpr (NS > 2) {
        if (kt + 2 < nk) k_tile(integral_constant<int, 2>{}, bool_constant<false>{}, kt + 2);
      }
      if constexpr (NS > 3) {
        if (kt + 3 < nk) k_tile(integral_constant<int, 3>{}, bool_constant<false>{}, kt + 3);
      }
    }

    // ---- next tile: its first k-tiles are requested before this tile's epilogue -----------
    const int itn = it + nslots;
    const bool more = itn < sched.ngemm;
    const int crow0 = row0, crow_end = row_end, cn0 = n0, cpart = part, cw = it;   // (a part is item cw < npart)
    unsigned char* const cC = (XSEG && e == p.E) ? p.xC : p.C;        // output of the current tile's segment
    const int64_t cldc = (XSEG && e == p.E) ? p.xldc : p.ldc;
    lds_barrier();                    // every wave holds its last fragments: LDS is free
    // Fused output decode: everything the epilogue needs from memory is requested here, ahead
    // of the next tile's first k-tiles (loads complete in issue order, and the epilogue has
    // nothing to overlap a round trip with): the token of each of the wave's 128 packed rows
    // (lane l: rows l and 64 + l; other lanes get them by a lane permute), their gate
    // weights, and the 16-byte pieces of the first slab's output rows that this lane will
    // add to (each slab then requests the next one's before it does its own work).
    constexpr int SLABS = MI / 2, PIECES = 32 / 8;     // 32-row slabs; a store instruction covers 8 rows
    int dtok[2] = {0, 0};
    float dscale[2] = {1.0f, 1.0f};
    uint4 dadd[PIECES];
    auto addend_loads = [&](int i) {                   // slab i's pieces of the rows to add to
      const int n = cn0 + wave_n * CFG::TN + (lane & 7) * 8;
#pragma unroll
      for (int g = 0; g < PIECES; ++g) {
        const int tok = __shfl(dtok[i >> 1], (i & 1) * 32 + g * 8 + (lane >> 3));
        dadd[g] = make_uint4(0u, 0u, 0u, 0u);
        if (n < p.N && p.addend != nullptr)
          dadd[g] = *reinterpret_cast<const uint4*>(p.addend + (static_cast<int64_t>(tok) * p.ldadd + n) * 2);
      }
    };
    auto decode_loads = [&]() {
      if constexpr (DECODE) {
#pragma unroll
        for (int q = 0; q < CFG::TM / 64; ++q) {
          int r = crow0 + wave_m * CFG::TM + q * 64 + lane;
          if (r > crow_end - 1) r = crow_end - 1;      // rows past the segment: its last row (never stored)
          dtok[q] = (DEC == 1) ? p.scatter[r] : r;
        }
#pragma unroll
        for (int q = 0; q < CFG::TM / 64; ++q) {
          if (DEC == 1) dscale[q] = p.row_scale[dtok[q]];
          else dscale[q] = p.row_scale ? p.row_scale[2 * static_cast<int64_t>(dtok[q])] : 1.0f;
        }
        addend_loads(0);
      }
    };
    constexpr bool dec = DECODE;
    if (dec && cpart < 0) decode_loads();
    if (more) {
      setup(itn);
      issue_prologue();
    }

    // ---- split-K items: leave the partial sums in scratch and count the part in; the finish
    // items at the end of the launch add the parts up.  The partial sums and the counter move
    // with relaxed device-scope accesses (sc1: past the caches that are not shared by the whole
    // device), ordered by a plain wait for the stores; device-scope fences would write back and
    // invalidate the whole L2 of the XCD on every use, which costs more than the split saves.
    const bool finish = cpart < 0;
    if (cpart >= 0) {
      constexpr int TILE = BM * BN;
      constexpr int FRAGS = MI * NJ;                                  // 16-byte pieces (accumulators) per lane
      const size_t slot0 = static_cast<size_t>(sched.xcd) * nslots;   // this XCD's scratch slots
      // accumulator (i, j) of wave w and lane l sits at float4 index (w * FRAGS + i * NJ + j) * 64 + l
      float* mine = p.splitk_part + (slot0 + cw) * TILE + ((wave * FRAGS) * 64 + lane) * 4;
      mfma_results_settle();
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j) store16_device_scope(mine + ((i * NJ + j) * 64) * 4, acc[i][j]);
      wait_vm(std::integral_constant<int, 0>{});                      // this wave's stores have been performed
      lds_barrier();                                                  // ... and every wave's
      if (tid == 0)
        __hip_atomic_fetch_add(p.splitk_count + slot0 + cw / sched.S, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }

    // ---- epilogue: activation, bf16; rows re-assembled in LDS, 16-byte stores ----------------
    // acc[i][j][v] is output row (lane % 16) of row-subtile i and column 4 * (lane / 16) + v of
    // column-subtile j.  A wave stages 32-row slabs (two row-subtiles) of its tile in its
    // private LDS patch and writes them out with TN/8 lanes per row, so that every store
    // instruction covers whole 128-byte lines.
    unsigned char* stg = smem + NS * STAGE + wave * CFG::STG_BYTES;
#pragma unroll
    for (int i = 0; i < MI / 2; ++i) {
      const int mbase = crow0 + wave_m * CFG::TM + i * 32;
      if (!finish || mbase >= crow_end) continue;   // wave-uniform: not the last part / slab past the segment
      float rscale[2] = {1.0f, 1.0f};             // fused decode: the gate weights of this lane's two rows
      uint4 add_cur[PIECES];
      if (dec) {
#pragma unroll
        for (int u = 0; u < 2; ++u) rscale[u] = __shfl(dscale[i >> 1], (i & 1) * 32 + u * 16 + l16);
#pragma unroll
        for (int g = 0; g < PIECES; ++g) add_cur[g] = dadd[g];
        if (i + 1 < SLABS) addend_loads(i + 1);
      }
#pragma unroll
      for (int h = 0; h < 32 / CFG::STG_ROWS; ++h) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const int sr = u * 16 + l16 - h * CFG::STG_ROWS;   // this lane's row inside the staged rows
          const bool mine = sr >= 0 && sr < CFG::STG_ROWS;
#pragma unroll
          for (int j = 0; j < NJ; ++j) {
            float v[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) v[q] = acc[2 * i + u][j][q];
            if (ACT) {
#pragma unroll
              for (int q = 0; q < 4; ++q)
                v[q] = (p.gelu_mode == SCMOE_GELU_TANH) ? gelu_tanh_fast(v[q]) : gelu_erf_fast(v[q]);
            }
            if (dec) {
#pragma unroll
              for (int q = 0; q < 4; ++q) v[q] *= rscale[u];
            }
            uint2 o;
            o.x = cvt_pk_bf16(v[0], v[1]);
            o.y = cvt_pk_bf16(v[2], v[3]);
            // columns 16 j + 4 lq ...: 16-byte chunk 2j + lq/2 of the row (swizzled like the
            // operand tiles), half lq % 2 of it
            if (mine)
              *reinterpret_cast<uint2*>(stg + sr * CFG::STG_ROW + (((2 * j + (lq >> 1)) ^ swz<8>(sr)) << 4) + (lq & 1) * 8) = o;
          }
        }
#pragma unroll
        for (int r0 = 0; r0 < CFG::STG_ROWS; r0 += 8) {
          const int r = r0 + (lane >> 3);       // 8 lanes of 16 bytes per 128-byte row
          const int c = lane & 7;
          uint4 o = *reinterpret_cast<const uint4*>(stg + r * CFG::STG_ROW + ((c ^ swz<8>(r)) << 4));
          const int m = mbase + h * CFG::STG_ROWS + r;
          const int n = cn0 + wave_n * CFG::TN + c * 8;
          const int g = (h * CFG::STG_ROWS + r0) / 8;          // which of the slab's 8-row pieces
          int64_t orow = m;
          if (dec) orow = __shfl(dtok[i >> 1], (i & 1) * 32 + g * 8 + (lane >> 3));   // (all lanes take part)
          if (m < crow_end && n < p.N) {
            if (dec) {
              // output decode: this packed row belongs to token orow; add the row already there
              const uint4 a = add_cur[g];
              o.x = add_bf16x2(o.x, a.x);
              o.y = add_bf16x2(o.y, a.y);
              o.z = add_bf16x2(o.z, a.z);
              o.w = add_bf16x2(o.w, a.w);
            }
            if (p.stream_out) {
              // an output far larger than the caches: stored with the streaming hint, so that it
              // does not push the operand panels out of the L2
              typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
              const u32x4_t ov = {o.x, o.y, o.z, o.w};
              __builtin_nontemporal_store(ov, reinterpret_cast<u32x4_t*>(cC + (orow * cldc + n) * 2));
            } else {
              *reinterpret_cast<uint4*>(cC + (orow * cldc + n) * 2) = o;
            }
          }
        }
      }
    }
    if (!more) break;
    it = itn;
  }
  it += nslots;
  }

  // ---- finish items: one per wave tile of a tile that was cut along K ------------------------
  // The parts are added up in part order (the result does not depend on who arrived when) by a
  // workgroup that has nothing else left to do: each of its waves takes MI / WAVES row-subtiles
  // of the wave tile, so the 256 KiB of a tile's partial sums per part are read by all waves of
  // WAVES workgroups at once.  The parts were counted in long ago (they are the first items of
  // their workgroups, which have lower ids and started earlier); the count is checked anyway,
  // with a bounded wait, so that no wave can be left waiting for good.
  for (; it < sched.ngemm + sched.nfin; it += nslots) {
    constexpr int TILE = BM * BN, FRAGS = MI * NJ, FS = CFG::WAVES, RPW = MI / CFG::WAVES;
    static_assert(MI % CFG::WAVES == 0 && NJ == 4, "row-subtiles of a wave tile are shared out among the waves");
    const int f = it - sched.ngemm;
    const int lt = f / FS, region = f - lt * FS;                      // cut tile (0 .. rem-1), wave tile of it
    const int S = sched.S;
    const size_t slot0 = static_cast<size_t>(sched.xcd) * nslots;
    int* cnt = p.splitk_count + slot0 + lt;
    int fe, frow0, frow_end, fn0;
    sched.locate(sched.full + lt, fe, frow0, frow_end, fn0);
    if (tid == 0) {
      for (int spin = 0; spin < (1 << 22); ++spin) {
        if ((__hip_atomic_load(cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & 0xff) >= S) break;
        __builtin_amdgcn_s_sleep(16);
      }
    }
    lds_barrier();
    const bool xseg = XSEG && fe == p.E;
    unsigned char* const fC = xseg ? p.xC : p.C;
    const int64_t fldc = xseg ? p.xldc : p.ldc;
    const int rm = region / CFG::WN, rn = region - rm * CFG::WN;      // the wave tile's place in the tile
    const float* first = p.splitk_part + (slot0 + static_cast<size_t>(lt) * S) * TILE;
#pragma unroll
    for (int u = 0; u < RPW; ++u) {
      const int i = wave * RPW + u;                                   // row-subtile of the wave tile
      const int m = frow0 + rm * CFG::TM + i * 16 + l16;              // this lane's row
      if (frow0 + rm * CFG::TM + i * 16 >= frow_end) continue;        // (wave-uniform) subtile past the segment
      const int mc = m < frow_end ? m : frow_end - 1;
      // what the output decode needs of this row
      int64_t orow = mc;
      float rscale = 1.0f;
      if constexpr (DEC == 1) {
        orow = p.scatter[mc];
        rscale = p.row_scale[orow];
      } else if constexpr (DEC == 2) {
        if (p.row_scale != nullptr) rscale = p.row_scale[2 * static_cast<int64_t>(mc)];
      }
      f32x4_t a[NJ];
      const float* src = first + ((region * FRAGS + i * NJ) * 64 + lane) * 4;
      for (int q0 = 0; q0 < S; q0 += 4) {           // four parts per round trip (parts past S - 1: S - 1 again, not added)
        f32x4_t t[16];
        const float* pq[4];
#pragma unroll
        for (int u4 = 0; u4 < 4; ++u4) pq[u4] = src + static_cast<size_t>(q0 + u4 < S ? q0 + u4 : S - 1) * TILE;
        load16x16_device_scope(pq[0], pq[1], pq[2], pq[3], t);
#pragma unroll
        for (int u4 = 0; u4 < 4; ++u4) {
          if (q0 + u4 < S) {                         // (wave-uniform)
#pragma unroll
            for (int j = 0; j < NJ; ++j) a[j] = (q0 + u4 == 0) ? t[u4 * NJ + j] : a[j] + t[u4 * NJ + j];
          }
        }
      }
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const int n = fn0 + rn * CFG::TN + j * 16 + 4 * lq;           // four consecutive columns
        float v[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          v[c] = a[j][c];
          if (ACT) v[c] = (p.gelu_mode == SCMOE_GELU_TANH) ? gelu_tanh_fast(v[c]) : gelu_erf_fast(v[c]);
          if (DECODE) v[c] *= rscale;
        }
        uint2 o;
        o.x = cvt_pk_bf16(v[0], v[1]);
        o.y = cvt_pk_bf16(v[2], v[3]);
        if (m < frow_end && n < p.N) {
          if constexpr (DECODE) {
            if (p.addend != nullptr) {
              const uint2 ad = *reinterpret_cast<const uint2*>(p.addend + (orow * p.ldadd + n) * 2);
              o.x = add_bf16x2(o.x, ad.x);
              o.y = add_bf16x2(o.y, ad.y);
            }
          }
          *reinterpret_cast<uint2*>(fC + (orow * fldc + n) * 2) = o;
        }
      }
    }
    // the last of a tile's finish items leaves the counter at zero for the next launch
    lds_barrier();
    if (tid == 0) {
      const int old = __hip_atomic_fetch_add(cnt, 0x100, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if ((old >> 8) == FS - 1) __hip_atomic_store(cnt, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

// ---- host side --------------------------------------------------------------------------------

using CfgA = TileCfg<256, 256, 64, 2, 4, 2>;   // 8 waves, 128 KiB LDS, one workgroup per CU
using CfgB = TileCfg<256, 256, 32, 2, 4, 4>;   // 8 waves, 4 stages, 128 KiB LDS
#ifndef SCMOE_SMALL_TILES
#define SCMOE_SMALL_TILES 4      // in quarters of the CU count
#endif
using CfgS = TileCfg<128, 128, 32, 1, 2, 2>;   // 2 waves, 40 KiB LDS, four workgroups per CU: small problems
using CfgT = TileCfg<128, 128, 64, 2, 2, 3>;   // 4 waves of 64 x 64, 104 KiB LDS, one workgroup per CU: fewer 128 x 128 tiles than CUs

// Tile configuration in use: 0 unless scmoe_set_gemm_variant has set another.  The one piece of
// process-wide state of the library: an atomic, read once per launch.
static std::atomic<int> g_variant{0};
constexpr int NUM_VARIANTS = 4;

static int gemm_variant() { return g_variant.load(std::memory_order_relaxed); }

int set_gemm_variant(int v) {
  if (v < 0 || v >= NUM_VARIANTS) return SCMOE_ERR_ARG;
  g_variant.store(v, std::memory_order_relaxed);
  return SCMOE_OK;
}

bool ffn_mfma_supported(int d, int F) { return d > 0 && F > 0 && (d % 64) == 0 && (F % 64) == 0; }

// which output decode a launch asks for (see gemm_bf16_kernel)
static int decode_kind(const GemmArgs& a) {
  return a.scatter != nullptr ? 1 : (a.row_scale != nullptr || a.addend != nullptr) ? 2 : 0;
}

template <class CFG, bool ACT, bool OFF32, int DEC>
static int launch_gemm_impl(GemmArgs a, int max_rows, hipStream_t stream) {
  // the dynamic-LDS limit is a per-device attribute of the kernel: raise it once per device
  static std::atomic<bool> attr_set[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = -1;
  if (dev < 0 || !attr_set[dev].load(std::memory_order_acquire)) {
    hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_kernel<CFG, ACT, OFF32, DEC>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, CFG::LDS_BYTES);
    if (err != hipSuccess) return hip_fail(err);
    if (dev >= 0) attr_set[dev].store(true, std::memory_order_release);
  }
  // a first GEMM (ACT) may carry the dense extra segment, a second one the output decode (DEC)
  if (ACT ? (a.scatter != nullptr || a.addend != nullptr) : a.xrows != 0) return SCMOE_ERR_ARG;
  if (DEC != decode_kind(a) || (DEC == 1 && a.row_scale == nullptr)) return SCMOE_ERR_ARG;
  // upper bound on row tiles: sum_e ceil(c_e / BM) <= max_rows / BM + E
  const int mtb = max_rows / CFG::BM + a.E + (a.xrows + CFG::BM - 1) / CFG::BM;
  a.nt = (a.N + CFG::BN - 1) / CFG::BN;
  // Large outputs are streamed past the caches (measured: -0.6 to -1 % layer time at the large and
  // medium workloads).  The hidden rows of a first GEMM are read back by the second one right
  // away: below 256 MiB (the size of the memory-side cache) they are left to the caches (the
  // small workload loses 4 % otherwise); a second GEMM's rows are final and stream from 64 MiB on.
  a.stream_out = (static_cast<int64_t>(max_rows) + a.xrows) * a.N * 2 >= (int64_t(ACT ? 256 : 64) << 20);
  int slots = (mtb * a.nt + 7) / 8;                            // tiles per XCD, upper bound
  const int resident = (num_cus() / 8) * CFG::WG_PER_CU;       // workgroups one XCD holds at once
  if (slots > resident) {
    slots = resident;
  } else if (a.splitk_part != nullptr && a.Kd >= SPLITK_MIN_K) {
    // Far fewer tiles than workgroups the chip can hold: launch the workgroups anyway, so
    // that the schedule cuts every tile along K (as many slots as the split-K scratch has room
    // for).  From a quarter of the capacity on it no longer pays (measured: tiles cut in two
    // cost the small workload 6 %).
    const int room = SPLITK_PARTS / 8;
    const int want = resident < room ? resident : room;
    if (want >= 4 * slots) slots = want;
  }
  // the split-K scratch is laid out for 8 * slots partial tiles of this shape
  if (8 * slots > SPLITK_PARTS ||
      static_cast<size_t>(8) * slots * CFG::BM * CFG::BN * 4 > SPLITK_WS_BYTES - SPLITK_COUNT_BYTES) {
    a.splitk_part = nullptr;
    a.splitk_count = nullptr;
  }
  hipLaunchKernelGGL((gemm_bf16_kernel<CFG, ACT, OFF32, DEC>), dim3(8 * slots), dim3(CFG::THREADS), CFG::LDS_BYTES,
                     stream, a);
  return launch_status();
}

// a_rows: rows of the activation matrix that can be addressed (through `gather` any of them).
template <class CFG, bool ACT>
static int launch_gemm(const GemmArgs& a, int max_rows, int64_t a_rows, hipStream_t stream) {
  const int64_t lim = int64_t(1) << 32;
  const bool off32 = a_rows * a.lda * 2 < lim && static_cast<int64_t>(a.N) * a.ldw * 2 < lim &&
                     static_cast<int64_t>(a.xrows) * a.xlda * 2 < lim && static_cast<int64_t>(a.N) * a.xldw * 2 < lim;
  if constexpr (!ACT) {
    switch (decode_kind(a)) {
      case 1:
        return off32 ? launch_gemm_impl<CFG, ACT, true, 1>(a, max_rows, stream)
                     : launch_gemm_impl<CFG, ACT, false, 1>(a, max_rows, stream);
      case 2:
        return off32 ? launch_gemm_impl<CFG, ACT, true, 2>(a, max_rows, stream)
                     : launch_gemm_impl<CFG, ACT, false, 2>(a, max_rows, stream);
      default: break;
    }
  }
  return off32 ? launch_gemm_impl<CFG, ACT, true, 0>(a, max_rows, stream)
               : launch_gemm_impl<CFG, ACT, false, 0>(a, max_rows, stream);
}

template <bool ACT>
static int launch_variant(const GemmArgs& a, int max_rows, int64_t a_rows, hipStream_t stream) {
  switch (gemm_variant()) {
    case 1: return launch_gemm<CfgB, ACT>(a, max_rows, a_rows, stream);
    case 2: return launch_gemm<CfgS, ACT>(a, max_rows, a_rows, stream);
    case 3: return launch_gemm<CfgT, ACT>(a, max_rows, a_rows, stream);
    default: break;
  }
  // Variant 0 picks by size: a problem whose 256 x 256 tiles would not give every CU one is
  // cut into 128 x 128 tiles instead (four small workgroups per CU).
  const int64_t tiles = (static_cast<int64_t>(max_rows) / CfgA::BM + a.E + (a.xrows + CfgA::BM - 1) / CfgA::BM) *
                        ((a.N + CfgA::BN - 1) / CfgA::BN);
  if (tiles < SCMOE_SMALL_TILES * num_cus() / 4) {
    // Not even one 128 x 128 tile per CU: every workgroup is alone on its CU and walks all of K,
    // and what the launch lacks is waves.  Then a tile gets four waves of 64 x 64 (one per
    // SIMD) and k-tiles 64 deep in three LDS stages (half as many barriers and waits for the
    // same arithmetic).  Measured on the small workload's second GEMMs (192 tiles): 27.8 -> 18.4 us
    // and 32.7 -> 21.0 us (two waves with 64-deep k-tiles: 24.1 and 28.1).  With more tiles than
    // CUs the two-wave 32-deep form is faster, the first GEMM there by a factor of two.
    const int64_t tiles_s = ((static_cast<int64_t>(max_rows) + CfgS::BM - 1) / CfgS::BM + a.E +
                             (a.xrows + CfgS::BM - 1) / CfgS::BM) * ((a.N + CfgS::BN - 1) / CfgS::BN);
    if (tiles_s <= num_cus()) return launch_gemm<CfgT, ACT>(a, max_rows, a_rows, stream);
    return launch_gemm<CfgS, ACT>(a, max_rows, a_rows, stream);
  }
  return launch_gemm<CfgA, ACT>(a, max_rows, a_rows, stream);
}

__global__ void zero_ints(int* p, int n) {
  for (int i = threadIdx.x; i < n; i += blockDim.x) p[i] = 0;
}

size_t ffn_mfma_scratch_bytes() { return SPLITK_WS_BYTES; }
int ffn_mfma_counter_ints() { return SPLITK_PARTS; }

// Split-K scratch of a call: arrival counters first (every launch leaves them at zero again),
// then the partial tiles.  Without scratch the last round of tiles is not split.
struct SplitK { float* parts = nullptr; int* counters = nullptr; };
static int prepare_splitk(const FfnArgs& a, SplitK& sk, hipStream_t stream) {
  if (a.scratch == nullptr || a.scratch_bytes < SPLITK_WS_BYTES) return SCMOE_OK;
  sk.counters = static_cast<int*>(a.scratch);
  sk.parts = reinterpret_cast<float*>(static_cast<unsigned char*>(a.scratch) + SPLITK_COUNT_BYTES);
  if (a.scratch_zeroed) return SCMOE_OK;
  hipLaunchKernelGGL(zero_ints, dim3(1), dim3(256), 0, stream, sk.counters, SPLITK_PARTS);
  return launch_status();
}

// hidden = act(x . W1^T + b1)
static GemmArgs first_gemm(const FfnArgs& a, const SplitK& sk) {
  GemmArgs g{};
  g.A = static_cast<const unsigned char*>(a.x);
  g.lda = a.ldx;
  g.gather = a.gather;
  g.offsets = a.offsets;
  g.W = static_cast<const unsigned char*>(a.W1);
  g.ldw = a.ldw1;
  g.bias = a.b1;
  g.C = static_cast<unsigned char*>(a.hidden);
  g.ldc = a.ldh;
  g.E = a.E;
  g.N = a.F;
  g.Kd = a.d;
  g.gelu_mode = a.gelu_mode;
  g.splitk_part = sk.parts;
  g.splitk_count = sk.counters;
  return g;
}

// y = hidden . W2^T + b2, optionally decoded on store
static GemmArgs second_gemm(const FfnArgs& a, const SplitK& sk) {
  GemmArgs g{};
  g.A = static_cast<const unsigned char*>(a.hidden);
  g.lda = a.ldh;
  g.gather = nullptr;
  g.offsets = a.offsets;
  g.W = static_cast<const unsigned char*>(a.W2);
  g.ldw = a.ldw2;
  g.bias = a.b2;
  g.C = static_cast<unsigned char*>(a.y);
  g.ldc = a.ldy;
  g.E = a.E;
  g.N = a.d;
  g.Kd = a.F;
  g.gelu_mode = a.gelu_mode;
  g.scatter = a.scatter;
  g.row_scale = a.row_scale;
  g.addend = static_cast<const unsigned char*>(a.addend);
  g.ldadd = a.ldadd;
  g.splitk_part = sk.parts;
  g.splitk_count = sk.counters;
  return g;
}

// Only the second GEMM of a call may depend on work of another stream (a fused output decode
// adds to rows that the shared expert writes there): the first GEMM runs beside it.
static int wait_before_second(const FfnArgs& a, hipStream_t stream) {
  if (a.before_second == nullptr) return SCMOE_OK;
  const hipError_t e = hipStreamWaitEvent(stream, a.before_second, 0);
  return e == hipSuccess ? SCMOE_OK : hip_fail(e);
}

int ffn_mfma_bf16(const FfnArgs& a, hipStream_t stream) {
  if (!ffn_mfma_supported(a.d, a.F)) return SCMOE_ERR_ARG;
  if (a.max_rows <= 0) return SCMOE_OK;
  if (gemm_skinny_fits(a.max_rows, a.E)) {
    // a handful of rows per expert (a decode step): bound by streaming the weights, not by the matrix cores
    if (a.scatter == nullptr && (a.row_scale != nullptr || a.addend != nullptr)) return SCMOE_ERR_ARG;
    const SplitK none;
    const int st1 = launch_gemm_skinny(first_gemm(a, none), true, a.max_rows, a.scratch, a.scratch_bytes, stream);
    if (st1 != SCMOE_OK) return st1;
    const int stw = wait_before_second(a, stream);
    if (stw != SCMOE_OK) return stw;
    return launch_gemm_skinny(second_gemm(a, none), false, a.max_rows, a.scratch, a.scratch_bytes, stream);
  }
  SplitK sk;
  int st = prepare_splitk(a, sk, stream);
  if (st != SCMOE_OK) return st;
  st = launch_variant<true>(first_gemm(a, sk), a.max_rows, a.gather ? a.x_rows : a.max_rows, stream);
  if (st != SCMOE_OK) return st;
  st = wait_before_second(a, stream);
  if (st != SCMOE_OK) return st;
  return launch_variant<false>(second_gemm(a, sk), a.max_rows, a.max_rows, stream);
}

// The shared expert (one dense segment of se.max_rows rows, no gather) and the routed experts
// in three launches instead of four: the first GEMMs of both run as one grouped GEMM with the
// shared expert as an extra segment; the second GEMMs stay apart and in this order, because
// the routed one may decode into the rows the shared one writes (rt.addend).
int ffn_mfma_bf16_pair(const FfnArgs& se, const FfnArgs& rt, hipStream_t stream) {
  if (!ffn_mfma_supported(rt.d, rt.F) || se.d != rt.d || se.F != rt.F || se.E != 1 || se.gather != nullptr ||
      se.gelu_mode != rt.gelu_mode)
    return SCMOE_ERR_ARG;
  if (se.max_rows <= 0) return ffn_mfma_bf16(rt, stream);
  if (rt.max_rows <= 0) return ffn_mfma_bf16(se, stream);
  if (gemm_skinny_fits(se.max_rows, se.E) || gemm_skinny_fits(rt.max_rows, rt.E)) {
    const int st0 = ffn_mfma_bf16(se, stream);      // the shared expert first: rt may add to its rows
    if (st0 != SCMOE_OK) return st0;
    return ffn_mfma_bf16(rt, stream);
  }
  SplitK sks, skr;
  int st = prepare_splitk(se, sks, stream);
  if (st != SCMOE_OK) return st;
  st = prepare_splitk(rt, skr, stream);
  if (st != SCMOE_OK) return st;
  GemmArgs g1 = first_gemm(rt, skr);
  g1.xrows = se.max_rows;
  g1.xA = static_cast<const unsigned char*>(se.x);
  g1.xlda = se.ldx;
  g1.xW = static_cast<const unsigned char*>(se.W1);
  g1.xldw = se.ldw1;
  g1.xbias = se.b1;
  g1.xC = static_cast<unsigned char*>(se.hidden);
  g1.xldc = se.ldh;
  st = launch_variant<true>(g1, rt.max_rows, rt.gather ? rt.x_rows : rt.max_rows, stream);
  if (st != SCMOE_OK) return st;
  st = launch_variant<false>(second_gemm(se, sks), se.max_rows, se.max_rows, stream);
  if (st != SCMOE_OK) return st;
  return launch_variant<false>(second_gemm(rt, skr), rt.max_rows, rt.max_rows, stream);
}

}  // namespace scmoe
