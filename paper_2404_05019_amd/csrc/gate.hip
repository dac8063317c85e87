// Gate routing (ScMoE paper Eq. (2)-(4)): logits, top-k selection, gate weights.
//
// The logits decide an integer (the arg max), so their arithmetic is fixed by the ABI:
// fp32, one fused multiply-add per input feature in ascending feature order, then one
// rounded add of the bias.  Every kernel here keeps that chain intact per (token, expert) and
// finds its parallelism elsewhere.  The chains run on the matrix cores (gate_mfma_kernel: the
// fp32 matrix instruction is such a chain, four features at a time).  The two vector-ALU
// kernels remain for a W_g that is not 16-byte aligned and for a few tokens with many experts.
// gate_kernel: a workgroup owns 64 tokens, lane = token, and each of
// its eight waves (four for E <= 4) owns a contiguous group of EPL experts, so every lane
// runs EPL independent FMA chains.  x is staged through LDS in [64 tokens x 256 bytes] tiles
// (coalesced HBM reads although each lane walks its own row), and so is the matching slab
// of W_g, which all lanes of a wave then read at one address (an LDS broadcast); the next
// tile of both is prefetched into registers while the current one is consumed (with
// unconditional loads: predicated ones were each followed by a full wait, and the x pieces
// then lived in scratch memory).  Tried without gain: W_g
// through the scalar cache into SGPRs (3x slower: one scalar load per feature and wave) and
// one W read per 16 features with a DPP row broadcast inside the FMA (same time: LDS traffic
// is not what bounds the kernel).
#include "common.hpp"
#include "mfma_common.hpp"

#include <atomic>

namespace scmoe {

constexpr int GATE_TOK = 64;            // tokens per workgroup (one per lane)
constexpr int GATE_ROW_BYTES = 256;     // bytes of one token row staged per tile
constexpr int GATE_ROW_STRIDE = 272;    // LDS row stride: +16 B keeps the row reads conflict-free

// Top-k selection and gate weights of one token from its E logits `l` (Eq. (2)-(3)); also
// returns the maximum and the sum of exp(l - max) for the caller's softmax output.
__device__ __forceinline__ void route_token(const float* l, int E, int k, int normalize, bool write, int64_t t,
                                            int32_t* __restrict__ expert_idx, float* __restrict__ gate_w,
                                            float& m_out, float& sum_out) {
  // the j-th choice: largest logit among the experts not chosen yet, lowest index among
  // equals, a NaN only if nothing else is left
  int sel[SCMOE_MAX_TOPK];
  unsigned long long taken = 0ull;
#pragma unroll
  for (int j = 0; j < SCMOE_MAX_TOPK; ++j) {
    int best = -1;
    if (j < k) {
      for (int e = 0; e < E; ++e) {
        if ((taken >> e) & 1ull) continue;
        if (best < 0) { best = e; continue; }
        const float v = l[e], b = l[best];
        if (v > b || (b != b && v == v)) best = e;
      }
      taken |= 1ull << best;
    }
    sel[j] = best;
  }
  float m = -INFINITY;
  for (int e = 0; e < E; ++e)
    if (l[e] > m) m = l[e];
  float sum = 0.0f;
  for (int e = 0; e < E; ++e) sum += expf(l[e] - m);
  m_out = m;
  sum_out = sum;
  if (write) {
    // normalize: softmax over the selected logits only, taken relative to the first
    // (largest) one, whose term is exactly 1
    float z[SCMOE_MAX_TOPK];
    float zsum = 0.0f;
#pragma unroll
    for (int j = 0; j < SCMOE_MAX_TOPK; ++j) {
      z[j] = 0.0f;
      if (j < k) {
        z[j] = (j == 0) ? 1.0f : expf(l[sel[j]] - l[sel[0]]);
        zsum += z[j];
      }
    }
#pragma unroll
    for (int j = 0; j < SCMOE_MAX_TOPK; ++j) {
      if (j < k) {
        expert_idx[t * k + j] = sel[j];
        gate_w[t * k + j] = normalize ? z[j] / zsum : expf(l[sel[j]] - m) / sum;
      }
    }
  }
}

// NW waves per workgroup, each owning EPL experts; a lane owns TPL tokens (lane, lane + 64),
// which share every read of W_g: the kernel is bound by LDS bandwidth, and most of that
// traffic is the waves re-reading their slab of W_g for every 64 tokens.
template <int EPL, int NW, int TPL, bool BF16>
__global__ __launch_bounds__(64 * NW) void gate_kernel(
    const unsigned char* __restrict__ x, int64_t ldx, const float* __restrict__ Wg,
    const float* __restrict__ bias, int T, int d, int E, int k, int normalize,
    int32_t* __restrict__ expert_idx, float* __restrict__ gate_w, float* __restrict__ probs) {
  constexpr int EB = BF16 ? 2 : 4;                 // element bytes
  constexpr int KC = GATE_ROW_BYTES / EB;          // features per tile
  constexpr int GATE_THREADS = 64 * NW;
  constexpr int TOK = GATE_TOK * TPL;              // tokens per workgroup
  constexpr int GATE_XV = TOK * 16 / GATE_THREADS; // 16-byte pieces of x per thread and tile
  constexpr int EPAD = NW * EPL;                   // expert columns held in LDS (zero padded)
  constexpr int LGS = EPAD + 1;                    // row stride of the logit exchange buffer
  __shared__ __attribute__((aligned(16))) unsigned char xs[TOK * GATE_ROW_STRIDE];
  constexpr int WS_ELEMS = (KC * EPAD > TOK * LGS) ? KC * EPAD : TOK * LGS;
  __shared__ __attribute__((aligned(16))) float ws[WS_ELEMS];    // reused for the logits at the end
  __shared__ float row_max[TOK];
  __shared__ float row_sum[TOK];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int e0 = wave * EPL;
  const int t0 = blockIdx.x * TOK;

  float acc[TPL][EPL];
#pragma unroll
  for (int tp = 0; tp < TPL; ++tp)
#pragma unroll
    for (int j = 0; j < EPL; ++j) acc[tp][j] = 0.0f;

  // this thread's pieces of the x tile: piece c = tid + u*256 -> row c/16, 16-byte column c%16
  // The prefetched pieces are four named registers, not an array: as an array written under
  // `if (more tiles)` they were kept in scratch memory (stored and re-loaded once per tile).
  static_assert(GATE_XV == 2 || GATE_XV == 4, "pieces of x per thread");
  auto row_of = [&](int u) {
    int t = t0 + ((tid + u * GATE_THREADS) >> 4);
    if (t >= T) t = T - 1;
    return x + static_cast<int64_t>(t) * ldx * EB;
  };
  const unsigned char* const src0 = row_of(0);
  const unsigned char* const src1 = row_of(1);
  const unsigned char* const src2 = row_of(GATE_XV > 2 ? 2 : 0);
  const unsigned char* const src3 = row_of(GATE_XV > 2 ? 3 : 0);
  uint4 pre0, pre1, pre2 = {}, pre3 = {};
  // a piece past the end of a short last tile re-reads piece 0 and is not stored to LDS
  auto piece = [&](const unsigned char* row, int u, int kc0, int nvec) {
    const int c15 = (tid + u * GATE_THREADS) & 15;
    return *reinterpret_cast<const uint4*>(row + static_cast<int64_t>(kc0) * EB + (c15 < nvec ? c15 : 0) * 16);
  };
  auto fetch = [&](int kc0) {
    const int nvec = ((d - kc0 < KC) ? d - kc0 : KC) * EB / 16;
    pre0 = piece(src0, 0, kc0, nvec);
    pre1 = piece(src1, 1, kc0, nvec);
    if constexpr (GATE_XV > 2) {
      pre2 = piece(src2, 2, kc0, nvec);
      pre3 = piece(src3, 3, kc0, nvec);
    }
  };
  auto stage = [&](int u, const uint4& v, int nvec) {
    const int c = tid + u * GATE_THREADS;
    if ((c & 15) < nvec) *reinterpret_cast<uint4*>(xs + (c >> 4) * GATE_ROW_STRIDE + (c & 15) * 16) = v;
  };
  // this thread's pieces of the W_g slab of a tile: KC x EPAD floats, WV float4 pieces each
  constexpr int WV = (KC * EPAD / 4 + GATE_THREADS - 1) / GATE_THREADS;
  float4 wpre[WV];
  auto fetch_w = [&](int kc0) {
    const int kn = (d - kc0 < KC) ? d - kc0 : KC;
#pragma unroll
    for (int u = 0; u < WV; ++u) {
      const int c = (tid + u * GATE_THREADS) * 4;          // first of four expert columns
      const int i = c / EPAD, e = c - i * EPAD;
      float w[4] = {0.0f, 0.0f, 0.0f, 0.0f};
      if (i < kn) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (e + q < E) w[q] = Wg[static_cast<int64_t>(kc0 + i) * E + e + q];
      }
      wpre[u] = make_float4(w[0], w[1], w[2], w[3]);
    }
  };
  fetch(0);
  fetch_w(0);

  for (int kc0 = 0; kc0 < d; kc0 += KC) {
    const int kn = (d - kc0 < KC) ? d - kc0 : KC;  // features in this tile (multiple of 8)
    const int nvec = kn * EB / 16;                 // 16-byte pieces per row
    __syncthreads();                               // the previous tile has been consumed
    stage(0, pre0, nvec);
    stage(1, pre1, nvec);
    if constexpr (GATE_XV > 2) {
      stage(2, pre2, nvec);
      stage(3, pre3, nvec);
    }
#pragma unroll
    for (int u = 0; u < WV; ++u) {
      const int c = (tid + u * GATE_THREADS) * 4;
      if (c < KC * EPAD) *reinterpret_cast<float4*>(ws + c) = wpre[u];
    }
    __syncthreads();
    if (kc0 + KC < d) {                            // in flight while this tile is consumed
      fetch(kc0 + KC);
      fetch_w(kc0 + KC);
    }
    if (e0 < E) {
      const unsigned char* myrow = xs + lane * GATE_ROW_STRIDE;
      constexpr int XPV = 16 / EB;                 // features per 16-byte piece
      for (int c = 0; c < nvec; ++c) {
        uint32_t wd[TPL][4];
#pragma unroll
        for (int tp = 0; tp < TPL; ++tp) {
          const uint4 v = *reinterpret_cast<const uint4*>(myrow + tp * (GATE_TOK * GATE_ROW_STRIDE) + c * 16);
          wd[tp][0] = v.x; wd[tp][1] = v.y; wd[tp][2] = v.z; wd[tp][3] = v.w;
        }
        const float* wrow = ws + (c * XPV) * EPAD + e0;
#pragma unroll
        for (int q = 0; q < XPV; ++q) {
          float xv[TPL];
#pragma unroll
          for (int tp = 0; tp < TPL; ++tp) {
            if (BF16) {
              const uint32_t word = wd[tp][q >> 1];
              xv[tp] = __uint_as_float((q & 1) ? (word & 0xffff0000u) : (word << 16));
            } else {
              xv[tp] = __uint_as_float(wd[tp][q]);
            }
          }
          float wv[EPL];
          if (EPL >= 4) {
#pragma unroll
            for (int j = 0; j < EPL; j += 4) {
              const float4 f = *reinterpret_cast<const float4*>(wrow + q * EPAD + j);
              wv[j] = f.x; wv[j + 1] = f.y; wv[j + 2] = f.z; wv[j + 3] = f.w;
            }
          } else if (EPL == 2) {
            const float2 f = *reinterpret_cast<const float2*>(wrow + q * EPAD);
            wv[0] = f.x; wv[EPL - 1] = f.y;
          } else {
#pragma unroll
            for (int j = 0; j < EPL; ++j) wv[j] = wrow[q * EPAD + j];
          }
#pragma unroll
          for (int tp = 0; tp < TPL; ++tp)
#pragma unroll
            for (int j = 0; j < EPL; ++j) acc[tp][j] = __fmaf_rn(xv[tp], wv[j], acc[tp][j]);
        }
      }
    }
  }
  __syncthreads();                                 // ws is free: reuse it for the logits
  float* lg = ws;
#pragma unroll
  for (int tp = 0; tp < TPL; ++tp) {
#pragma unroll
    for (int j = 0; j < EPL; ++j) {
      if (e0 + j < E) {
        float v = acc[tp][j];
        if (bias != nullptr) v = __fadd_rn(v, bias[e0 + j]);
        lg[(tp * GATE_TOK + lane) * LGS + e0 + j] = v;
      }
    }
  }
  __syncthreads();

  if (wave < TPL) {                                // wave w routes tokens 64 w .. 64 w + 63 of the workgroup
    const int tl = wave * GATE_TOK + lane;
    route_token(lg + tl * LGS, E, k, normalize, t0 + tl < T, t0 + tl, expert_idx, gate_w, row_max[tl], row_sum[tl]);
  }
  if (probs != nullptr) {
    __syncthreads();
    const int ntok = (T - t0 < TOK) ? T - t0 : TOK;
    for (int c = tid; c < ntok * E; c += GATE_THREADS) {
      const int tok = c / E, e = c - tok * E;
      probs[static_cast<int64_t>(t0) * E + c] = expf(lg[tok * LGS + e] - row_max[tok]) / row_sum[tok];
    }
  }
}

// The chains on the matrix cores.  The fp32
// matrix instruction v_mfma_f32_16x16x4_f32 adds its four products to the accumulator one
// after the other in ascending k, each step rounded like a fused multiply-add (checked bit for
// bit against fmaf chains, subnormal sums and cancellation included), so one instruction
// advances the 16 x 16 chains of 16 tokens and 16 experts by four features: the same bits as
// the kernels below at a quarter of a dependent instruction per feature and chain.  With more
// than 16 experts a wave keeps EG = 2 or 4 accumulators, one per group of 16 experts, and
// every step issues EG independent instructions on the same x operand.
// A wave owns 16 tokens.  Nothing passes through registers on the way in: x rows and W_g are
// copied global -> LDS directly (so the compiler never waits for a register load, which with
// such copies in flight would drain all of them), x into a ring of XS stages per wave (a
// stage: 128 bytes of each of the 16 rows, two copies of 1 KiB), W_g in tiles of 256 / EG
// features into a ring of buffers shared by the workgroup (its natural [feature][expert] order
// is already the operand order: lane (c, kq) of step s reads expert c of feature 4 s + kq).
// Operands are read from LDS a few steps ahead of the matrix instructions that use them.  Waits
// are explicit: copies complete in issue order, so "all but the newest n" names a stage.
constexpr int GM_STAGE = 2048;           // bytes per stage: 16 rows x 128 bytes
constexpr int GM_WBUF = 16 * 1024;       // bytes per W_g buffer: a tile of 256 features of 16 experts, 128 of 32, 64 of 64

// LDS reads and waits of the matrix-core gate kernel's main loop, written out (see there).
// The result register of a read is not valid before an lds_wait that names it.
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return static_cast<uint32_t>(reinterpret_cast<uintptr_t>(SCMOE_LDS_PTR(p)));
}
template <int OFF>
__device__ __forceinline__ void lds_read_b32(uint32_t& r, uint32_t addr) {
  asm volatile("ds_read_b32 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
}
// a bf16 into the upper half of r (whose lower half stays as it is: zero), i.e. the fp32 value
template <bool BF16, int OFF>
__device__ __forceinline__ void lds_read_x(uint32_t& r, uint32_t addr) {
  if constexpr (BF16) asm volatile("ds_read_u16_d16_hi %0, %1 offset:%2" : "+v"(r) : "v"(addr), "n"(OFF));
  else asm volatile("ds_read_b32 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
}
// byte offset, inside a stage, of the x operand of step S (for the lane's row and feature)
template <bool BF16>
constexpr int gm_x_off(int S) { return BF16 ? (S >> 1) * 256 + (S & 1) * 8 : S * 256; }
// until at most N of the LDS reads issued so far are outstanding; x and w are valid afterwards
template <int N, int EG>
__device__ __forceinline__ void lds_wait(uint32_t& x, uint32_t (&w)[EG]) {
  static_assert(N >= 0 && N < 15 && (EG == 1 || EG == 2 || EG == 4), "lgkmcnt field");
  if constexpr (EG == 1) asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(x), "+v"(w[0]) : "n"(N));
  else if constexpr (EG == 2) asm volatile("s_waitcnt lgkmcnt(%3)" : "+v"(x), "+v"(w[0]), "+v"(w[1]) : "n"(N));
  else asm volatile("s_waitcnt lgkmcnt(%5)" : "+v"(x), "+v"(w[0]), "+v"(w[1]), "+v"(w[2]), "+v"(w[3]) : "n"(N));
}

// Shape of the kernel for EG groups of 16 experts (E <= 16 EG) and NW waves per workgroup.
template <bool BF16, int NW, int EG>
struct GateMfmaCfg {
  static constexpr int EB = BF16 ? 2 : 4;
  static constexpr int SF = 128 / EB;                 // features per stage of x
  static constexpr int SS = SF / 4;                   // steps (of four features) per stage
  static constexpr int KC = 256 / EG;                 // features per W_g tile: at most 16 KiB
  static constexpr int IPT = KC / SF;                 // stages per W_g tile
  static constexpr int WB = EG == 1 ? 2 : EG == 2 ? 3 : 4;             // W_g buffers: tile j + WB - 1 is requested when tile j begins
  static constexpr int XS = EG == 1 ? (NW == 8 ? 7 : 8) : EG == 2 ? 6 : 5;   // x ring stages per wave
  static constexpr int P = EG == 1 ? SS / 2 : EG == 2 ? 4 : 2;         // steps the operand reads run ahead of their use
  static constexpr int LGS = 16 * EG + 1;             // row stride of the logit exchange buffer
  static constexpr int TOK = 16 * NW;
  static constexpr int LDS = WB * GM_WBUF + NW * XS * GM_STAGE;
  static_assert(IPT >= 1 && SS % P == 0 && P <= SS / 2, "steps per stage and per tile");
  static_assert((P - 1) * (1 + EG) < 15, "LDS reads a wait can count");
  static_assert(XS >= 3 && 2 * (XS - 2) < 64, "ring depth");
  static_assert(TOK * LGS * 4 <= WB * GM_WBUF, "the logits fit the W_g buffers");
  static_assert(LDS + 2 * TOK * 4 <= 160 * 1024, "LDS of a compute unit");
};

template <bool BF16, int NW, int EG>
__global__ __launch_bounds__(64 * NW) void gate_mfma_kernel(
    const unsigned char* __restrict__ x, int64_t ldx, const float* __restrict__ Wg,
    const float* __restrict__ bias, int T, int d, int E, int k, int normalize,
    int32_t* __restrict__ expert_idx, float* __restrict__ gate_w, float* __restrict__ probs) {
  using C = GateMfmaCfg<BF16, NW, EG>;
  constexpr int EB = C::EB, SS = C::SS, KC = C::KC, IPT = C::IPT, WB = C::WB, XS = C::XS, P = C::P;
  constexpr int TOK = C::TOK, LGS = C::LGS;
  extern __shared__ __attribute__((aligned(1024))) unsigned char gm[];   // [WB W_g buffers][NW rings]
  __shared__ float row_max[TOK];
  __shared__ float row_sum[TOK];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int c16 = lane & 15, kq = lane >> 4;
  const int t0 = blockIdx.x * TOK;
  const int NS = d / 4;                                   // steps in all
  const int NI = (NS + SS - 1) / SS;                      // stages in all
  unsigned char* const ring = gm + WB * GM_WBUF + wave * (XS * GM_STAGE);

  // ---- copies --------------------------------------------------------------------------------
  // x: lane p of a copy fetches 16 bytes of row p % 16 at 16-byte column p / 16 of the 64 bytes
  // the copy covers; they land at ring position p.  Columns past the row's end re-read its last
  // 16 bytes (never consumed), and so do whole stages past the end, which keeps the number of
  // copies per stage fixed for the waits below.
  int trow = t0 + wave * 16 + c16;
  if (trow > T - 1) trow = T - 1;
  const unsigned char* const xrow = x + static_cast<int64_t>(trow) * ldx * EB;
  const int row_last = d * EB - 16;
  auto issue_x = [&](int i, int slot) {
    unsigned char* dst = ring + slot * GM_STAGE;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      int off = i * 128 + h * 64 + kq * 16;
      if (off > row_last) off = row_last;
      __builtin_amdgcn_global_load_lds(SCMOE_GLB_PTR(xrow + off), SCMOE_LDS_PTR(dst + h * 1024), 16, 0, 0);
    }
  };
  // W_g tile j is the bytes [4 KC E j, 4 KC E (j + 1)) of the matrix (whole rows), copied 1 KiB at
  // a time by the waves in turn; the last copy of a tile may reach into the next tile, and past
  // the end of the matrix a copy re-reads its last 16 bytes (never consumed).
  const unsigned char* const wg = reinterpret_cast<const unsigned char*>(Wg);
  const int64_t w_last = static_cast<int64_t>(d) * E * 4 - 16;
  const int w_copies = (E + EG - 1) / EG;                 // = ceil(4 KC E / 1024)
  auto issue_w = [&](int j, int buf) {
    unsigned char* dst = gm + buf * GM_WBUF;
    for (int u = wave; u < w_copies; u += NW) {
      int64_t off = static_cast<int64_t>(j) * (4 * KC) * E + u * 1024 + lane * 16;
      if (off > w_last) off = w_last;
      __builtin_amdgcn_global_load_lds(SCMOE_GLB_PTR(wg + off), SCMOE_LDS_PTR(dst + u * 1024), 16, 0, 0);
    }
  };
  auto wait_vm = [&](auto n_c) {
    constexpr int n = decltype(n_c)::value;
    static_assert(n < 64, "vmcnt field");
    __builtin_amdgcn_s_waitcnt((n & 15) | ((n >> 4) << 14) | 0x0F70);
    asm volatile("" ::: "memory");
  };
  // Copies that may still be on their way when stage i + 1 is needed: those of the XS - 2 stages
  // after it.  At the end of a W_g tile the next tile must be in as well; it was requested
  // (WB - 1) IPT stages of x ago (copies complete in issue order).
  using InFlight = std::integral_constant<int, 2 * (XS - 2)>;
  using InFlightTileEnd = std::integral_constant<int, (XS - 2 < (WB - 1) * IPT) ? 2 * (XS - 2) : 2 * (WB - 1) * IPT>;

  // ---- operands ------------------------------------------------------------------------------
  // x: token c16's 16 bytes of 16-byte column q sit at ring position 16 q + c16; W_g: feature
  // row f of the tile starts at byte 4 E f.  Lanes past the last expert read expert E - 1 again
  // (their rows of the product are never looked at).
  const int xl = c16 * 16 + kq * EB;
  int wl[EG];
#pragma unroll
  for (int g = 0; g < EG; ++g) wl[g] = (kq * E + (16 * g + c16 < E ? 16 * g + c16 : E - 1)) * 4;
  // Operand registers hold what the matrix instruction takes: fp32 bits (a bf16 in the upper half).
  // P steps are in registers or on their way at any time: step s uses slot s % P.
  uint32_t xr[P], wr[P][EG];
  f32x4_t acc[EG];
#pragma unroll
  for (int g = 0; g < EG; ++g) acc[g] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
  // experts are the rows of the product (first operand), tokens its columns: lane (c16, kq)
  // ends with token c16 and experts 16 g + 4 kq .. 16 g + 4 kq + 3 of every group g
  auto chain_step = [&](int slot_r) {
#pragma unroll
    for (int g = 0; g < EG; ++g)
      acc[g] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(wr[slot_r][g]), __uint_as_float(xr[slot_r]), acc[g], 0, 0, 0);
  };
  // step S of the stage at xs, whose W_g rows start at wrow (plain reads: the compiler waits for them)
  auto read_step = [&](int slot_r, const unsigned char* xs, const unsigned char* wrow, int S) {
    if (BF16) xr[slot_r] = static_cast<uint32_t>(*reinterpret_cast<const uint16_t*>(xs + gm_x_off<BF16>(S))) << 16;
    else xr[slot_r] = *reinterpret_cast<const uint32_t*>(xs + gm_x_off<BF16>(S));
#pragma unroll
    for (int g = 0; g < EG; ++g) wr[slot_r][g] = *reinterpret_cast<const uint32_t*>(wrow + wl[g]);
  };

#pragma unroll
  for (int j = 0; j < WB - 1; ++j)
    if (j * KC < d) issue_w(j, j);
#pragma unroll
  for (int i = 0; i < XS - 1; ++i) issue_x(i, i);
  wait_vm(InFlight{});                                    // the first W_g tiles and stage 0 are in LDS
  lds_barrier();
#pragma unroll
  for (int s = 0; s < P; ++s) read_step(s, ring + xl, gm + s * 16 * E, s);
  int slot = 0, slot_free = XS - 1;                       // ring slots of stage i and of stage i - 1
  int wbuf = 0, wbuf_free = WB - 1;                       // buffers of W_g tile j and of tile j - 1
  int i = 0;
  auto next_slot = [&]() {
    slot_free = slot;
    slot = (slot + 1 == XS) ? 0 : slot + 1;
  };
  auto next_wbuf = [&]() {
    wbuf_free = wbuf;
    wbuf = (wbuf + 1 == WB) ? 0 : wbuf + 1;
  };

  // Whole W_g tiles: IPT stages in straight-line code.  A dependent matrix instruction issues
  // only when the one before it has finished, and the wave issues in order, so everything else
  // (the reads of the operands P steps ahead, their addresses, the copies) is placed between
  // the matrix instructions, where it costs nothing, and not in a block in front of them.
  // The operand reads and their waits are written out here (lds_read_*, lds_wait): with
  // global -> LDS copies in flight every wait the compiler generates is a wait for everything,
  // i.e. for the reads issued just before.  LDS reads complete in order: a step's operands were
  // read P steps earlier, (P - 1) (1 + EG) reads ago.
  const int NTF = NS / (IPT * SS);
  for (int j = 0; j < NTF; ++j) {
    if ((j + WB - 1) * KC < d) issue_w(j + WB - 1, wbuf_free);   // that buffer was released by the last barrier
    const unsigned char* const wt = gm + wbuf * GM_WBUF;
    next_wbuf();
    const unsigned char* const wt_next = gm + wbuf * GM_WBUF;
    static_for<0, IPT>([&](auto q_c) {
      constexpr int q = decltype(q_c)::value;
      issue_x(i + XS - 1, slot_free);
      const uint32_t xs = lds_addr(ring + slot * GM_STAGE + xl);
      next_slot();
      const uint32_t xs_next = lds_addr(ring + slot * GM_STAGE + xl);
      static_for<0, SS>([&](auto s_c) {
        constexpr int s = decltype(s_c)::value, s2 = s + P;
        if constexpr (s == SS - P) {                      // the reads of the next stage begin with this step
          if (q == IPT - 1) {
            wait_vm(InFlightTileEnd{});                   // stage i + 1 and this wave's share of the next W_g tile are in LDS
            lds_barrier();                                // every wave has read its last operands of this tile; all shares of the next are in
          } else {
            wait_vm(InFlight{});                          // stage i + 1 is in LDS
          }
        }
        lds_wait<(P - 1) * (1 + EG)>(xr[s % P], wr[s % P]);
        chain_step(s % P);
        // (after the last stage: stale but in-bounds LDS, unused)
        const uint32_t xa = s2 < SS ? xs : xs_next;
        const unsigned char* const wrow = s2 < SS ? wt + (q * SS + s2) * 16 * E
                                        : q == IPT - 1 ? wt_next + (s2 - SS) * 16 * E : wt + ((q + 1) * SS + s2 - SS) * 16 * E;
        lds_read_x<BF16, gm_x_off<BF16>(s2 % SS)>(xr[s % P], xa);
#pragma unroll
        for (int g = 0; g < EG; ++g) lds_read_b32<0>(wr[s % P][g], lds_addr(wrow + wl[g]));
      });
      ++i;
    });
    // the operands just read are carried into the next round in registers the compiler may
    // copy: they have to be there before it does
    static_for<0, P>([&](auto s_c) { lds_wait<0>(xr[decltype(s_c)::value], wr[decltype(s_c)::value]); });
  }
  // The rest of a last, partial tile, stage by stage, with plain reads (the last stage may be short).
  while (i < NI) {
    const int q = i % IPT;
    if (q == 0 && (i / IPT + WB - 1) * KC < d) issue_w(i / IPT + WB - 1, wbuf_free);
    issue_x(i + XS - 1, slot_free);
    const int steps = NS - i * SS;                        // at least 2; SS or more unless this is the last stage
    const unsigned char* const xs = ring + slot * GM_STAGE + xl;
    next_slot();
    const unsigned char* const xs_next = ring + slot * GM_STAGE + xl;
    const unsigned char* const wt = gm + wbuf * GM_WBUF;
    const unsigned char* const wt_next = gm + (wbuf + 1 == WB ? 0 : wbuf + 1) * GM_WBUF;
    if (q == IPT - 1) next_wbuf();
    static_for<0, SS>([&](auto s_c) {
      constexpr int s = decltype(s_c)::value, s2 = s + P;
      if constexpr (s == SS - P) {
        if (q == IPT - 1 && i + 1 < NI) {
          wait_vm(InFlightTileEnd{});
          lds_barrier();
        } else {
          wait_vm(InFlight{});
        }
      }
      if (s < steps) chain_step(s % P);
      if (s2 < SS) read_step(s % P, xs, wt + (q * SS + s2) * 16 * E, s2);
      else read_step(s % P, xs_next, q == IPT - 1 ? wt_next + (s2 - SS) * 16 * E : wt + ((q + 1) * SS + s2 - SS) * 16 * E, s2 - SS);
    });
    ++i;
  }
  wait_vm(std::integral_constant<int, 0>{});              // no copy may land after the workgroup has given up its LDS
  if (EG == 1 && k == 1 && probs == nullptr) {
    // Top-1 without the probability output is routed in registers: a lane folds its four logits,
    // then the four lanes of a token (16 lanes apart, in ascending expert order) fold theirs.
    // Same rule and same operations in the same order as route_token, hence the same bits: the
    // largest logit wins, the lowest index among equals, a NaN only against another NaN; the
    // softmax denominator is summed expert after expert, handed from lane to lane.
    // (written with selects, on copies of the accumulators pinned to vector registers: the
    // same logic as nested branches on the accumulator tuple came out of the compiler with two
    // of the four logits overwritten by the first one)
    float v[4];
    float bv = 0.0f, mx = -INFINITY;
    int bi = -1;                                          // (no expert yet)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int e = 4 * kq + r;
      const bool valid = e < E;
      float a = acc[0][r];
      asm volatile("" : "+v"(a));
      if (bias != nullptr) a = __fadd_rn(a, bias[valid ? e : 0]);
      v[r] = a;
      const bool take = valid && (bi < 0 || a > bv || (bv != bv && a == a));
      bi = take ? e : bi;
      bv = take ? a : bv;
      mx = (valid && a > mx) ? a : mx;
    }
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {
      const float pv = __shfl_xor(bv, off), pm = __shfl_xor(mx, off);
      const int pi = __shfl_xor(bi, off);
      if (pi >= 0) {
        if (bi < 0) { bi = pi; bv = pv; }
        else {
          const bool mine_first = bi < pi;
          const float lo = mine_first ? bv : pv, hi = mine_first ? pv : bv;
          const int lo_i = mine_first ? bi : pi, hi_i = mine_first ? pi : bi;
          const bool take_hi = hi > lo || (lo != lo && hi == hi);
          bv = take_hi ? hi : lo;
          bi = take_hi ? hi_i : lo_i;
        }
      }
      if (pm > mx) mx = pm;
    }
    float w = 1.0f;                                       // normalize: the one selected logit's softmax over itself
    if (!normalize) {
      float t[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) t[r] = expf(v[r] - mx);
      float sum = 0.0f;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float sg = sum;                                   // (meaningful in the lanes that hold group g)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (4 * g + r < E) sg += t[r];
        sum = __shfl(sg, c16 + 16 * g);
      }
      w = expf(bv - mx) / sum;
    }
    const int t = t0 + wave * 16 + c16;
    if (kq == 0 && t < T) {
      expert_idx[t] = bi;
      gate_w[t] = w;
    }
    return;
  }
  lds_barrier();                                          // the W_g buffers are free: reuse them for the logits
  float* lg = reinterpret_cast<float*>(gm);
#pragma unroll
  for (int g = 0; g < EG; ++g) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int e = 16 * g + 4 * kq + r;
      if (e < E) {
        float v = acc[g][r];
        if (bias != nullptr) v = __fadd_rn(v, bias[e]);
        lg[(wave * 16 + c16) * LGS + e] = v;
      }
    }
  }
  __syncthreads();
  if (tid < TOK)
    route_token(lg + tid * LGS, E, k, normalize, t0 + tid < T, t0 + tid, expert_idx, gate_w, row_max[tid], row_sum[tid]);
  if (probs != nullptr) {
    __syncthreads();
    const int ntok = (T - t0 < TOK) ? T - t0 : TOK;
    for (int c = tid; c < ntok * E; c += 64 * NW) {
      const int tok = c / E, e = c - tok * E;
      probs[static_cast<int64_t>(t0) * E + c] = expf(lg[tok * LGS + e] - row_max[tok]) / row_sum[tok];
    }
  }
}

template <bool BF16, int NW, int EG>
static int launch_gate_mfma(const void* x, int64_t ldx, const float* Wg, const float* bias, int T, int d, int E,
                            int k, int normalize, int32_t* idx, float* gw, float* probs, hipStream_t stream) {
  constexpr int LDS = GateMfmaCfg<BF16, NW, EG>::LDS;
  static std::atomic<bool> attr_set[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = -1;
  if (dev < 0 || !attr_set[dev].load(std::memory_order_acquire)) {
    hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(&gate_mfma_kernel<BF16, NW, EG>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
    if (err != hipSuccess) return hip_fail(err);
    if (dev >= 0) attr_set[dev].store(true, std::memory_order_release);
  }
  dim3 grid((T + 16 * NW - 1) / (16 * NW)), block(64 * NW);
  hipLaunchKernelGGL((gate_mfma_kernel<BF16, NW, EG>), grid, block, LDS, stream, static_cast<const unsigned char*>(x), ldx,
                     Wg, bias, T, d, E, k, normalize, idx, gw, probs);
  return launch_status();
}

// Few tokens (decode steps, small batches: up to one workgroup of this kernel per CU;
// measured d = 2048, E = 16, bf16: 32 us against 59 us for 512 to 2048 tokens, 36 against 60 at
// 4096): the kernel above would run few workgroups whose lanes each walk a serial chain over
// 64 tokens' worth of LDS traffic.  Here a lane owns one (token,
// expert) chain: EPAD = E rounded up to a power of two lanes per token, 256 / EPAD tokens per
// workgroup.  W_g and the tokens' rows are staged through LDS in chunks of `kch` features
// with fully coalesced, independent loads (one memory latency per chunk, and the next chunk's
// are in flight meanwhile); W_g is transposed and x widened to fp32 on the way in, so a chain
// reads 4 consecutive features of its expert and of its token with one 16-byte LDS read each,
// 32 features ahead of the FMAs.  Same chain, same bits.
// Dynamic LDS: W chunk [E][kch + 4] fp32, then the x chunk [256 / EPAD][kch] fp32 with 16
// bytes of row padding (both paddings spread the rows over the banks).
constexpr int GATE_SMALL_WREGS = 32;   // W_g values a thread holds of a chunk: ceil(kch / tokens per workgroup)
constexpr int GATE_SMALL_XREGS = 8;    // 16-byte pieces of x a thread holds of a chunk
template <bool BF16>
__global__ __launch_bounds__(256) void gate_small_kernel(
    const unsigned char* __restrict__ x, int64_t ldx, const float* __restrict__ Wg,
    const float* __restrict__ bias, int T, int d, int E, int epad, int kch, int k, int normalize,
    int32_t* __restrict__ expert_idx, float* __restrict__ gate_w, float* __restrict__ probs) {
  constexpr int EB = BF16 ? 2 : 4;
  extern __shared__ __attribute__((aligned(16))) unsigned char gsm[];
  __shared__ float lg[256 + 256];                  // [tokens][epad + 1]
  __shared__ float row_max[256];
  __shared__ float row_sum[256];
  const int tid = threadIdx.x;
  const int tpw = 256 / epad;                      // tokens per workgroup
  const int tl = tid / epad, e = tid - tl * epad;
  const int t = blockIdx.x * tpw + tl;
  const bool active = t < T && e < E;
  const int ec = e < E ? e : E - 1;
  float* wsm = reinterpret_cast<float*>(gsm);
  const int wrs = kch + 4;                         // float stride of a staged (transposed) W_g row
  const int xrs = kch * 4 + 16;                    // byte stride of a staged x row (widened to fp32)
  unsigned char* xsm = gsm + static_cast<size_t>(wrs) * E * 4;
  float acc = 0.0f;
  // A chunk travels global memory -> registers -> LDS, and the next chunk's loads are in flight
  // while this one is consumed (with few workgroups nothing else hides their latency; loaded
  // and staged in one step, a call of 8 tokens spent 25 of its 40 us waiting for them).
  // Thread (tl, e) holds column e of W_g rows tl, tl + tpw, ... of the chunk (consecutive e:
  // coalesced reads; epad is a power of two, so no division by E is needed) and the 16-byte
  // pieces tid, tid + 256, ... of the x rows.  All loads are unconditional on clamped indices.
  constexpr int WMAX = GATE_SMALL_WREGS, XMAX = GATE_SMALL_XREGS;
  float wpre[WMAX];
  uint4 xpre[XMAX];
  auto fetch = [&](int c0) {
    const int kn = (d - c0 < kch) ? d - c0 : kch;
    const float* wsrc = Wg + static_cast<int64_t>(c0) * E + ec;
#pragma unroll
    for (int u = 0; u < WMAX; ++u) {
      int f = tl + u * tpw;
      if (f > kn - 1) f = kn - 1;
      wpre[u] = wsrc[static_cast<int64_t>(f) * E];
    }
    const int vpr = kn * EB / 16;                  // 16-byte pieces per row
    // 256 / tpw = epad consecutive threads share a row and take consecutive pieces of it, epad
    // more per pass (epad is a power of two: no division)
    int tr = blockIdx.x * tpw + tl;
    if (tr > T - 1) tr = T - 1;
    const unsigned char* xrow = x + (static_cast<int64_t>(tr) * ldx + c0) * EB;
#pragma unroll
    for (int u = 0; u < XMAX; ++u) {
      int v = e + u * epad;
      if (v > vpr - 1) v = vpr - 1;
      xpre[u] = *reinterpret_cast<const uint4*>(xrow + v * 16);
    }
  };
  auto stage = [&](int c0) {
    const int kn = (d - c0 < kch) ? d - c0 : kch;
    float* wdst = wsm + ec * wrs;
#pragma unroll
    for (int u = 0; u < WMAX; ++u) {
      const int f = tl + u * tpw;
      if (e < E && f < kn) wdst[f] = wpre[u];
    }
    const int vpr = kn * EB / 16;
#pragma unroll
    for (int u = 0; u < XMAX; ++u) {
      const int r = tl, v = e + u * epad;
      if (v < vpr) {
        if (BF16) {      // 8 bf16 -> 8 fp32 (exact), so that the chain below has no conversions in it
          const uint32_t wd[4] = {xpre[u].x, xpre[u].y, xpre[u].z, xpre[u].w};
          float4 lo, hi;
          lo.x = __uint_as_float(wd[0] << 16); lo.y = __uint_as_float(wd[0] & 0xffff0000u);
          lo.z = __uint_as_float(wd[1] << 16); lo.w = __uint_as_float(wd[1] & 0xffff0000u);
          hi.x = __uint_as_float(wd[2] << 16); hi.y = __uint_as_float(wd[2] & 0xffff0000u);
          hi.z = __uint_as_float(wd[3] << 16); hi.w = __uint_as_float(wd[3] & 0xffff0000u);
          *reinterpret_cast<float4*>(xsm + r * xrs + v * 32) = lo;
          *reinterpret_cast<float4*>(xsm + r * xrs + v * 32 + 16) = hi;
        } else {
          *reinterpret_cast<uint4*>(xsm + r * xrs + v * 16) = xpre[u];
        }
      }
    }
  };
  fetch(0);
  for (int c0 = 0; c0 < d; c0 += kch) {
    const int kn = (d - c0 < kch) ? d - c0 : kch;  // multiple of 8
    __syncthreads();                               // the previous chunk has been consumed
    stage(c0);
    __syncthreads();
    if (c0 + kch < d) fetch(c0 + kch);
    // The chain itself: operands of the next 32 features are read from LDS while the 32
    // dependent FMAs of the current ones run (one wave per SIMD: nothing else hides a wait).
    const float* xr = reinterpret_cast<const float*>(xsm + tl * xrs);
    const float* wc = wsm + ec * wrs;
    float4 xa[8], wa[8], xb[8], wb[8];                     // two operand sets, used in turn
    auto read32 = [&](float4 (&xv)[8], float4 (&wv)[8], int i0) {
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        xv[q] = *reinterpret_cast<const float4*>(xr + i0 + 4 * q);
        wv[q] = *reinterpret_cast<const float4*>(wc + i0 + 4 * q);
      }
    };
    auto fma32 = [&](const float4 (&xv)[8], const float4 (&wv)[8]) {
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        acc = __fmaf_rn(xv[q].x, wv[q].x, acc);
        acc = __fmaf_rn(xv[q].y, wv[q].y, acc);
        acc = __fmaf_rn(xv[q].z, wv[q].z, acc);
        acc = __fmaf_rn(xv[q].w, wv[q].w, acc);
      }
    };
    const int k32 = kn & ~63;                              // done 64 features per round
    if (k32 > 0) read32(xa, wa, 0);
    for (int i0 = 0; i0 < k32; i0 += 64) {
      read32(xb, wb, i0 + 32);
      fma32(xa, wa);
      read32(xa, wa, (i0 + 64 < k32) ? i0 + 64 : i0);      // (the last round re-reads a block of its own)
      fma32(xb, wb);
    }
    for (int i0 = k32; i0 < kn; i0 += 4) {                 // the rest of the chunk (a multiple of 8)
      const float4 xv = *reinterpret_cast<const float4*>(xr + i0);
      const float4 wv = *reinterpret_cast<const float4*>(wc + i0);
      acc = __fmaf_rn(xv.x, wv.x, acc);
      acc = __fmaf_rn(xv.y, wv.y, acc);
      acc = __fmaf_rn(xv.z, wv.z, acc);
      acc = __fmaf_rn(xv.w, wv.w, acc);
    }
  }
  if (active) {
    if (bias != nullptr) acc = __fadd_rn(acc, bias[e]);
    lg[tl * (epad + 1) + e] = acc;
  }
  __syncthreads();
  if (tid < tpw) {
    const int tt = blockIdx.x * tpw + tid;
    if (tt < T) route_token(lg + tid * (epad + 1), E, k, normalize, true, tt, expert_idx, gate_w, row_max[tid], row_sum[tid]);
  }
  if (probs != nullptr) {
    __syncthreads();
    if (active) probs[static_cast<int64_t>(t) * E + e] = expf(lg[tl * (epad + 1) + e] - row_max[tl]) / row_sum[tl];
  }
}

constexpr int GATE_SMALL_LANES = 65536;   // T * EPAD up to which the kernel above is used (256 workgroups: one per CU)

template <int EPL, int NW, int TPL>
static void launch_gate(int dtype, const void* x, int64_t ldx, const float* Wg, const float* bias,
                        int T, int d, int E, int k, int normalize, int32_t* idx, float* gw,
                        float* probs, hipStream_t stream) {
  dim3 grid((T + GATE_TOK * TPL - 1) / (GATE_TOK * TPL)), block(64 * NW);
  const unsigned char* xb = static_cast<const unsigned char*>(x);
  if (dtype == SCMOE_BF16)
    hipLaunchKernelGGL((gate_kernel<EPL, NW, TPL, true>), grid, block, 0, stream, xb, ldx, Wg, bias, T, d, E, k,
                       normalize, idx, gw, probs);
  else
    hipLaunchKernelGGL((gate_kernel<EPL, NW, TPL, false>), grid, block, 0, stream, xb, ldx, Wg, bias, T, d, E, k,
                       normalize, idx, gw, probs);
}

int gate_topk(const void* x, int64_t ldx, int dtype, const float* Wg, const float* bias, int T,
              int d, int E, int k, int normalize, int32_t* idx, float* gw, float* probs,
              hipStream_t stream) {
  if (!dtype_ok(dtype)) return SCMOE_ERR_DTYPE;
  if (T < 0 || d <= 0 || (d % 8) != 0 || E < 1 || E > SCMOE_MAX_EXPERTS) return SCMOE_ERR_SHAPE;
  if (k < 1 || k > SCMOE_MAX_TOPK) return SCMOE_ERR_ARG;
  if (k > E) return SCMOE_ERR_SHAPE;
  if (normalize != 0 && normalize != 1) return SCMOE_ERR_ARG;
  if (T == 0) return SCMOE_OK;
  if (!x || !Wg || !idx || !gw) return SCMOE_ERR_NULL;
  if (!view_ok(x, ldx, d, dtype)) return SCMOE_ERR_SHAPE;
  // The matrix-core kernel, at any number of tokens (measured against the two kernels below,
  // bf16, d = 2048: E = 16, 8 to 4096 tokens: 23 us against 24-26; 32768 tokens: 32 against 66 us;
  // E = 4, 8 to 8192 tokens: 18 against 66-69 us).  Its copies of W_g need 16-byte alignment.
  int epad = 1;
  while (epad < E) epad <<= 1;
  // (a few tokens with more than 16 experts: a wave would walk 2-4 chains per step alone; the
  // one-lane-per-chain kernel below is 10-20 % faster there: 64 tokens, d = 2048, E = 32: 35
  // against 43 us, E = 64: 75 against 80)
  const bool few_many = E > 16 && static_cast<int64_t>(T) * epad <= GATE_SMALL_LANES / 8;
  if (aligned16(Wg) && !few_many) {
    // A wave takes 16 tokens.  Up to one wave per SIMD: one workgroup of four waves per CU (fewer
    // waves per workgroup when that leaves CUs idle); beyond that eight waves.
    const int64_t waves = (static_cast<int64_t>(T) + 15) / 16;
    const bool bf = dtype == SCMOE_BF16;
    const int nw = waves > 4 * num_cus() ? 8 : waves > 2 * num_cus() ? 4 : waves > num_cus() ? 2 : 1;
#define SCMOE_GATE_MFMA(NW, EG)                                                                                    \
  return bf ? launch_gate_mfma<true, NW, EG>(x, ldx, Wg, bias, T, d, E, k, normalize, idx, gw, probs, stream)      \
            : launch_gate_mfma<false, NW, EG>(x, ldx, Wg, bias, T, d, E, k, normalize, idx, gw, probs, stream)
#define SCMOE_GATE_MFMA_NW(EG)                                                                                     \
  switch (nw) {                                                                                                    \
    case 8: SCMOE_GATE_MFMA(8, EG);                                                                                \
    case 4: SCMOE_GATE_MFMA(4, EG);                                                                                \
    case 2: SCMOE_GATE_MFMA(2, EG);                                                                                \
    default: SCMOE_GATE_MFMA(1, EG);                                                                               \
  }
    if (E <= 16) { SCMOE_GATE_MFMA_NW(1) }
    else if (E <= 32) { SCMOE_GATE_MFMA_NW(2) }
    else { SCMOE_GATE_MFMA_NW(4) }
#undef SCMOE_GATE_MFMA_NW
#undef SCMOE_GATE_MFMA
  }
  if (static_cast<int64_t>(T) * epad <= GATE_SMALL_LANES) {
    const int tpw = 256 / epad, eb = elem_bytes(dtype);
    // features per chunk: W chunk <= 32 KiB, x chunk <= 28 KiB (60 KiB of dynamic LDS beside
    // the 4 KiB of static arrays), a multiple of 8, no more than d
    int kch = 8192 / E - 4;
    const int kx = (28672 / tpw - 16) / 4;         // x is staged as fp32
    if (kx < kch) kch = kx;
    if (d < kch) kch = d;
    if (kch > GATE_SMALL_WREGS * tpw) kch = GATE_SMALL_WREGS * tpw;                       // what a thread can hold of W_g
    if (kch > (GATE_SMALL_XREGS * 256 / tpw) * (16 / eb)) kch = (GATE_SMALL_XREGS * 256 / tpw) * (16 / eb);   // and of x
    kch &= (kch >= 64) ? ~63 : ~7;                  // whole rounds of the chain loop where possible
    if (kch < 8) kch = 8;
    const size_t lds = static_cast<size_t>(kch + 4) * E * 4 + static_cast<size_t>(tpw) * (kch * 4 + 16);
    dim3 grid((T + tpw - 1) / tpw), block(256);
    const unsigned char* xb = static_cast<const unsigned char*>(x);
    if (dtype == SCMOE_BF16)
      hipLaunchKernelGGL((gate_small_kernel<true>), grid, block, lds, stream, xb, ldx, Wg, bias, T, d, E, epad, kch,
                         k, normalize, idx, gw, probs);
    else
      hipLaunchKernelGGL((gate_small_kernel<false>), grid, block, lds, stream, xb, ldx, Wg, bias, T, d, E, epad, kch,
                         k, normalize, idx, gw, probs);
    return launch_status();
  }
  // Eight waves per workgroup, each with an eighth of the experts (measured against four waves
  // with twice the experts each, bf16: E = 16, T = 32768: 107 -> 89 us; E = 16, T = 16384:
  // 51 -> 35 us; E = 8, T = 8192: 12.7 -> 8.8 us).
  // Two tokens per lane once that still leaves every CU a workgroup of 128 tokens.
#define SCMOE_GATE(EPL, NW, TPL) launch_gate<EPL, NW, TPL>(dtype, x, ldx, Wg, bias, T, d, E, k, normalize, idx, gw, probs, stream)
  const bool two = static_cast<int64_t>(T) >= static_cast<int64_t>(2 * GATE_TOK) * num_cus();
  if (E <= 4) SCMOE_GATE(1, 4, 1);
  else if (E <= 8) { if (two) SCMOE_GATE(1, 8, 2); else SCMOE_GATE(1, 8, 1); }
  else if (E <= 16) { if (two) SCMOE_GATE(2, 8, 2); else SCMOE_GATE(2, 8, 1); }
  else if (E <= 32) { if (two) SCMOE_GATE(4, 8, 2); else SCMOE_GATE(4, 8, 1); }
  else SCMOE_GATE(8, 8, 1);                        // two tokens per lane would need more than 64 KiB of LDS
#undef SCMOE_GATE
  return launch_status();
}

}  // namespace scmoe

extern "C" int scmoe_gate_top1(const void* x, int64_t ldx, int32_t dtype, const float* W_g,
                               const float* bias, int32_t T, int32_t d, int32_t E,
                               int32_t normalize, int32_t* expert_idx, float* gate_w,
                               float* probs, void* stream) {
  return scmoe::gate_topk(x, ldx, dtype, W_g, bias, T, d, E, 1, normalize, expert_idx, gate_w, probs,
                          static_cast<hipStream_t>(stream));
}

extern "C" int scmoe_gate_top2(const void* x, int64_t ldx, int32_t dtype, const float* W_g,
                               const float* bias, int32_t T, int32_t d, int32_t E,
                               int32_t normalize, int32_t* expert_idx, float* gate_w,
                               float* probs, void* stream) {
  return scmoe::gate_topk(x, ldx, dtype, W_g, bias, T, d, E, 2, normalize, expert_idx, gate_w, probs,
                          static_cast<hipStream_t>(stream));
}

extern "C" int scmoe_gate_topk(const void* x, int64_t ldx, int32_t dtype, const float* W_g,
                               const float* bias, int32_t T, int32_t d, int32_t E, int32_t k,
                               int32_t normalize, int32_t* expert_idx, float* gate_w,
                               float* probs, void* stream) {
  return scmoe::gate_topk(x, ldx, dtype, W_g, bias, T, d, E, k, normalize, expert_idx, gate_w, probs,
                          static_cast<hipStream_t>(stream));
}
