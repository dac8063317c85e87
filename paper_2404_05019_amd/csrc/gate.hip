// Gate routing (ScMoE paper Eq. (2)-(4)): logits, top-k selection, gate weights.
//
// The logits decide an integer (the arg max), so their arithmetic is fixed by the ABI:
// fp32, one fused multiply-add per input feature in ascending feature order, then one
// rounded add of the bias.  The kernel keeps that chain intact per (token, expert) and
// finds its parallelism elsewhere: a workgroup owns 64 tokens, lane = token, and each of
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
  // experts per wave (four waves per workgroup)
  int epad = 1;
  while (epad < E) epad <<= 1;
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
