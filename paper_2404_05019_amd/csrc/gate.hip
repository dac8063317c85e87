// Gate routing (ScMoE paper Eq. (2)-(4)): logits, top-k selection, gate weights.
//
// The logits decide an integer (the arg max), so their arithmetic is fixed by the ABI:
// fp32, one fused multiply-add per input feature in ascending feature order, then one
// rounded add of the bias.  The kernel keeps that chain intact per (token, expert) and
// finds its parallelism elsewhere: a workgroup owns 64 tokens, lane = token, and each of
// its four (or, to fill the chip at smaller T, eight) waves owns a contiguous group of EPL
// experts, so every lane runs EPL independent FMA chains.  x is staged through LDS in [64 tokens x 256 bytes] tiles (coalesced HBM
// reads although each lane walks its own row), and so is the matching slab of W_g, which all
// lanes of a wave then read at one address (an LDS broadcast); the next tile of both is
// prefetched into registers while the current one is consumed.  Tried without gain: W_g
// through the scalar cache into SGPRs (3x slower: one scalar load per feature and wave) and
// one W read per 16 features with a DPP row broadcast inside the FMA (same time: LDS traffic
// is not what bounds the kernel).
#include "common.hpp"

namespace scmoe {

constexpr int GATE_TOK = 64;            // tokens per workgroup (one per lane)
constexpr int GATE_ROW_BYTES = 256;     // bytes of one token row staged per tile
constexpr int GATE_ROW_STRIDE = 272;    // LDS row stride: +16 B keeps the row reads conflict-free

// NW waves per workgroup, each owning EPL experts.
template <int EPL, int NW, bool BF16>
__global__ __launch_bounds__(64 * NW) void gate_kernel(
    const unsigned char* __restrict__ x, int64_t ldx, const float* __restrict__ Wg,
    const float* __restrict__ bias, int T, int d, int E, int k, int normalize,
    int32_t* __restrict__ expert_idx, float* __restrict__ gate_w, float* __restrict__ probs) {
  constexpr int EB = BF16 ? 2 : 4;                 // element bytes
  constexpr int KC = GATE_ROW_BYTES / EB;          // features per tile
  constexpr int GATE_THREADS = 64 * NW;
  constexpr int GATE_XV = GATE_TOK * 16 / GATE_THREADS;   // 16-byte pieces of x per thread and tile
  constexpr int EPAD = NW * EPL;                   // expert columns held in LDS (zero padded)
  constexpr int LGS = EPAD + 1;                    // row stride of the logit exchange buffer
  __shared__ __attribute__((aligned(16))) unsigned char xs[GATE_TOK * GATE_ROW_STRIDE];
  constexpr int WS_ELEMS = (KC * EPAD > GATE_TOK * LGS) ? KC * EPAD : GATE_TOK * LGS;
  __shared__ __attribute__((aligned(16))) float ws[WS_ELEMS];    // reused for the logits at the end
  __shared__ float row_max[GATE_TOK];
  __shared__ float row_sum[GATE_TOK];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int e0 = wave * EPL;
  const int t0 = blockIdx.x * GATE_TOK;

  float acc[EPL];
#pragma unroll
  for (int j = 0; j < EPL; ++j) acc[j] = 0.0f;

  // this thread's pieces of the x tile: piece c = tid + u*256 -> row c/16, 16-byte column c%16
  const unsigned char* src[GATE_XV];
#pragma unroll
  for (int u = 0; u < GATE_XV; ++u) {
    const int c = tid + u * GATE_THREADS;
    int t = t0 + (c >> 4);
    if (t >= T) t = T - 1;
    src[u] = x + static_cast<int64_t>(t) * ldx * EB + (c & 15) * 16;
  }
  uint4 pre[GATE_XV];
  auto fetch = [&](int kc0) {
    const int nvec = ((d - kc0 < KC) ? d - kc0 : KC) * EB / 16;
#pragma unroll
    for (int u = 0; u < GATE_XV; ++u)
      if (((tid + u * GATE_THREADS) & 15) < nvec)
        pre[u] = *reinterpret_cast<const uint4*>(src[u] + static_cast<int64_t>(kc0) * EB);
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
#pragma unroll
    for (int u = 0; u < GATE_XV; ++u) {
      const int c = tid + u * GATE_THREADS;
      if ((c & 15) < nvec) *reinterpret_cast<uint4*>(xs + (c >> 4) * GATE_ROW_STRIDE + (c & 15) * 16) = pre[u];
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
        const uint4 v = *reinterpret_cast<const uint4*>(myrow + c * 16);
        const uint32_t wd[4] = {v.x, v.y, v.z, v.w};
        const float* wrow = ws + (c * XPV) * EPAD + e0;
#pragma unroll
        for (int q = 0; q < XPV; ++q) {
          float xv;
          if (BF16) {
            const uint32_t word = wd[q >> 1];
            xv = __uint_as_float((q & 1) ? (word & 0xffff0000u) : (word << 16));
          } else {
            xv = __uint_as_float(wd[q]);
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
          for (int j = 0; j < EPL; ++j) acc[j] = __fmaf_rn(xv, wv[j], acc[j]);
        }
      }
    }
  }
  __syncthreads();                                 // ws is free: reuse it for the logits
  float* lg = ws;
#pragma unroll
  for (int j = 0; j < EPL; ++j) {
    if (e0 + j < E) {
      float v = acc[j];
      if (bias != nullptr) v = __fadd_rn(v, bias[e0 + j]);
      lg[lane * LGS + e0 + j] = v;
    }
  }
  __syncthreads();

  if (wave == 0) {
    const int t = t0 + lane;
    const float* l = lg + lane * LGS;
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
    row_max[lane] = m;
    row_sum[lane] = sum;
    if (t < T) {
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
          expert_idx[static_cast<int64_t>(t) * k + j] = sel[j];
          gate_w[static_cast<int64_t>(t) * k + j] = normalize ? z[j] / zsum : expf(l[sel[j]] - m) / sum;
        }
      }
    }
  }
  if (probs != nullptr) {
    __syncthreads();
    const int ntok = (T - t0 < GATE_TOK) ? T - t0 : GATE_TOK;
    for (int c = tid; c < ntok * E; c += GATE_THREADS) {
      const int tok = c / E, e = c - tok * E;
      probs[static_cast<int64_t>(t0) * E + c] = expf(lg[tok * LGS + e] - row_max[tok]) / row_sum[tok];
    }
  }
}

template <int EPL, int NW>
static void launch_gate(int dtype, const void* x, int64_t ldx, const float* Wg, const float* bias,
                        int T, int d, int E, int k, int normalize, int32_t* idx, float* gw,
                        float* probs, hipStream_t stream) {
  dim3 grid((T + GATE_TOK - 1) / GATE_TOK), block(64 * NW);
  const unsigned char* xb = static_cast<const unsigned char*>(x);
  if (dtype == SCMOE_BF16)
    hipLaunchKernelGGL((gate_kernel<EPL, NW, true>), grid, block, 0, stream, xb, ldx, Wg, bias, T, d, E, k,
                       normalize, idx, gw, probs);
  else
    hipLaunchKernelGGL((gate_kernel<EPL, NW, false>), grid, block, 0, stream, xb, ldx, Wg, bias, T, d, E, k,
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
  // Experts per wave.  Four waves per workgroup do the least redundant work (every wave reads
  // the whole x tile).  Eight waves with half the experts each pay only where that leaves a
  // single wave per SIMD with two FMA chains (measured, T = 16384: E = 8 45 -> 34 us, but
  // E = 16 42 -> 44 us; and E = 16 at T = 32768 94 -> 115 us, E = 8 at T = 8192 17 -> 18 us).
  const int64_t wgs = (T + GATE_TOK - 1) / GATE_TOK, cus = num_cus();
  const bool wide = wgs >= cus && wgs < 2 * cus;
#define SCMOE_GATE(EPL, NW) launch_gate<EPL, NW>(dtype, x, ldx, Wg, bias, T, d, E, k, normalize, idx, gw, probs, stream)
  if (E <= 4) SCMOE_GATE(1, 4);
  else if (E <= 8) { if (wide) SCMOE_GATE(1, 8); else SCMOE_GATE(2, 4); }
  else if (E <= 16) SCMOE_GATE(4, 4);
  else if (E <= 32) SCMOE_GATE(8, 4);
  else SCMOE_GATE(16, 4);
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
