// Gate routing (ScMoE paper Eq. (2)-(4)): logits, top-1 / top-2 selection, gate weights.
//
// The logits decide an integer (the arg max), so their arithmetic is fixed by the ABI:
// fp32, one fused multiply-add per input feature in ascending feature order, then one
// rounded add of the bias.  The kernel keeps that chain intact per (token, expert) and
// finds its parallelism elsewhere: a workgroup owns 64 tokens, lane = token, and each wave
// of the workgroup owns a contiguous group of EPL experts, so that the gate-matrix
// operands are wave-uniform (scalar loads) and every lane runs EPL independent FMA chains.
// x is staged through LDS in [64 tokens x 256 bytes] tiles so that HBM reads are coalesced
// although each lane walks its own row.
#include "common.hpp"

namespace scmoe {

constexpr int GATE_TOK = 64;            // tokens per workgroup (one per lane)
constexpr int GATE_ROW_BYTES = 256;     // bytes of one token row staged per tile
constexpr int GATE_ROW_STRIDE = 272;    // LDS row stride: +16 B keeps 16-lane reads conflict-free
constexpr int GATE_LG_STRIDE = SCMOE_MAX_EXPERTS + 1;

template <int EPL, bool BF16>
__global__ __launch_bounds__(256) void gate_kernel(
    const unsigned char* __restrict__ x, int64_t ldx, const float* __restrict__ Wg,
    const float* __restrict__ bias, int T, int d, int E, int k, int normalize,
    int32_t* __restrict__ expert_idx, float* __restrict__ gate_w, float* __restrict__ probs) {
  constexpr int EB = BF16 ? 2 : 4;                 // element bytes
  constexpr int KC = GATE_ROW_BYTES / EB;          // features per tile
  __shared__ __attribute__((aligned(16))) unsigned char xs[GATE_TOK * GATE_ROW_STRIDE];
  __shared__ float lg[GATE_TOK * GATE_LG_STRIDE];
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
  // column of W_g each chain reads; chains past E read the last column and are discarded
  int ecol[EPL];
#pragma unroll
  for (int j = 0; j < EPL; ++j) ecol[j] = (e0 + j < E) ? e0 + j : E - 1;

  for (int kc0 = 0; kc0 < d; kc0 += KC) {
    const int kn = (d - kc0 < KC) ? d - kc0 : KC;  // features in this tile (multiple of 8)
    const int nvec = kn * EB / 16;                 // 16-byte chunks per row
    __syncthreads();
    for (int c = tid; c < GATE_TOK * 16; c += blockDim.x) {
      const int row = c >> 4, col = c & 15;
      if (col < nvec) {
        int t = t0 + row;
        if (t >= T) t = T - 1;
        const uint4 v = *reinterpret_cast<const uint4*>(x + (static_cast<int64_t>(t) * ldx + kc0) * EB + col * 16);
        *reinterpret_cast<uint4*>(xs + row * GATE_ROW_STRIDE + col * 16) = v;
      }
    }
    __syncthreads();
    const unsigned char* myrow = xs + lane * GATE_ROW_STRIDE;
    for (int c = 0; c < nvec; ++c) {
      const uint4 v = *reinterpret_cast<const uint4*>(myrow + c * 16);
      const uint32_t wd[4] = {v.x, v.y, v.z, v.w};
      if (BF16) {
        const float* wrow = Wg + static_cast<int64_t>(kc0 + c * 8) * E;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          const uint32_t word = wd[q >> 1];
          const float xv = __uint_as_float((q & 1) ? (word & 0xffff0000u) : (word << 16));
#pragma unroll
          for (int j = 0; j < EPL; ++j) acc[j] = __fmaf_rn(xv, wrow[q * E + ecol[j]], acc[j]);
        }
      } else {
        const float* wrow = Wg + static_cast<int64_t>(kc0 + c * 4) * E;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const float xv = __uint_as_float(wd[q]);
#pragma unroll
          for (int j = 0; j < EPL; ++j) acc[j] = __fmaf_rn(xv, wrow[q * E + ecol[j]], acc[j]);
        }
      }
    }
  }
#pragma unroll
  for (int j = 0; j < EPL; ++j) {
    if (e0 + j < E) {
      float v = acc[j];
      if (bias != nullptr) v = __fadd_rn(v, bias[e0 + j]);
      lg[lane * GATE_LG_STRIDE + e0 + j] = v;
    }
  }
  __syncthreads();

  if (wave == 0) {
    const int t = t0 + lane;
    const float* l = lg + lane * GATE_LG_STRIDE;
    int sel0 = 0, sel1 = -1;
    for (int e = 1; e < E; ++e) {
      const float v = l[e], b = l[sel0];
      if (v > b || (b != b && v == v)) sel0 = e;
    }
    if (k == 2) {
      for (int e = 0; e < E; ++e) {
        if (e == sel0) continue;
        if (sel1 < 0) { sel1 = e; continue; }
        const float v = l[e], b = l[sel1];
        if (v > b || (b != b && v == v)) sel1 = e;
      }
    }
    float m = -INFINITY;
    for (int e = 0; e < E; ++e)
      if (l[e] > m) m = l[e];
    float sum = 0.0f;
    for (int e = 0; e < E; ++e) sum += expf(l[e] - m);
    row_max[lane] = m;
    row_sum[lane] = sum;
    if (t < T) {
      if (k == 1) {
        expert_idx[t] = sel0;
        gate_w[t] = normalize ? 1.0f : expf(l[sel0] - m) / sum;
      } else {
        expert_idx[2 * t] = sel0;
        expert_idx[2 * t + 1] = sel1;
        if (normalize) {
          const float z1 = expf(l[sel1] - l[sel0]);
          gate_w[2 * t] = 1.0f / (1.0f + z1);
          gate_w[2 * t + 1] = z1 / (1.0f + z1);
        } else {
          gate_w[2 * t] = expf(l[sel0] - m) / sum;
          gate_w[2 * t + 1] = expf(l[sel1] - m) / sum;
        }
      }
    }
  }
  if (probs != nullptr) {
    __syncthreads();
    const int ntok = (T - t0 < GATE_TOK) ? T - t0 : GATE_TOK;
    for (int c = tid; c < ntok * E; c += blockDim.x) {
      const int tok = c / E, e = c - tok * E;
      probs[static_cast<int64_t>(t0) * E + c] = expf(lg[tok * GATE_LG_STRIDE + e] - row_max[tok]) / row_sum[tok];
    }
  }
}

template <int EPL>
static void launch_gate(int dtype, const void* x, int64_t ldx, const float* Wg, const float* bias,
                        int T, int d, int E, int k, int normalize, int32_t* idx, float* gw,
                        float* probs, hipStream_t stream) {
  const int nwaves = (E + EPL - 1) / EPL;
  dim3 grid((T + GATE_TOK - 1) / GATE_TOK), block(64 * nwaves);
  const unsigned char* xb = static_cast<const unsigned char*>(x);
  if (dtype == SCMOE_BF16)
    hipLaunchKernelGGL((gate_kernel<EPL, true>), grid, block, 0, stream, xb, ldx, Wg, bias, T, d, E, k,
                       normalize, idx, gw, probs);
  else
    hipLaunchKernelGGL((gate_kernel<EPL, false>), grid, block, 0, stream, xb, ldx, Wg, bias, T, d, E, k,
                       normalize, idx, gw, probs);
}

int gate_topk(const void* x, int64_t ldx, int dtype, const float* Wg, const float* bias, int T,
              int d, int E, int k, int normalize, int32_t* idx, float* gw, float* probs,
              hipStream_t stream) {
  if (!dtype_ok(dtype)) return SCMOE_ERR_DTYPE;
  if (T < 0 || d <= 0 || (d % 8) != 0 || E < 1 || E > SCMOE_MAX_EXPERTS) return SCMOE_ERR_SHAPE;
  if (k != 1 && k != 2) return SCMOE_ERR_ARG;
  if (k == 2 && E < 2) return SCMOE_ERR_SHAPE;
  if (normalize != 0 && normalize != 1) return SCMOE_ERR_ARG;
  if (T == 0) return SCMOE_OK;
  if (!x || !Wg || !idx || !gw) return SCMOE_ERR_NULL;
  if (!view_ok(x, ldx, d, dtype)) return SCMOE_ERR_SHAPE;
  // experts per wave: at most four waves per workgroup
  if (E <= 4) launch_gate<1>(dtype, x, ldx, Wg, bias, T, d, E, k, normalize, idx, gw, probs, stream);
  else if (E <= 8) launch_gate<2>(dtype, x, ldx, Wg, bias, T, d, E, k, normalize, idx, gw, probs, stream);
  else if (E <= 16) launch_gate<4>(dtype, x, ldx, Wg, bias, T, d, E, k, normalize, idx, gw, probs, stream);
  else if (E <= 32) launch_gate<8>(dtype, x, ldx, Wg, bias, T, d, E, k, normalize, idx, gw, probs, stream);
  else launch_gate<16>(dtype, x, ldx, Wg, bias, T, d, E, k, normalize, idx, gw, probs, stream);
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
