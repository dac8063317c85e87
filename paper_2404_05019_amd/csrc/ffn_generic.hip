// Expert computation (ScMoE paper Eq. (1); experts are two-layer MLPs, Sec. 2.1) for any
// shape and both storage types: a plain LDS-tiled grouped GEMM on the vector ALUs with fp32
// accumulation.  It is the fp32 path and the fallback for bf16 shapes the MFMA kernels do
// not cover; the bf16 hot path lives in ffn_mfma.hip.
//
//   C[r, n] = act( sum_k A[r, k] * W[e, n, k] + bias[e, n] )   for r in segment e
#include "common.hpp"

namespace scmoe {

constexpr int GT = 64;   // tile edge (rows and columns)
constexpr int GK = 64;   // depth of one LDS stage (a stage is one round trip to memory: few, deep stages)
constexpr int GQ = GT * GK / 256;   // elements of each operand a thread moves per stage

template <bool BF16>
__device__ __forceinline__ float load_elem(const unsigned char* p, int64_t i) {
  if (BF16) return bf16_to_f32(reinterpret_cast<const uint16_t*>(p)[i]);
  return reinterpret_cast<const float*>(p)[i];
}

template <bool BF16>
__device__ __forceinline__ void store_elem(unsigned char* p, int64_t i, float v) {
  if (BF16) reinterpret_cast<uint16_t*>(p)[i] = f32_to_bf16(v);
  else reinterpret_cast<float*>(p)[i] = v;
}

template <bool BF16, bool ACT>
__global__ __launch_bounds__(256) void ffn_generic_kernel(
    const unsigned char* __restrict__ A, int64_t lda, const int32_t* __restrict__ offsets, int E,
    int N, int Kd, const unsigned char* __restrict__ W, int64_t ldw, const float* __restrict__ bias,
    unsigned char* __restrict__ C, int64_t ldc, int gelu_mode) {
  __shared__ __attribute__((aligned(16))) float As[GK][GT + 4];   // (rows stay 16-byte aligned: 4 values per read)
  __shared__ __attribute__((aligned(16))) float Bs[GK][GT + 4];
  // which expert segment does this row tile belong to?
  int mt = blockIdx.x, e = 0, row0 = 0, row_end = 0;
  bool found = false;
  for (e = 0; e < E; ++e) {
    const int s = offsets[e], c = offsets[e + 1] - s;
    const int nt = (c + GT - 1) / GT;
    if (mt < nt) {
      row0 = s + mt * GT;
      row_end = s + c;
      found = true;
      break;
    }
    mt -= nt;
  }
  if (!found) return;
  const int n0 = blockIdx.y * GT;
  const unsigned char* We = W + static_cast<int64_t>(e) * N * ldw * (BF16 ? 2 : 4);
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.0f;

  // The next stage's elements are fetched into registers while the current one is consumed
  // (a tile of a small problem is a chain of Kd / GK round trips to memory otherwise).  Loads
  // are unconditional on clamped indices; what lies outside the operands becomes zero.
  float pa[GQ], pb[GQ];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int q = 0; q < GQ; ++q) {
      const int idx = tid + q * 256;
      const int r = idx / GK, kk = idx % GK;
      const int row = row0 + r, kg = k0 + kk, n = n0 + r;
      const int rowc = row < row_end ? row : row_end - 1, nc = n < N ? n : N - 1, kc = kg < Kd ? kg : Kd - 1;
      const float av = load_elem<BF16>(A, static_cast<int64_t>(rowc) * lda + kc);
      const float bv = load_elem<BF16>(We, static_cast<int64_t>(nc) * ldw + kc);
      pa[q] = (row < row_end && kg < Kd) ? av : 0.0f;
      pb[q] = (n < N && kg < Kd) ? bv : 0.0f;
    }
  };
  fetch(0);
  for (int k0 = 0; k0 < Kd; k0 += GK) {
#pragma unroll
    for (int q = 0; q < GQ; ++q) {
      const int idx = tid + q * 256;
      As[idx % GK][idx / GK] = pa[q];
      Bs[idx % GK][idx / GK] = pb[q];
    }
    __syncthreads();
    if (k0 + GK < Kd) fetch(k0 + GK);
#pragma unroll
    for (int kk = 0; kk < GK; ++kk) {
      const float4 a4 = *reinterpret_cast<const float4*>(&As[kk][ty * 4]);
      const float4 b4 = *reinterpret_cast<const float4*>(&Bs[kk][tx * 4]);
      const float a[4] = {a4.x, a4.y, a4.z, a4.w}, b[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = row0 + ty * 4 + i;
    if (row >= row_end) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      float v = acc[i][j];
      if (bias != nullptr) v += bias[static_cast<int64_t>(e) * N + n];
      if (ACT) v = gelu_f32(v, gelu_mode);
      store_elem<BF16>(C, static_cast<int64_t>(row) * ldc + n, v);
    }
  }
}

int ffn_generic(const FfnArgs& a, int dtype, hipStream_t stream) {
  const int mt = (a.max_rows + GT - 1) / GT + a.E;  // upper bound on row tiles over all segments
  const unsigned char* xb = static_cast<const unsigned char*>(a.x);
  const unsigned char* w1 = static_cast<const unsigned char*>(a.W1);
  const unsigned char* w2 = static_cast<const unsigned char*>(a.W2);
  unsigned char* hb = static_cast<unsigned char*>(a.hidden);
  unsigned char* yb = static_cast<unsigned char*>(a.y);
  dim3 block(256);
  dim3 g1(mt, (a.F + GT - 1) / GT), g2(mt, (a.d + GT - 1) / GT);
  if (dtype == SCMOE_BF16) {
    hipLaunchKernelGGL((ffn_generic_kernel<true, true>), g1, block, 0, stream, xb, a.ldx, a.offsets, a.E, a.F,
                       a.d, w1, a.ldw1, a.b1, hb, a.ldh, a.gelu_mode);
    hipLaunchKernelGGL((ffn_generic_kernel<true, false>), g2, block, 0, stream, hb, a.ldh, a.offsets, a.E, a.d,
                       a.F, w2, a.ldw2, a.b2, yb, a.ldy, a.gelu_mode);
  } else {
    hipLaunchKernelGGL((ffn_generic_kernel<false, true>), g1, block, 0, stream, xb, a.ldx, a.offsets, a.E, a.F,
                       a.d, w1, a.ldw1, a.b1, hb, a.ldh, a.gelu_mode);
    hipLaunchKernelGGL((ffn_generic_kernel<false, false>), g2, block, 0, stream, hb, a.ldh, a.offsets, a.E, a.d,
                       a.F, w2, a.ldw2, a.b2, yb, a.ldy, a.gelu_mode);
  }
  return launch_status();
}

}  // namespace scmoe
