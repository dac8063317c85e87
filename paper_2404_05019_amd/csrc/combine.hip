// Output decode (ScMoE paper Sec. 2.2) fused with the merge of Eq. (6)/(7), and the
// coefficient gates of Eq. (14)-(17).  On one GPU this replaces "All-to-All combine +
// decode": every output row is gathered from the packed expert outputs, scaled by its gate
// weight and added to the shared expert's row.  HBM-bound: each thread moves 16-byte pieces.
#include "common.hpp"

namespace scmoe {

template <bool BF16>
__device__ __forceinline__ void load8(const unsigned char* p, float* v) {
  // 16 bytes: 8 bf16 or 4 fp32 (then only v[0..3] are used)
  const uint4 q = *reinterpret_cast<const uint4*>(p);
  if (BF16) {
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = __uint_as_float(w[i] << 16);
      v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  } else {
    v[0] = __uint_as_float(q.x);
    v[1] = __uint_as_float(q.y);
    v[2] = __uint_as_float(q.z);
    v[3] = __uint_as_float(q.w);
  }
}

template <bool BF16>
__device__ __forceinline__ void store8(unsigned char* p, const float* v) {
  uint4 q;
  if (BF16) {
    q.x = pack_bf16x2(v[0], v[1]);
    q.y = pack_bf16x2(v[2], v[3]);
    q.z = pack_bf16x2(v[4], v[5]);
    q.w = pack_bf16x2(v[6], v[7]);
  } else {
    q.x = __float_as_uint(v[0]);
    q.y = __float_as_uint(v[1]);
    q.z = __float_as_uint(v[2]);
    q.w = __float_as_uint(v[3]);
  }
  *reinterpret_cast<uint4*>(p) = q;
}

// One thread per 16-byte piece of y.  vpr = pieces per row.
template <bool BF16, int K>
__global__ __launch_bounds__(256) void combine_kernel(
    const unsigned char* __restrict__ y_perm, int64_t ldyp, const int32_t* __restrict__ dst_row,
    const float* __restrict__ gate_w, int T, int vpr, const unsigned char* base, int64_t ldbase,
    const unsigned char* residual, int64_t ldres, const float* __restrict__ coef,
    unsigned char* y, int64_t ldy) {
  constexpr int NV = BF16 ? 8 : 4;
  const int64_t total = static_cast<int64_t>(T) * vpr;
  for (int64_t c = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; c < total;
       c += static_cast<int64_t>(gridDim.x) * blockDim.x) {
    const int t = static_cast<int>(c / vpr);
    const int col = static_cast<int>(c - static_cast<int64_t>(t) * vpr) * 16;  // byte offset in the row
    float acc[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) acc[i] = 0.0f;
#pragma unroll
    for (int j = 0; j < K; ++j) {
      const int r = dst_row[static_cast<int64_t>(t) * K + j];
      if (r >= 0) {
        const float w = gate_w[static_cast<int64_t>(t) * K + j];
        float v[8];
        load8<BF16>(y_perm + r * ldyp + col, v);
#pragma unroll
        for (int i = 0; i < NV; ++i) acc[i] = fmaf(w, v[i], acc[i]);
      }
    }
    float c0 = 1.0f, c1 = 1.0f;
    if (coef != nullptr) {
      c0 = coef[2 * static_cast<int64_t>(t)];
      c1 = coef[2 * static_cast<int64_t>(t) + 1];
#pragma unroll
      for (int i = 0; i < NV; ++i) acc[i] *= c1;
    }
    if (base != nullptr) {
      float v[8];
      load8<BF16>(base + t * ldbase + col, v);
#pragma unroll
      for (int i = 0; i < NV; ++i) acc[i] = fmaf(c0, v[i], acc[i]);
    }
    if (residual != nullptr) {
      float v[8];
      load8<BF16>(residual + t * ldres + col, v);
#pragma unroll
      for (int i = 0; i < NV; ++i) acc[i] += v[i];
    }
    store8<BF16>(y + t * ldy + col, acc);
  }
}

int combine(const void* y_perm, int64_t ldyp, int dtype, const int32_t* dst_row, const float* gate_w,
            int T, int d, int k, const void* base, int64_t ldbase, const void* residual,
            int64_t ldres, const float* coef, void* y, int64_t ldy, hipStream_t stream) {
  if (!dtype_ok(dtype)) return SCMOE_ERR_DTYPE;
  if (T < 0 || d <= 0 || (d % 8) != 0) return SCMOE_ERR_SHAPE;
  if (k < 1 || k > SCMOE_MAX_TOPK) return SCMOE_ERR_ARG;
  if (T == 0) return SCMOE_OK;
  if (!dst_row || !gate_w || !y) return SCMOE_ERR_NULL;
  if (!view_ok(y, ldy, d, dtype)) return SCMOE_ERR_SHAPE;
  // y_perm may be NULL only when nothing can be kept; the kernel reads it for dst_row >= 0
  if (!y_perm) return SCMOE_ERR_NULL;
  if (!view_ok(y_perm, ldyp, d, dtype)) return SCMOE_ERR_SHAPE;
  if (base && !view_ok(base, ldbase, d, dtype)) return SCMOE_ERR_SHAPE;
  if (residual && !view_ok(residual, ldres, d, dtype)) return SCMOE_ERR_SHAPE;
  const int eb = elem_bytes(dtype);
  const int vpr = d * eb / 16;
  const int64_t total = static_cast<int64_t>(T) * vpr;
  int64_t blocks = (total + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  dim3 grid(static_cast<unsigned>(blocks)), block(256);
  const unsigned char* yp = static_cast<const unsigned char*>(y_perm);
  const unsigned char* bs = static_cast<const unsigned char*>(base);
  const unsigned char* rs = static_cast<const unsigned char*>(residual);
  unsigned char* yo = static_cast<unsigned char*>(y);
#define SCMOE_COMBINE(BF, KK)                                                                       \
  hipLaunchKernelGGL((combine_kernel<BF, KK>), grid, block, 0, stream, yp, ldyp * eb, dst_row, gate_w, T, \
                     vpr, bs, ldbase * eb, rs, ldres * eb, coef, yo, ldy * eb)
  static_assert(SCMOE_MAX_TOPK == 4, "one instantiation per k below");
  if (dtype == SCMOE_BF16) {
    switch (k) {
      case 1: SCMOE_COMBINE(true, 1); break;
      case 2: SCMOE_COMBINE(true, 2); break;
      case 3: SCMOE_COMBINE(true, 3); break;
      default: SCMOE_COMBINE(true, 4); break;
    }
  } else {
    switch (k) {
      case 1: SCMOE_COMBINE(false, 1); break;
      case 2: SCMOE_COMBINE(false, 2); break;
      case 3: SCMOE_COMBINE(false, 3); break;
      default: SCMOE_COMBINE(false, 4); break;
    }
  }
#undef SCMOE_COMBINE
  return launch_status();
}

// Coefficient gate: one wave per token at a time, fp32 dot products reduced across the wave.
// LDS_W: the gate's one or two weight rows are staged in LDS once per workgroup, which then
// walks over many tokens (read from global memory per token they cost two to four times
// the bytes of the token's row in cache traffic); otherwise they are read in place (rows too
// long for the LDS).
template <bool BF16, bool LDS_W>
__global__ __launch_bounds__(256) void coef_gate_kernel(const unsigned char* __restrict__ x, int64_t ldx_bytes,
                                                        const float* __restrict__ Wcg, int mode, int T,
                                                        int d, float* __restrict__ coef) {
  constexpr int NV = BF16 ? 8 : 4;
  extern __shared__ __attribute__((aligned(16))) float cg_w[];
  if (LDS_W) {
    const int n = (mode == SCMOE_CG_2 ? 2 : 1) * d;
    for (int i = threadIdx.x; i < n; i += blockDim.x) cg_w[i] = Wcg[i];
    __syncthreads();
  }
  auto w = [&](int i) { return LDS_W ? cg_w[i] : Wcg[i]; };
  const int lane = threadIdx.x & 63;
  const int waves = blockDim.x >> 6;
  for (int t = blockIdx.x * waves + (threadIdx.x >> 6); t < T; t += gridDim.x * waves) {
    const unsigned char* row = x + static_cast<int64_t>(t) * ldx_bytes;
    float a = 0.0f, b = 0.0f;
    for (int i0 = lane * NV; i0 < d; i0 += 64 * NV) {
      float v[8];
      load8<BF16>(row + static_cast<int64_t>(i0) * (BF16 ? 2 : 4), v);
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        a = fmaf(v[i], w(i0 + i), a);
        if (mode == SCMOE_CG_2) b = fmaf(v[i], w(d + i0 + i), b);
      }
    }
    for (int off = 32; off > 0; off >>= 1) {
      a += __shfl_xor(a, off, 64);
      b += __shfl_xor(b, off, 64);
    }
    if (lane == 0) {
      float c0, c1;
      if (mode == SCMOE_CG_1) {
        c0 = 1.0f / (1.0f + expf(-a));
        c1 = 1.0f;
      } else {
        const float m = fmaxf(a, b);
        const float ea = expf(a - m), eb = expf(b - m);
        c0 = ea / (ea + eb);
        c1 = eb / (ea + eb);
      }
      coef[2 * static_cast<int64_t>(t)] = c0;
      coef[2 * static_cast<int64_t>(t) + 1] = c1;
    }
  }
}

int coef_gate(const void* x, int64_t ldx, int dtype, const float* Wcg, int mode, int T, int d,
              float* coef, hipStream_t stream) {
  if (!dtype_ok(dtype)) return SCMOE_ERR_DTYPE;
  if (mode != SCMOE_CG_1 && mode != SCMOE_CG_2) return SCMOE_ERR_ARG;
  if (T < 0 || d <= 0 || (d % 8) != 0) return SCMOE_ERR_SHAPE;
  if (T == 0) return SCMOE_OK;
  if (!x || !Wcg || !coef) return SCMOE_ERR_NULL;
  if (!view_ok(x, ldx, d, dtype)) return SCMOE_ERR_SHAPE;
  const unsigned char* xb = static_cast<const unsigned char*>(x);
  const size_t lds = static_cast<size_t>(mode == SCMOE_CG_2 ? 2 : 1) * d * sizeof(float);
  const int wgs = (T + 3) / 4;
  if (lds <= 48 * 1024) {
    // weight rows in LDS: a few workgroups per CU, each over many tokens
    const int cap = 8 * num_cus();
    dim3 grid(wgs < cap ? wgs : cap), block(256);
    if (dtype == SCMOE_BF16)
      hipLaunchKernelGGL((coef_gate_kernel<true, true>), grid, block, lds, stream, xb, ldx * 2, Wcg, mode, T, d, coef);
    else
      hipLaunchKernelGGL((coef_gate_kernel<false, true>), grid, block, lds, stream, xb, ldx * 4, Wcg, mode, T, d, coef);
  } else {
    dim3 grid(wgs), block(256);
    if (dtype == SCMOE_BF16)
      hipLaunchKernelGGL((coef_gate_kernel<true, false>), grid, block, 0, stream, xb, ldx * 2, Wcg, mode, T, d, coef);
    else
      hipLaunchKernelGGL((coef_gate_kernel<false, false>), grid, block, 0, stream, xb, ldx * 4, Wcg, mode, T, d, coef);
  }
  return launch_status();
}

}  // namespace scmoe

extern "C" int scmoe_combine(const void* y_perm, int64_t ldyp, int32_t dtype, const int32_t* dst_row,
                             const float* gate_w, int32_t T, int32_t d, int32_t k, const void* base,
                             int64_t ldbase, const void* residual, int64_t ldres, const float* coef,
                             void* y, int64_t ldy, void* stream) {
  return scmoe::combine(y_perm, ldyp, dtype, dst_row, gate_w, T, d, k, base, ldbase, residual, ldres,
                        coef, y, ldy, static_cast<hipStream_t>(stream));
}

extern "C" int scmoe_coef_gate(const void* x, int64_t ldx, int32_t dtype, const float* W_cg,
                               int32_t cg_mode, int32_t T, int32_t d, float* coef, void* stream) {
  return scmoe::coef_gate(x, ldx, dtype, W_cg, cg_mode, T, d, coef, static_cast<hipStream_t>(stream));
}
