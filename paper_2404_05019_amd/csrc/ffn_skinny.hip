// Grouped GEMM for a handful of rows (a decode step: at most 32 packed rows in the whole
// call, so no expert has more).  With so few rows the weights are read once and barely
// reused: the kernel is bound by streaming W from HBM, not by the matrix cores, and the
// 256-row tiles of the main grouped GEMM would spend a full tile of MFMA work per weight
// panel.  Here a workgroup owns 64 output columns of one expert and walks all of K:
//   * the expert's rows of A (at most 32) are staged through LDS in chunks of 512 k;
//   * each of the four waves owns 16 columns and loads its W rows straight from global
//     memory into MFMA operand registers, 32 contiguous bytes per lane, so the four lanes of
//     a row cover a whole 128-byte line per step of 64 k (the k order inside a step is
//     permuted the same way for both operands, which a dot product does not notice);
//   * v_mfma_f32_16x16x32_bf16 with the weight fragment as first operand: a lane ends with
//     4 consecutive output columns of one row.
// Same operand conventions and fused epilogues (bias, GELU, output decode) as the main kernel
// (ScMoE paper Sec. 2.2 for encode/decode, Eq. (1) for the expert); the paper's
// memory-limited inference setting (Sec. 5.3) is where such calls come from.
#include "mfma_common.hpp"

namespace scmoe {

constexpr int SK_ROWS = 32;              // most rows of one segment (and of the whole call)
constexpr int SK_BN = 64;                // output columns per workgroup (16 per wave)
constexpr int SK_KC = 512;               // k per LDS chunk of the activations
constexpr int SK_ROW_BYTES = SK_KC * 2 + 16;   // LDS row stride: +16 B spreads the 16 rows of a fragment read over the banks
constexpr int SK_THREADS = 256;

constexpr int SK_STEPS = SK_KC / 64;     // 64-k steps per chunk

// PARTIAL: the workgroup covers k-chunks [z * cpp, (z + 1) * cpp) only and leaves raw fp32
// sums in partial[z][packed row][N]; gemm_skinny_finish adds the parts up in order.
template <bool ACT, bool PARTIAL>
__global__ __launch_bounds__(SK_THREADS) void gemm_skinny_kernel(const GemmArgs p, int cpp, float* __restrict__ partial) {
  __shared__ __attribute__((aligned(16))) unsigned char xs[SK_ROWS * SK_ROW_BYTES];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int e = blockIdx.y;
  const int n0 = blockIdx.x * SK_BN;
  const int s = p.offsets[e];
  int c = p.offsets[e + 1] - s;
  if (s < 0 || s >= SK_ROWS) return;     // the host admits the call only if all packed rows are below SK_ROWS
  if (c > SK_ROWS - s) c = SK_ROWS - s;
  if (c <= 0) return;
  const int nsub = (c + 15) >> 4;        // 16-row MFMA subtiles in use (1 or 2)
  const int l16 = lane & 15, lq = lane >> 4;
  const int kbeg = PARTIAL ? blockIdx.z * cpp * SK_KC : 0;
  int kend = PARTIAL ? kbeg + cpp * SK_KC : p.Kd;
  if (kend > p.Kd) kend = p.Kd;

  // this lane's weight row (an output column) and its 32 bytes inside a 64-k step
  int n = n0 + wave * 16 + l16;
  if (n > p.N - 1) n = p.N - 1;          // columns past N re-read the last row; never stored
  const unsigned char* wrow = p.W + (static_cast<int64_t>(e) * p.N + n) * p.ldw * 2 + lq * 32;
  const int nc = n0 + wave * 16 + 4 * lq;          // the 4 consecutive columns this lane ends with

  f32x4_t acc[2];
  {
    f32x4_t b = {0.0f, 0.0f, 0.0f, 0.0f};
    if (!PARTIAL && p.bias != nullptr && nc < p.N)
      b = *reinterpret_cast<const f32x4_t*>(p.bias + static_cast<int64_t>(e) * p.N + nc);
    acc[0] = b;
    acc[1] = b;
  }

  // The weights of a whole chunk (8 steps x 32 bytes per lane) are requested at once, one
  // chunk ahead of the arithmetic: 16 KiB per wave in flight while the previous chunk is
  // computed and the activations are staged.
  bf16x8_t wa[2 * SK_STEPS], wb[2 * SK_STEPS];
  auto load_w = [&](bf16x8_t (&w)[2 * SK_STEPS], int kc0) {
    const int kn = (kend - kc0 < SK_KC) ? kend - kc0 : SK_KC;    // multiple of 64
    const unsigned char* wk = wrow + static_cast<int64_t>(kc0) * 2;
#pragma unroll
    for (int st = 0; st < SK_STEPS; ++st) {
      if (st * 64 < kn) {
        w[2 * st] = *reinterpret_cast<const bf16x8_t*>(wk + st * 128);
        w[2 * st + 1] = *reinterpret_cast<const bf16x8_t*>(wk + st * 128 + 16);
      }
    }
  };
  auto chunk = [&](const bf16x8_t (&w)[2 * SK_STEPS], int kc0) {
    const int kn = (kend - kc0 < SK_KC) ? kend - kc0 : SK_KC;
    const int vpr = kn / 8;                                       // 16-byte pieces per row
    __syncthreads();                                              // the previous chunk has been consumed
    for (int i = tid; i < c * vpr; i += SK_THREADS) {
      const int r = i / vpr, v = i - r * vpr;
      const int64_t src = p.gather ? p.gather[s + r] : s + r;
      *reinterpret_cast<uint4*>(xs + r * SK_ROW_BYTES + v * 16) =
          *reinterpret_cast<const uint4*>(p.A + (src * p.lda + kc0) * 2 + v * 16);
    }
    __syncthreads();
    const unsigned char* xl = xs + l16 * SK_ROW_BYTES + lq * 32;
#pragma unroll
    for (int st = 0; st < SK_STEPS; ++st) {
      if (st * 64 < kn) {
        const bf16x8_t a0 = *reinterpret_cast<const bf16x8_t*>(xl + st * 128);
        const bf16x8_t a1 = *reinterpret_cast<const bf16x8_t*>(xl + st * 128 + 16);
        acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[2 * st], a0, acc[0], 0, 0, 0);
        acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[2 * st + 1], a1, acc[0], 0, 0, 0);
        if (nsub > 1) {                                           // workgroup-uniform
          const bf16x8_t b0 = *reinterpret_cast<const bf16x8_t*>(xl + 16 * SK_ROW_BYTES + st * 128);
          const bf16x8_t b1 = *reinterpret_cast<const bf16x8_t*>(xl + 16 * SK_ROW_BYTES + st * 128 + 16);
          acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[2 * st], b0, acc[1], 0, 0, 0);
          acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[2 * st + 1], b1, acc[1], 0, 0, 0);
        }
      }
    }
  };
  if (kbeg < kend) load_w(wa, kbeg);
  for (int kc0 = kbeg; kc0 < kend; kc0 += 2 * SK_KC) {
    if (kc0 + SK_KC < kend) load_w(wb, kc0 + SK_KC);
    chunk(wa, kc0);
    if (kc0 + SK_KC < kend) {
      if (kc0 + 2 * SK_KC < kend) load_w(wa, kc0 + 2 * SK_KC);
      chunk(wb, kc0 + SK_KC);
    }
  }

  // acc[sub][v] = output row 16 sub + lane % 16, column nc + v
  if (nc >= p.N) return;
#pragma unroll
  for (int sub = 0; sub < 2; ++sub) {
    const int r = sub * 16 + l16;
    if (r >= c) continue;
    if (PARTIAL) {
      *reinterpret_cast<f32x4_t*>(partial + (static_cast<int64_t>(blockIdx.z) * SK_ROWS + s + r) * p.N + nc) = acc[sub];
      continue;
    }
    float v[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      v[q] = acc[sub][q];
      if (ACT) v[q] = (p.gelu_mode == SCMOE_GELU_TANH) ? gelu_tanh_fast(v[q]) : gelu_erf_fast(v[q]);
    }
    int64_t orow = s + r;
    uint2 o;
    if (p.scatter) {
      // output decode: packed row s + r belongs to token orow; scale by its gate weight and
      // add the row already there
      orow = p.scatter[s + r];
      const float g = p.row_scale[orow];
      o.x = cvt_pk_bf16(v[0] * g, v[1] * g);
      o.y = cvt_pk_bf16(v[2] * g, v[3] * g);
      const uint2 a = *reinterpret_cast<const uint2*>(p.addend + (orow * p.ldadd + nc) * 2);
      o.x = add_bf16x2(o.x, a.x);
      o.y = add_bf16x2(o.y, a.y);
    } else {
      o.x = cvt_pk_bf16(v[0], v[1]);
      o.y = cvt_pk_bf16(v[2], v[3]);
    }
    *reinterpret_cast<uint2*>(p.C + (orow * p.ldc + nc) * 2) = o;
  }
}

// Sum of the k-parts in part order, then the epilogue of the unsplit kernel.  One thread per
// 4 consecutive columns of one packed row; grid.y = SK_ROWS.
template <bool ACT>
__global__ __launch_bounds__(256) void gemm_skinny_finish(const GemmArgs p, int parts, const float* __restrict__ partial) {
  const int row = blockIdx.y;
  int total = p.offsets[p.E];
  if (total > SK_ROWS) total = SK_ROWS;
  if (row >= total) return;
  const int nc = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (nc >= p.N) return;
  int e = 0;
  while (e < p.E - 1 && p.offsets[e + 1] <= row) ++e;
  f32x4_t sum = {0.0f, 0.0f, 0.0f, 0.0f};
  if (p.bias != nullptr) sum = *reinterpret_cast<const f32x4_t*>(p.bias + static_cast<int64_t>(e) * p.N + nc);
  for (int z = 0; z < parts; ++z)
    sum += *reinterpret_cast<const f32x4_t*>(partial + (static_cast<int64_t>(z) * SK_ROWS + row) * p.N + nc);
  float v[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    v[q] = sum[q];
    if (ACT) v[q] = (p.gelu_mode == SCMOE_GELU_TANH) ? gelu_tanh_fast(v[q]) : gelu_erf_fast(v[q]);
  }
  int64_t orow = row;
  uint2 o;
  if (p.scatter) {
    orow = p.scatter[row];
    const float g = p.row_scale[orow];
    o.x = cvt_pk_bf16(v[0] * g, v[1] * g);
    o.y = cvt_pk_bf16(v[2] * g, v[3] * g);
    const uint2 a = *reinterpret_cast<const uint2*>(p.addend + (orow * p.ldadd + nc) * 2);
    o.x = add_bf16x2(o.x, a.x);
    o.y = add_bf16x2(o.y, a.y);
  } else {
    o.x = cvt_pk_bf16(v[0], v[1]);
    o.y = cvt_pk_bf16(v[2], v[3]);
  }
  *reinterpret_cast<uint2*>(p.C + (orow * p.ldc + nc) * 2) = o;
}

bool gemm_skinny_fits(int max_rows) { return max_rows <= SK_ROWS; }

// One grouped GEMM of at most SK_ROWS rows in total (max_rows: the caller's bound on them).
// Kd must be a multiple of 64 and the dense extra segment of GemmArgs is not supported
// (xrows == 0).  With scratch the k range is cut into parts, one workgroup each, so that a
// call with few column blocks (the shared expert: one segment) still streams its weights
// with the whole chip; the parts meet in `scratch` ([parts][SK_ROWS][N] fp32).
int launch_gemm_skinny(const GemmArgs& a, bool act, int max_rows, void* scratch, size_t scratch_bytes,
                       hipStream_t stream) {
  if (a.xrows != 0 || (a.Kd % 64) != 0 || a.E < 1 || a.N < 1 || max_rows > SK_ROWS) return SCMOE_ERR_ARG;
  const int cols = (a.N + SK_BN - 1) / SK_BN;
  const int nch = (a.Kd + SK_KC - 1) / SK_KC;
  const int segs = a.E < max_rows ? a.E : max_rows;           // segments that can hold a row
  int parts = 512 / (cols * (segs > 0 ? segs : 1));           // aim: about two workgroups per CU
  if (parts > nch) parts = nch;
  if (parts < 1) parts = 1;
  int cpp = (nch + parts - 1) / parts;
  parts = (nch + cpp - 1) / cpp;                               // every part holds at least one chunk
  if (scratch == nullptr || static_cast<size_t>(parts) * SK_ROWS * a.N * sizeof(float) > scratch_bytes) parts = 1;
  dim3 block(SK_THREADS);
  if (parts == 1) {
    dim3 grid(cols, a.E);
    if (act) hipLaunchKernelGGL((gemm_skinny_kernel<true, false>), grid, block, 0, stream, a, nch, nullptr);
    else hipLaunchKernelGGL((gemm_skinny_kernel<false, false>), grid, block, 0, stream, a, nch, nullptr);
    return launch_status();
  }
  float* partial = static_cast<float*>(scratch);
  hipLaunchKernelGGL((gemm_skinny_kernel<false, true>), dim3(cols, a.E, parts), block, 0, stream, a, cpp, partial);
  int st = launch_status();
  if (st != SCMOE_OK) return st;
  dim3 fgrid((a.N / 4 + 255) / 256, SK_ROWS);
  if (act) hipLaunchKernelGGL((gemm_skinny_finish<true>), fgrid, dim3(256), 0, stream, a, parts, partial);
  else hipLaunchKernelGGL((gemm_skinny_finish<false>), fgrid, dim3(256), 0, stream, a, parts, partial);
  return launch_status();
}

}  // namespace scmoe
