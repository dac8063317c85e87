// Grouped GEMM for a handful of rows per expert (decode steps: at most 32 packed rows in the
// whole call, or segments that average 16 rows or fewer).  With so few rows the weights are
// read once and barely reused: the kernel is bound by streaming W from HBM, not by the
// matrix cores, and the 128- or 256-row tiles of the main grouped GEMM would spend a full
// tile of MFMA work per weight panel.  Here a workgroup owns 64 output columns of one expert
// and walks all of K:
//   * the expert's rows of A (32 or 64 at a time) are staged through LDS in chunks of 512 or
//     256 k;
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

constexpr int SK_ROWS = 64;              // most packed rows of a call that may be cut along K (they index the partial sums)
constexpr int SK_BN = 64;                // output columns per workgroup (16 per wave)
constexpr int SK_THREADS = 256;

// NSUB 16-row MFMA subtiles per row block: 2 (a call of at most 32 rows: one block per
// segment, 512-k chunks) or 4 (segments of any length walked in blocks of 64 rows, 256-k
// chunks; meant for calls of at most 64 rows or whose segments average 16 rows or fewer).
// PARTIAL (only for calls of at most 16 NSUB rows in all): the workgroup covers k-chunks
// [z * cpp, (z + 1) * cpp) and leaves raw fp32 sums in partial[z][packed row][N], 16 NSUB
// rows per part; gemm_skinny_finish adds the parts up in order.
template <bool ACT, bool PARTIAL, int NSUB>
__global__ __launch_bounds__(SK_THREADS) void gemm_skinny_kernel(const GemmArgs p, int cpp, float* __restrict__ partial) {
  static_assert(NSUB == 2 || NSUB == 4, "row-block shapes");
  constexpr int RB = 16 * NSUB;                    // rows per block
  constexpr int KC = NSUB == 2 ? 512 : 256;        // k per LDS chunk of the activations
  constexpr int ROW_BYTES = KC * 2 + 16;           // LDS row stride: +16 B spreads the 16 rows of a fragment read over the banks
  constexpr int STEPS = KC / 64;                   // 64-k steps per chunk
  __shared__ __attribute__((aligned(16))) unsigned char xs[RB * ROW_BYTES];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int e = blockIdx.y;
  const int n0 = blockIdx.x * SK_BN;
  const int s = p.offsets[e];
  int c = p.offsets[e + 1] - s;
  if (s < 0) return;
  if (PARTIAL) {                         // the host admits such a call only if all packed rows are below RB
    if (s >= RB) return;
    if (c > RB - s) c = RB - s;
  }
  if (c <= 0) return;
  const int l16 = lane & 15, lq = lane >> 4;
  const int kbeg = PARTIAL ? blockIdx.z * cpp * KC : 0;
  int kend = PARTIAL ? kbeg + cpp * KC : p.Kd;
  if (kend > p.Kd) kend = p.Kd;

  // this lane's weight row (an output column) and its 32 bytes inside a 64-k step
  int n = n0 + wave * 16 + l16;
  if (n > p.N - 1) n = p.N - 1;          // columns past N re-read the last row; never stored
  const unsigned char* wrow = p.W + (static_cast<int64_t>(e) * p.N + n) * p.ldw * 2 + lq * 32;
  const int nc = n0 + wave * 16 + 4 * lq;          // the 4 consecutive columns this lane ends with
  f32x4_t bias4 = {0.0f, 0.0f, 0.0f, 0.0f};
  if (!PARTIAL && p.bias != nullptr && nc < p.N)
    bias4 = *reinterpret_cast<const f32x4_t*>(p.bias + static_cast<int64_t>(e) * p.N + nc);

  for (int r0 = 0; r0 < c; r0 += RB) {             // row blocks of the segment (one in a decode step)
    const int cc = (c - r0 < RB) ? c - r0 : RB;
    const int nsub = (cc + 15) >> 4;               // subtiles in use; workgroup-uniform
    f32x4_t acc[NSUB];
#pragma unroll
    for (int sub = 0; sub < NSUB; ++sub) acc[sub] = bias4;

    // The weights of a whole chunk (32 bytes per lane and 64-k step) are requested at once,
    // one chunk ahead of the arithmetic: 8-16 KiB per wave in flight while the previous chunk
    // is computed and the activations are staged.
    bf16x8_t wa[2 * STEPS], wb[2 * STEPS];
    auto load_w = [&](bf16x8_t (&w)[2 * STEPS], int kc0) {
      const int kn = (kend - kc0 < KC) ? kend - kc0 : KC;        // multiple of 64
      const unsigned char* wk = wrow + static_cast<int64_t>(kc0) * 2;
#pragma unroll
      for (int st = 0; st < STEPS; ++st) {
        if (st * 64 < kn) {
          w[2 * st] = *reinterpret_cast<const bf16x8_t*>(wk + st * 128);
          w[2 * st + 1] = *reinterpret_cast<const bf16x8_t*>(wk + st * 128 + 16);
        }
      }
    };
    auto chunk = [&](const bf16x8_t (&w)[2 * STEPS], int kc0) {
      const int kn = (kend - kc0 < KC) ? kend - kc0 : KC;
      const int vpr = kn / 8;                                     // 16-byte pieces per row
      __syncthreads();                                            // the previous chunk has been consumed
      for (int i = tid; i < cc * vpr; i += SK_THREADS) {
        const int r = i / vpr, v = i - r * vpr;
        const int64_t src = p.gather ? p.gather[s + r0 + r] : s + r0 + r;
        *reinterpret_cast<uint4*>(xs + r * ROW_BYTES + v * 16) =
            *reinterpret_cast<const uint4*>(p.A + (src * p.lda + kc0) * 2 + v * 16);
      }
      __syncthreads();
      const unsigned char* xl = xs + l16 * ROW_BYTES + lq * 32;
#pragma unroll
      for (int st = 0; st < STEPS; ++st) {
        if (st * 64 < kn) {
#pragma unroll
          for (int sub = 0; sub < NSUB; ++sub) {
            if (sub < nsub) {
              const bf16x8_t a0 = *reinterpret_cast<const bf16x8_t*>(xl + sub * 16 * ROW_BYTES + st * 128);
              const bf16x8_t a1 = *reinterpret_cast<const bf16x8_t*>(xl + sub * 16 * ROW_BYTES + st * 128 + 16);
              acc[sub] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[2 * st], a0, acc[sub], 0, 0, 0);
              acc[sub] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[2 * st + 1], a1, acc[sub], 0, 0, 0);
            }
          }
        }
      }
    };
    if (kbeg < kend) load_w(wa, kbeg);
    for (int kc0 = kbeg; kc0 < kend; kc0 += 2 * KC) {
      if (kc0 + KC < kend) load_w(wb, kc0 + KC);
      chunk(wa, kc0);
      if (kc0 + KC < kend) {
        if (kc0 + 2 * KC < kend) load_w(wa, kc0 + 2 * KC);
        chunk(wb, kc0 + KC);
      }
    }

    // acc[sub][v] = output row r0 + 16 sub + lane % 16 of the segment, column nc + v
    if (nc < p.N) {
#pragma unroll
      for (int sub = 0; sub < NSUB; ++sub) {
        const int r = sub * 16 + l16;
        if (r >= cc) continue;
        const int prow = s + r0 + r;               // packed row
        if (PARTIAL) {
          *reinterpret_cast<f32x4_t*>(partial + (static_cast<int64_t>(blockIdx.z) * RB + prow) * p.N + nc) = acc[sub];
          continue;
        }
        float v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          v[q] = acc[sub][q];
          if (ACT) v[q] = (p.gelu_mode == SCMOE_GELU_TANH) ? gelu_tanh_fast(v[q]) : gelu_erf_fast(v[q]);
        }
        int64_t orow = prow;
        uint2 o;
        if (p.scatter) {
          // output decode: the packed row belongs to token orow; scale by its gate weight and
          // add the row already there
          orow = p.scatter[prow];
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
  }
}

// Sum of the k-parts in part order, then the epilogue of the unsplit kernel.  One thread per
// 4 consecutive columns of one packed row; grid.y = prows, the rows a part holds.
template <bool ACT>
__global__ __launch_bounds__(256) void gemm_skinny_finish(const GemmArgs p, int parts, int prows,
                                                          const float* __restrict__ partial) {
  const int row = blockIdx.y;
  int total = p.offsets[p.E];
  if (total > prows) total = prows;
  if (row >= total) return;
  const int nc = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (nc >= p.N) return;
  int e = 0;
  while (e < p.E - 1 && p.offsets[e + 1] <= row) ++e;
  f32x4_t sum = {0.0f, 0.0f, 0.0f, 0.0f};
  if (p.bias != nullptr) sum = *reinterpret_cast<const f32x4_t*>(p.bias + static_cast<int64_t>(e) * p.N + nc);
  for (int z = 0; z < parts; ++z)
    sum += *reinterpret_cast<const f32x4_t*>(partial + (static_cast<int64_t>(z) * prows + row) * p.N + nc);
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

// A call is one for these kernels if it has at most SK_ROWS rows in all, or if its segments
// average 16 rows or fewer (then a 128- or 256-row tile would be mostly padding).
bool gemm_skinny_fits(int max_rows, int E) {
  return max_rows <= SK_ROWS || (max_rows <= 16 * E && max_rows <= 1024);
}

template <int NSUB>
static int launch_skinny_rows(const GemmArgs& a, bool act, int max_rows, void* scratch, size_t scratch_bytes,
                              hipStream_t stream) {
  constexpr int RB = 16 * NSUB, KC = NSUB == 2 ? 512 : 256;
  const int cols = (a.N + SK_BN - 1) / SK_BN;
  dim3 block(SK_THREADS);
  int parts = 1, cpp = 0;
  if (max_rows <= RB && scratch != nullptr) {
    const int nch = (a.Kd + KC - 1) / KC;
    const int segs = a.E < max_rows ? a.E : max_rows;         // segments that can hold a row
    parts = 512 / (cols * (segs > 0 ? segs : 1));             // aim: about two workgroups per CU
    if (parts > nch) parts = nch;
    if (parts < 1) parts = 1;
    cpp = (nch + parts - 1) / parts;
    parts = (nch + cpp - 1) / cpp;                             // every part holds at least one chunk
    if (static_cast<size_t>(parts) * RB * a.N * sizeof(float) > scratch_bytes) parts = 1;
  }
  if (parts == 1) {
    dim3 grid(cols, a.E);
    if (act) hipLaunchKernelGGL((gemm_skinny_kernel<true, false, NSUB>), grid, block, 0, stream, a, 0, nullptr);
    else hipLaunchKernelGGL((gemm_skinny_kernel<false, false, NSUB>), grid, block, 0, stream, a, 0, nullptr);
    return launch_status();
  }
  float* partial = static_cast<float*>(scratch);
  hipLaunchKernelGGL((gemm_skinny_kernel<false, true, NSUB>), dim3(cols, a.E, parts), block, 0, stream, a, cpp, partial);
  int st = launch_status();
  if (st != SCMOE_OK) return st;
  dim3 fgrid((a.N / 4 + 255) / 256, RB);
  if (act) hipLaunchKernelGGL((gemm_skinny_finish<true>), fgrid, dim3(256), 0, stream, a, parts, RB, partial);
  else hipLaunchKernelGGL((gemm_skinny_finish<false>), fgrid, dim3(256), 0, stream, a, parts, RB, partial);
  return launch_status();
}

// One grouped GEMM of few rows per segment (max_rows: the caller's bound on the packed rows).
// Kd must be a multiple of 64 and the dense extra segment of GemmArgs is not supported
// (xrows == 0).  At most SK_ROWS rows and scratch given: the k range is cut into parts, one
// workgroup each, so that a call with few column blocks (the shared expert: one segment)
// still streams its weights with the whole chip; the parts meet in `scratch`
// ([parts][32 or 64][N] fp32).
int launch_gemm_skinny(const GemmArgs& a, bool act, int max_rows, void* scratch, size_t scratch_bytes,
                       hipStream_t stream) {
  if (a.xrows != 0 || (a.Kd % 64) != 0 || a.E < 1 || a.N < 1 || !gemm_skinny_fits(max_rows, a.E)) return SCMOE_ERR_ARG;
  if (max_rows <= 32) return launch_skinny_rows<2>(a, act, max_rows, scratch, scratch_bytes, stream);
  return launch_skinny_rows<4>(a, act, max_rows, scratch, scratch_bytes, stream);
}

}  // namespace scmoe
