// Internal helpers shared by the HIP sources of libscmoe (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "scmoe.h"

namespace scmoe {

// Last HIP error seen by an entry point on this thread (reported by scmoe_last_hip_error).
extern thread_local int g_last_hip_error;

inline int hip_fail(hipError_t e) {
  g_last_hip_error = static_cast<int>(e);
  return SCMOE_ERR_HIP;
}

// Status of the kernel launch that was just enqueued.
inline int launch_status() {
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? SCMOE_OK : hip_fail(e);
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline int elem_bytes(int dtype) { return dtype == SCMOE_BF16 ? 2 : 4; }

// Elements per 16-byte vector.
inline int vec_elems(int dtype) { return dtype == SCMOE_BF16 ? 8 : 4; }

inline bool dtype_ok(int dtype) { return dtype == SCMOE_F32 || dtype == SCMOE_BF16; }

// A matrix view is acceptable when its base is 16-byte aligned and its row stride keeps
// every row 16-byte aligned and covers `cols`.
inline bool view_ok(const void* p, int64_t ld, int64_t cols, int dtype) {
  return aligned16(p) && ld >= cols && (ld % vec_elems(dtype)) == 0;
}

// ---- bf16 <-> fp32 on the device (bit manipulation; round to nearest even) -------------
__device__ __forceinline__ float bf16_to_f32(uint16_t v) {
  return __uint_as_float(static_cast<uint32_t>(v) << 16);
}

__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7f800000u) == 0x7f800000u) {  // inf / nan: keep the class, quiet a nan
    return static_cast<uint16_t>((u >> 16) | ((u & 0xffffu) ? 0x40u : 0u));
  }
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<uint16_t>(u >> 16);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return static_cast<uint32_t>(f32_to_bf16(lo)) | (static_cast<uint32_t>(f32_to_bf16(hi)) << 16);
}

// GELU of the expert MLPs: exact erf form or the tanh approximation.
__device__ __forceinline__ float gelu_f32(float v, int mode) {
  if (mode == SCMOE_GELU_TANH) {
    const float c = 0.7978845608028654f;
    return 0.5f * v * (1.0f + tanhf(c * (v + 0.044715f * v * v * v)));
  }
  return 0.5f * v * (1.0f + erff(v * 0.70710678118654752f));
}

// Small chores that a layer call would otherwise launch kernels of their own for; the single
// workgroup of the dispatch scan does them on the side: pair[0..1] = {0, pair_hi} (the segment
// bounds of the shared expert) and nzero zeros at each of zero_a, zero_b.  All optional.
struct ScanChores {
  int32_t* pair = nullptr;
  int pair_hi = 0;
  int* zero_a = nullptr;
  int* zero_b = nullptr;
  int nzero = 0;
};

// ---- entry points implemented in one source and used by the layer orchestration --------
// One expert-FFN call over packed segments.  All strides in elements.
struct FfnArgs {
  const void* x; int64_t ldx;      // [rows, d] activations
  const int32_t* gather;           // row r reads x[gather[r]] (the dispatch permutation applied
                                   // on load); nullptr = identity.  MFMA path only.
  int64_t x_rows;                  // with gather: rows of x that gather may name
  const int32_t* offsets;          // [E + 1] segment starts, device
  int max_rows, E, d, F;
  const void* W1; int64_t ldw1; const float* b1;   // [E, F, d]
  const void* W2; int64_t ldw2; const float* b2;   // [E, d, F]
  void* hidden; int64_t ldh;       // [rows, F] scratch
  void* y; int64_t ldy;            // [rows, d]
  int gelu_mode;
  // Fused output decode of the second GEMM (MFMA path only; all three pointers nullptr: off).
  // With scatter (addend optional in the tiled kernel, required by the few-row one):
  //   y[scatter[r], :] = addend[scatter[r], :] + row_scale[scatter[r]] * (W2 . hidden[r] + b2)
  // Without scatter (rows stay in place; tiled kernel only, not the few-row one), row_scale
  // holding PAIRS of coefficients per row of which the first is used, either pointer optional:
  //   y[r, :] = addend[r, :] + row_scale[2 r] * (W2 . hidden[r] + b2)
  const int32_t* scatter; const float* row_scale; const void* addend; int64_t ldadd;
  // Scratch of the MFMA path (split-K of the last round of tiles); may be nullptr: no split.
  void* scratch; size_t scratch_bytes;
  bool scratch_zeroed;             // the arrival counters at the start of scratch are zero already
  // Event the stream waits for between the first and the second GEMM (nullptr: none).  MFMA path.
  hipEvent_t before_second;
};

int ffn_generic(const FfnArgs& a, int dtype, hipStream_t stream);

// bf16 MFMA path.  Returns SCMOE_ERR_ARG when the shape is outside what the MFMA kernels
// cover (the caller then uses ffn_generic).
int ffn_mfma_bf16(const FfnArgs& a, hipStream_t stream);
// shared expert `se` (one dense segment) and routed experts `rt` with their first GEMMs in one launch
int ffn_mfma_bf16_pair(const FfnArgs& se, const FfnArgs& rt, hipStream_t stream);

// Row stride the grouped GEMM likes for an operand of `width` columns: rows at a multiple
// of 512 bytes get 128 bytes of padding.
inline int64_t padded_ld(int64_t width, int dtype) {
  const int64_t eb = elem_bytes(dtype);
  return ((width * eb) % 512 == 0) ? width + 128 / eb : width;
}
bool ffn_mfma_supported(int d, int F);
bool gemm_skinny_fits(int max_rows, int E);   // the MFMA path would take its few-row kernel for such a call
size_t ffn_mfma_scratch_bytes();   // scratch the MFMA path can use (16-byte aligned)
int ffn_mfma_counter_ints();       // ints at the start of that scratch that must be zero before a call

// Compute units of the current device (256 on MI355X), cached per device.
inline int num_cus() {
  static std::atomic<int> cached[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  int n = cached[dev].load(std::memory_order_relaxed);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 8) n = 256;
    cached[dev].store(n, std::memory_order_relaxed);
  }
  return n;
}

}  // namespace scmoe
