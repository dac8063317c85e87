// C-ABI entry points that are not a single kernel: status text, capacity, workspace sizes,
// the expert FFN dispatcher, and the layer orchestration of ScMoE (paper Eq. (7), Sec. 3.2)
// and of the standard top-k MoE layer (Eq. (1)-(4)).
#include "common.hpp"

#include <math.h>

namespace scmoe {

thread_local int g_last_hip_error = 0;

int gate_topk(const void* x, int64_t ldx, int dtype, const float* Wg, const float* bias, int T,
              int d, int E, int k, int normalize, int32_t* idx, float* gw, float* probs,
              hipStream_t stream);
size_t dispatch_ws_bytes(int T, int E, int k);
int dispatch(const void* x, int64_t ldx, int dtype, const int32_t* expert_idx, int T, int d, int E,
             int k, int capacity, int32_t* counts, int32_t* offsets, int32_t* dst_row,
             int32_t* src_token, void* x_perm, int64_t ld_perm, void* workspace, size_t ws_bytes,
             hipStream_t stream, const ScanChores* chores);
int combine(const void* y_perm, int64_t ldyp, int dtype, const int32_t* dst_row, const float* gate_w,
            int T, int d, int k, const void* base, int64_t ldbase, const void* residual,
            int64_t ldres, const float* coef, void* y, int64_t ldy, hipStream_t stream);
int coef_gate(const void* x, int64_t ldx, int dtype, const float* Wcg, int mode, int T, int d,
              float* coef, hipStream_t stream);

static inline size_t align256(size_t v) { return (v + 255) & ~static_cast<size_t>(255); }

// Rows the packed buffers must hold: min(T*k, E*C) without overflow.
static inline int64_t packed_rows(int T, int E, int k, int capacity) {
  const int64_t items = static_cast<int64_t>(T) * k;
  const int64_t cap = static_cast<int64_t>(E) * capacity;
  return items < cap ? items : cap;
}

static int check_desc(const scmoe_desc* D, int kmin, int kmax) {
  if (!D) return SCMOE_ERR_NULL;
  if (!dtype_ok(D->dtype)) return SCMOE_ERR_DTYPE;
  if (D->T < 0 || D->d <= 0 || D->F <= 0 || (D->d % 8) || (D->F % 8) || D->E < 1 ||
      D->E > SCMOE_MAX_EXPERTS || D->capacity < 0)
    return SCMOE_ERR_SHAPE;
  if (static_cast<int64_t>(D->T) * SCMOE_MAX_TOPK > 0x7fffffffLL) return SCMOE_ERR_SHAPE;
  if (D->k < kmin || D->k > kmax) return SCMOE_ERR_ARG;
  if (D->k > D->E) return SCMOE_ERR_SHAPE;
  if (D->gelu_mode != SCMOE_GELU_ERF && D->gelu_mode != SCMOE_GELU_TANH) return SCMOE_ERR_ARG;
  if (D->normalize != 0 && D->normalize != 1) return SCMOE_ERR_ARG;
  if (D->cg_mode < SCMOE_CG_NONE || D->cg_mode > SCMOE_CG_2) return SCMOE_ERR_ARG;
  return SCMOE_OK;
}

// Carves the layer workspace.  Every piece starts on a 256-byte boundary.
struct LayerWs {
  int32_t* expert_idx; float* gate_w; int32_t* counts; int32_t* offsets; int32_t* dst_row;
  int32_t* src_token; int32_t* offsets_shared; int32_t* offsets_c; float* coef; float* gate_cg; void* disp_ws; size_t disp_bytes;
  void* x_perm; void* hidden; void* y_perm; void* hidden_s; void* s;
  void* scratch_r; void* scratch_s; size_t scratch_bytes;   // GEMM scratch of the routed / shared chain
  int64_t ldh;   // row stride of hidden and hidden_s
  size_t total;
};

static LayerWs carve(const scmoe_desc* D, void* base, bool shared) {
  LayerWs w{};
  size_t off = 0;
  unsigned char* b = static_cast<unsigned char*>(base);
  auto take = [&](size_t bytes) {
    void* p = b ? b + off : nullptr;
    off += align256(bytes);
    return p;
  };
  const size_t items = static_cast<size_t>(D->T) * D->k;
  const size_t rows = static_cast<size_t>(packed_rows(D->T, D->E, D->k, D->capacity));
  const size_t eb = elem_bytes(D->dtype);
  w.expert_idx = static_cast<int32_t*>(take(items * 4));
  w.gate_w = static_cast<float*>(take(items * 4));
  w.counts = static_cast<int32_t*>(take(static_cast<size_t>(D->E) * 4));
  w.offsets = static_cast<int32_t*>(take(static_cast<size_t>(D->E + 1) * 4));
  w.dst_row = static_cast<int32_t*>(take(items * 4));
  w.src_token = static_cast<int32_t*>(take(rows * 4));
  w.offsets_shared = static_cast<int32_t*>(take(8));
  w.offsets_c = static_cast<int32_t*>(take(static_cast<size_t>(D->E + 1) * 4));   // offload: present experts only
  w.coef = static_cast<float*>(take(D->cg_mode ? static_cast<size_t>(D->T) * 8 : 0));
  w.gate_cg = static_cast<float*>(take(D->cg_mode ? static_cast<size_t>(D->T) * 4 : 0));   // gate weight x routed coefficient
  w.disp_bytes = dispatch_ws_bytes(D->T, D->E, D->k);
  w.disp_ws = take(w.disp_bytes);
  w.x_perm = take(rows * D->d * eb);
  w.ldh = padded_ld(D->F, D->dtype);
  w.hidden = take(rows * w.ldh * eb);
  w.y_perm = take(rows * D->d * eb);
  w.scratch_bytes = (D->dtype == SCMOE_BF16 && ffn_mfma_supported(D->d, D->F)) ? ffn_mfma_scratch_bytes() : 0;
  w.scratch_r = take(w.scratch_bytes);
  if (shared) {
    w.scratch_s = take(w.scratch_bytes);   // the two chains may run at the same time
    w.hidden_s = take(static_cast<size_t>(D->T) * w.ldh * eb);
    w.s = take(static_cast<size_t>(D->T) * D->d * eb);
  }
  w.total = off;
  return w;
}

// out[t] = gate_w[t] * coef[2 t + 1]: the factor of a token's routed row under a coefficient gate (top-1)
__global__ void scale_gate(const float* __restrict__ gate_w, const float* __restrict__ coef, float* __restrict__ out, int T) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t < T) out[t] = gate_w[t] * coef[2 * static_cast<int64_t>(t) + 1];
}

// One wave per token: the output row of a token whose (single) routed item was dropped is
// set to zero (standard top-1 layer with the decode fused into the second GEMM, which only
// writes the rows of kept tokens).  pieces = 16-byte pieces per row.
__global__ __launch_bounds__(256) void zero_dropped_rows(unsigned char* __restrict__ y, int64_t ldy_bytes,
                                                         const int32_t* __restrict__ dst_row, int T, int pieces) {
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T || dst_row[t] >= 0) return;
  for (int c = threadIdx.x & 63; c < pieces; c += 64)
    *reinterpret_cast<uint4*>(y + static_cast<int64_t>(t) * ldy_bytes + static_cast<int64_t>(c) * 16) = make_uint4(0u, 0u, 0u, 0u);
}

__global__ void set_pair(int32_t* p, int a, int b) {
  if (threadIdx.x == 0) {
    p[0] = a;
    p[1] = b;
  }
}

// FFN over segments: MFMA path for bf16 shapes it covers, else the generic kernel.
static int expert_ffn_any(const FfnArgs& a, int dtype, hipStream_t stream) {
  if (a.max_rows <= 0) return SCMOE_OK;
  if (dtype == SCMOE_BF16 && ffn_mfma_supported(a.d, a.F)) return ffn_mfma_bf16(a, stream);
  if (a.gather != nullptr || a.scatter != nullptr) return SCMOE_ERR_ARG;  // packed rows in, packed rows out only
  return ffn_generic(a, dtype, stream);
}

static inline int64_t ld_or(int64_t ld, int64_t dense) { return ld ? ld : dense; }

static bool gather_on_load(const scmoe_desc* D) {
  return D->dtype == SCMOE_BF16 && ffn_mfma_supported(D->d, D->F);
}

// Fork/join events of the two-stream layer call: one pair per host thread and device.
struct EventPair { hipEvent_t fork = nullptr, join = nullptr; };
static int get_events(EventPair** out) {
  constexpr int MAXDEV = 64;
  static thread_local EventPair pairs[MAXDEV];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e);
  if (dev < 0 || dev >= MAXDEV) return SCMOE_ERR_ARG;
  EventPair& p = pairs[dev];
  if (!p.fork) {
    e = hipEventCreateWithFlags(&p.fork, hipEventDisableTiming);
    if (e != hipSuccess) return hip_fail(e);
    e = hipEventCreateWithFlags(&p.join, hipEventDisableTiming);
    if (e != hipSuccess) return hip_fail(e);
  }
  *out = &p;
  return SCMOE_OK;
}

#define SCMOE_TRY(expr)            \
  do {                             \
    int st__ = (expr);             \
    if (st__ != SCMOE_OK) return st__; \
  } while (0)

static int copy_routing(const scmoe_desc* D, const LayerWs& w, const scmoe_routing_out* r,
                        hipStream_t stream) {
  if (!r || D->T == 0) return SCMOE_OK;
  const size_t items = static_cast<size_t>(D->T) * D->k;
  const size_t rows = static_cast<size_t>(packed_rows(D->T, D->E, D->k, D->capacity));
  struct { void* dst; const void* src; size_t bytes; } cp[6] = {
      {r->expert_idx, w.expert_idx, items * 4}, {r->gate_w, w.gate_w, items * 4},
      {r->counts, w.counts, static_cast<size_t>(D->E) * 4},
      {r->offsets, w.offsets, static_cast<size_t>(D->E + 1) * 4},
      {r->dst_row, w.dst_row, items * 4}, {r->src_token, w.src_token, rows * 4}};
  for (auto& c : cp) {
    if (c.dst && c.bytes) {
      hipError_t e = hipMemcpyAsync(c.dst, c.src, c.bytes, hipMemcpyDeviceToDevice, stream);
      if (e != hipSuccess) return hip_fail(e);
    }
  }
  return SCMOE_OK;
}

// gate -> encode -> experts on `stream`; leaves y_perm, dst_row, gate_w in the workspace.
// With fused_y != nullptr the second GEMM decodes in its epilogue instead (Sec. 2.2 "output
// decode"): row r goes to fused_y[src_token[r], :] += gate_w * expert output, on top of what
// the shared expert has written there; `before_ffn` (optional: the shared expert on another
// stream) is waited for between the first and the second GEMM, so that gate, encode and the
// first GEMM run beside the shared expert.
// With shared != nullptr (MFMA path, same stream) the shared expert runs here too: its first
// GEMM rides in the launch of the routed experts' first GEMM as one more segment.
// With fused_y and row_coef != nullptr (coefficient gate, Eq. (14)-(17)) the decoded rows are
// also scaled by the routed coefficient row_coef[2 t + 1] of their token.
// With fused_y and nothing_below (standard top-1 layer: no shared expert has written fused_y)
// the decoded rows are stored as they are and the rows of dropped tokens are set to zero.
static int routed_chain(const scmoe_desc* D, const void* x, int64_t ldx, const scmoe_weights* W,
                        const LayerWs& w, hipStream_t stream, void* fused_y = nullptr, int64_t ld_fused = 0,
                        hipEvent_t before_ffn = nullptr, const FfnArgs* shared = nullptr,
                        const ScanChores* chores = nullptr, const float* row_coef = nullptr,
                        bool nothing_below = false) {
  SCMOE_TRY(gate_topk(x, ldx, D->dtype, W->W_g, W->bias, D->T, D->d, D->E, D->k, D->normalize,
                      w.expert_idx, w.gate_w, nullptr, stream));
  const bool gol = gather_on_load(D);
  SCMOE_TRY(dispatch(x, ldx, D->dtype, w.expert_idx, D->T, D->d, D->E, D->k, D->capacity, w.counts,
                     w.offsets, w.dst_row, w.src_token, gol ? nullptr : w.x_perm, D->d, w.disp_ws,
                     w.disp_bytes, stream, chores));
  const int rows = static_cast<int>(packed_rows(D->T, D->E, D->k, D->capacity));
  FfnArgs a{};
  a.x = gol ? x : w.x_perm;
  a.ldx = gol ? ldx : D->d;
  a.gather = gol ? w.src_token : nullptr;
  a.x_rows = D->T;
  a.offsets = w.offsets;
  a.max_rows = rows; a.E = D->E; a.d = D->d; a.F = D->F;
  a.W1 = W->W1; a.ldw1 = ld_or(W->ld_w1, D->d); a.b1 = W->b1;
  a.W2 = W->W2; a.ldw2 = ld_or(W->ld_w2, D->F); a.b2 = W->b2;
  a.hidden = w.hidden; a.ldh = w.ldh;
  a.y = w.y_perm; a.ldy = D->d;
  a.gelu_mode = D->gelu_mode;
  a.scratch = w.scratch_bytes ? w.scratch_r : nullptr; a.scratch_bytes = w.scratch_bytes;
  a.scratch_zeroed = chores != nullptr && chores->nzero > 0 && chores->zero_a == a.scratch && a.scratch != nullptr;
  if (fused_y) {
    a.before_second = before_ffn;        // only the decoding second GEMM needs the shared expert's rows
    a.y = fused_y; a.ldy = ld_fused;
    a.scatter = w.src_token; a.row_scale = w.gate_w; a.addend = fused_y; a.ldadd = ld_fused;
    if (nothing_below) {
      a.addend = nullptr;
      hipLaunchKernelGGL(zero_dropped_rows, dim3((D->T + 3) / 4), dim3(256), 0, stream, static_cast<unsigned char*>(fused_y),
                         ld_fused * static_cast<int64_t>(elem_bytes(D->dtype)), w.dst_row, D->T,
                         static_cast<int>(D->d * elem_bytes(D->dtype) / 16));
      SCMOE_TRY(launch_status());
    }
    if (row_coef != nullptr) {
      hipLaunchKernelGGL(scale_gate, dim3((D->T + 255) / 256), dim3(256), 0, stream, w.gate_w, row_coef, w.gate_cg, D->T);
      SCMOE_TRY(launch_status());
      a.row_scale = w.gate_cg;
    }
  }
  if (shared != nullptr) {
    FfnArgs se = *shared;
    se.scratch_zeroed = chores != nullptr && chores->nzero > 0 && chores->zero_b == se.scratch && se.scratch != nullptr;
    return ffn_mfma_bf16_pair(se, a, stream);
  }
  return expert_ffn_any(a, D->dtype, stream);
}

}  // namespace scmoe

using namespace scmoe;

extern "C" const char* scmoe_status_string(int status) {
  switch (status) {
    case SCMOE_OK: return "ok";
    case SCMOE_ERR_NULL: return "a required pointer is NULL";
    case SCMOE_ERR_SHAPE: return "size, stride or alignment outside the contract";
    case SCMOE_ERR_DTYPE: return "unknown dtype";
    case SCMOE_ERR_WORKSPACE: return "workspace too small";
    case SCMOE_ERR_HIP: return "HIP call failed (see scmoe_last_hip_error)";
    case SCMOE_ERR_ARG: return "unsupported option value";
    default: return "unknown status";
  }
}

extern "C" int scmoe_last_hip_error(void) { return g_last_hip_error; }

namespace scmoe { int set_gemm_variant(int v); }
extern "C" int scmoe_set_gemm_variant(int32_t variant) { return scmoe::set_gemm_variant(variant); }

extern "C" int scmoe_padded_ld(int32_t width, int32_t dtype, int64_t* ld) {
  if (!ld) return SCMOE_ERR_NULL;
  if (!dtype_ok(dtype)) return SCMOE_ERR_DTYPE;
  if (width <= 0) return SCMOE_ERR_SHAPE;
  *ld = padded_ld(width, dtype);
  return SCMOE_OK;
}

extern "C" int scmoe_capacity(int32_t T, int32_t E, int32_t k, double cf, int32_t* C) {
  if (!C) return SCMOE_ERR_NULL;
  if (T < 0 || E < 1 || k < 1 || !(cf >= 0.0)) return SCMOE_ERR_SHAPE;
  const long double v = static_cast<long double>(cf) * k * T / E;
  const long double r = nearbyintl(v);
  const long double tol = 1e-9L * (fabsl(v) > 1.0L ? fabsl(v) : 1.0L);
  const long double c = (fabsl(v - r) <= tol) ? r : ceill(v);
  if (c > 2147483647.0L) return SCMOE_ERR_SHAPE;
  *C = static_cast<int32_t>(c);
  return SCMOE_OK;
}

extern "C" int scmoe_expert_ffn(const void* x_perm, int64_t ld_perm, int32_t dtype,
                                const int32_t* offsets, int32_t max_rows, int32_t E, int32_t d,
                                int32_t F, const void* W1, int64_t ldw1, const float* b1,
                                const void* W2, int64_t ldw2, const float* b2, void* hidden,
                                int64_t ldh, void* y_perm, int64_t ldy, int32_t gelu_mode,
                                void* workspace, size_t ws_bytes, void* stream) {
  if (!dtype_ok(dtype)) return SCMOE_ERR_DTYPE;
  if (max_rows < 0 || E < 1 || d <= 0 || F <= 0 || (d % 8) || (F % 8)) return SCMOE_ERR_SHAPE;
  if (gelu_mode != SCMOE_GELU_ERF && gelu_mode != SCMOE_GELU_TANH) return SCMOE_ERR_ARG;
  if (max_rows == 0) return SCMOE_OK;
  if (!x_perm || !offsets || !W1 || !W2 || !hidden || !y_perm) return SCMOE_ERR_NULL;
  if (!view_ok(x_perm, ld_perm, d, dtype) || !view_ok(y_perm, ldy, d, dtype) || !view_ok(hidden, ldh, F, dtype) ||
      !view_ok(W1, ldw1, d, dtype) || !view_ok(W2, ldw2, F, dtype))
    return SCMOE_ERR_SHAPE;
  if ((b1 && !aligned16(b1)) || (b2 && !aligned16(b2))) return SCMOE_ERR_SHAPE;
  FfnArgs a{};
  a.x = x_perm; a.ldx = ld_perm; a.gather = nullptr; a.offsets = offsets;
  a.max_rows = max_rows; a.E = E; a.d = d; a.F = F;
  a.W1 = W1; a.ldw1 = ldw1; a.b1 = b1; a.W2 = W2; a.ldw2 = ldw2; a.b2 = b2;
  a.hidden = hidden; a.ldh = ldh; a.y = y_perm; a.ldy = ldy; a.gelu_mode = gelu_mode;
  if (workspace != nullptr) {
    if (!aligned16(workspace)) return SCMOE_ERR_SHAPE;
    a.scratch = workspace; a.scratch_bytes = ws_bytes;
  }
  return expert_ffn_any(a, dtype, static_cast<hipStream_t>(stream));
}

extern "C" int scmoe_expert_ffn_workspace_bytes(int32_t dtype, int32_t d, int32_t F, size_t* out) {
  if (!out) return SCMOE_ERR_NULL;
  if (!dtype_ok(dtype)) return SCMOE_ERR_DTYPE;
  if (d <= 0 || F <= 0) return SCMOE_ERR_SHAPE;
  *out = (dtype == SCMOE_BF16 && ffn_mfma_supported(d, F)) ? ffn_mfma_scratch_bytes() : 0;
  return SCMOE_OK;
}

extern "C" int scmoe_workspace_bytes(const scmoe_desc* desc, size_t* out) {
  if (!out) return SCMOE_ERR_NULL;
  SCMOE_TRY(check_desc(desc, 1, SCMOE_MAX_TOPK));
  // sized for the shared-expert form; the standard layer uses a prefix of it
  *out = carve(desc, nullptr, true).total;
  return SCMOE_OK;
}

static int check_weights(const scmoe_desc* D, const scmoe_weights* W, bool shared) {
  if (!W) return SCMOE_ERR_NULL;
  if (!W->W_g || !W->W1 || !W->W2) return SCMOE_ERR_NULL;
  if (shared && (!W->W1s || !W->W2s)) return SCMOE_ERR_NULL;
  if (shared && D->cg_mode != SCMOE_CG_NONE && !W->W_cg) return SCMOE_ERR_NULL;
  const void* ptrs[] = {W->W1, W->W2, W->b1, W->b2, shared ? W->W1s : nullptr,
                        shared ? W->W2s : nullptr, shared ? W->b1s : nullptr, shared ? W->b2s : nullptr};
  for (const void* p : ptrs)
    if (p && !aligned16(p)) return SCMOE_ERR_SHAPE;
  const int v = vec_elems(D->dtype);
  if (W->ld_w1 && (W->ld_w1 < D->d || W->ld_w1 % v)) return SCMOE_ERR_SHAPE;
  if (W->ld_w2 && (W->ld_w2 < D->F || W->ld_w2 % v)) return SCMOE_ERR_SHAPE;
  return SCMOE_OK;
}

extern "C" int scmoe_layer_forward(const scmoe_desc* D, const void* x_prev, int64_t ld_prev,
                                   const void* x_cur, int64_t ld_cur, const scmoe_weights* W,
                                   const void* residual, int64_t ldres, void* y, int64_t ldy,
                                   const scmoe_routing_out* routing, void* workspace,
                                   size_t ws_bytes, void* stream_main, void* stream_aux) {
  SCMOE_TRY(check_desc(D, 1, SCMOE_MAX_TOPK));
  SCMOE_TRY(check_weights(D, W, true));
  if (D->T == 0) return SCMOE_OK;
  if (!x_prev || !x_cur || !y || !workspace) return SCMOE_ERR_NULL;
  if (!view_ok(x_prev, ld_prev, D->d, D->dtype) || !view_ok(x_cur, ld_cur, D->d, D->dtype) ||
      !view_ok(y, ldy, D->d, D->dtype) || !aligned16(workspace))
    return SCMOE_ERR_SHAPE;
  if (residual && !view_ok(residual, ldres, D->d, D->dtype)) return SCMOE_ERR_SHAPE;
  const LayerWs w = carve(D, workspace, true);
  if (ws_bytes < w.total) return SCMOE_ERR_WORKSPACE;
  hipStream_t sm = static_cast<hipStream_t>(stream_main);
  hipStream_t sa = static_cast<hipStream_t>(stream_aux);
  const bool two = stream_aux != nullptr && sa != sm;
  hipStream_t s_shared = two ? sa : sm;
  EventPair* ev = nullptr;
  if (two) {
    SCMOE_TRY(get_events(&ev));
    hipError_t e = hipEventRecord(ev->fork, sm);
    if (e != hipSuccess) return hip_fail(e);
    e = hipStreamWaitEvent(sa, ev->fork, 0);
    if (e != hipSuccess) return hip_fail(e);
  }
  // One stream and the MFMA path: the shared expert's first GEMM joins the routed experts'
  // (one launch over E + 1 segments), and the dispatch scan also writes the shared expert's
  // segment bounds and clears the split-K counters of both chains; otherwise the shared expert
  // runs on its own, ahead of the routing, with kernels of its own for those chores.
  const bool joint = !two && gather_on_load(D);
  ScanChores chores;
  if (joint) {
    chores.pair = w.offsets_shared;
    chores.pair_hi = D->T;
    chores.zero_a = static_cast<int*>(w.scratch_r);
    chores.zero_b = static_cast<int*>(w.scratch_s);
    chores.nzero = w.scratch_bytes ? ffn_mfma_counter_ints() : 0;
  } else {
    // shared expert on the current-layer representation (Eq. (6)/(7)): independent of routing
    hipLaunchKernelGGL(set_pair, dim3(1), dim3(64), 0, s_shared, w.offsets_shared, 0, D->T);
    SCMOE_TRY(launch_status());
  }
  // Fused output decode: for top-1 routing on the MFMA path, the shared expert writes y and the
  // routed GEMM2 adds its gate-weighted rows into y[src_token[r]] (every row is written once,
  // dropped tokens keep SE(x_cur)): no y_perm round trip and no combine kernel.  Needs y not
  // to overlap the inputs, which are still being read when y is first written.  With a
  // coefficient gate or a residual the shared expert's GEMM2 decodes too (in place: its rows
  // times the shared coefficient, plus the residual rows), and the routed rows carry the
  // routed coefficient in their factor; the few-row kernels do not have that form.
  const size_t eb = elem_bytes(D->dtype);
  auto overlaps = [&](const void* a, int64_t lda_, const void* b, int64_t ldb_) {
    const unsigned char* a0 = static_cast<const unsigned char*>(a);
    const unsigned char* b0 = static_cast<const unsigned char*>(b);
    const size_t an = static_cast<size_t>(D->T) * lda_ * eb, bn = static_cast<size_t>(D->T) * ldb_ * eb;
    return a0 < b0 + bn && b0 < a0 + an;
  };
  const bool extras = D->cg_mode != SCMOE_CG_NONE || residual != nullptr;
  const bool tiled = !gemm_skinny_fits(D->T, 1) &&
                     !gemm_skinny_fits(static_cast<int>(packed_rows(D->T, D->E, D->k, D->capacity)), D->E);
  const bool fused = D->k == 1 && gather_on_load(D) && !overlaps(y, ldy, x_prev, ld_prev) &&
                     !overlaps(y, ldy, x_cur, ld_cur) &&
                     (!extras || (tiled && (!residual || !overlaps(y, ldy, residual, ldres))));
  FfnArgs se{};
  se.x = x_cur; se.ldx = ld_cur; se.gather = nullptr; se.offsets = w.offsets_shared;
  se.max_rows = D->T; se.E = 1; se.d = D->d; se.F = D->F;
  se.W1 = W->W1s; se.ldw1 = ld_or(W->ld_w1, D->d); se.b1 = W->b1s;
  se.W2 = W->W2s; se.ldw2 = ld_or(W->ld_w2, D->F); se.b2 = W->b2s;
  se.hidden = w.hidden_s; se.ldh = w.ldh; se.gelu_mode = D->gelu_mode;
  se.scratch = w.scratch_bytes ? w.scratch_s : nullptr; se.scratch_bytes = w.scratch_bytes;
  se.y = fused ? y : w.s;
  se.ldy = fused ? ldy : D->d;
  const float* coef = D->cg_mode != SCMOE_CG_NONE ? w.coef : nullptr;
  if (fused && extras) {
    se.row_scale = coef;
    se.addend = residual;
    se.ldadd = ldres;
  }
  if (coef != nullptr)
    SCMOE_TRY(coef_gate(x_cur, ld_cur, D->dtype, W->W_cg, D->cg_mode, D->T, D->d, w.coef, s_shared));
  if (!joint) SCMOE_TRY(expert_ffn_any(se, D->dtype, s_shared));
  if (two) {
    hipError_t e = hipEventRecord(ev->join, sa);
    if (e != hipSuccess) return hip_fail(e);
  }
  // routed experts on the preceding-layer representation
  if (fused) {
    SCMOE_TRY(routed_chain(D, x_prev, ld_prev, W, w, sm, y, ldy, two ? ev->join : nullptr, joint ? &se : nullptr,
                           joint ? &chores : nullptr, coef));
    return copy_routing(D, w, routing, sm);
  }
  SCMOE_TRY(routed_chain(D, x_prev, ld_prev, W, w, sm, nullptr, 0, nullptr, joint ? &se : nullptr,
                         joint ? &chores : nullptr));
  if (two) {
    hipError_t e = hipStreamWaitEvent(sm, ev->join, 0);
    if (e != hipSuccess) return hip_fail(e);
  }
  SCMOE_TRY(combine(w.y_perm, D->d, D->dtype, w.dst_row, w.gate_w, D->T, D->d, D->k, w.s, D->d, residual, ldres,
                    D->cg_mode != SCMOE_CG_NONE ? w.coef : nullptr, y, ldy, sm));
  return copy_routing(D, w, routing, sm);
}

// ---- expert offloading with determinate migration (paper Sec. 5.3 and appendix A.3) --------

namespace scmoe {
// Device pool that receives the migrated experts: slot s holds W1, W2, b1, b2 of one expert.
struct OffloadPool { unsigned char* W1; unsigned char* W2; float* b1; float* b2; size_t total; };
static OffloadPool carve_pool(const scmoe_desc* D, void* base, int slots) {
  OffloadPool p{};
  size_t off = 0;
  unsigned char* b = static_cast<unsigned char*>(base);
  auto take = [&](size_t bytes) {
    unsigned char* q = b ? b + off : nullptr;
    off += align256(bytes);
    return q;
  };
  const size_t eb = elem_bytes(D->dtype), n = static_cast<size_t>(slots);
  p.W1 = take(n * D->F * D->d * eb);
  p.W2 = take(n * D->d * D->F * eb);
  p.b1 = reinterpret_cast<float*>(take(n * D->F * 4));
  p.b2 = reinterpret_cast<float*>(take(n * D->d * 4));
  p.total = off;
  return p;
}
}  // namespace scmoe

extern "C" int scmoe_offload_pool_bytes(const scmoe_desc* D, int32_t pool_experts, size_t* out) {
  if (!out) return SCMOE_ERR_NULL;
  SCMOE_TRY(check_desc(D, 1, SCMOE_MAX_TOPK));
  if (pool_experts < 1 || pool_experts > D->E) return SCMOE_ERR_SHAPE;
  *out = carve_pool(D, nullptr, pool_experts).total;
  return SCMOE_OK;
}

// Checks shared by the three offload entry points.
static int check_offload(const scmoe_desc* D, const scmoe_weights* W, const void* expert_pool, int32_t pool_experts,
                         int32_t async_copy, const int32_t* host_plan, const void* workspace, size_t ws_bytes) {
  SCMOE_TRY(check_desc(D, 1, SCMOE_MAX_TOPK));
  SCMOE_TRY(check_weights(D, W, true));
  if ((W->ld_w1 != 0 && W->ld_w1 != D->d) || (W->ld_w2 != 0 && W->ld_w2 != D->F))
    return SCMOE_ERR_ARG;                                          // host experts are stored dense
  if (async_copy != 0 && async_copy != 1) return SCMOE_ERR_ARG;
  if (pool_experts < 1 || pool_experts > D->E) return SCMOE_ERR_SHAPE;
  if (D->T == 0) return SCMOE_OK;
  if (!workspace || !expert_pool || !host_plan) return SCMOE_ERR_NULL;
  if (!aligned16(workspace) || (reinterpret_cast<uintptr_t>(expert_pool) & 255u) != 0) return SCMOE_ERR_SHAPE;
  if (ws_bytes < carve(D, nullptr, true).total) return SCMOE_ERR_WORKSPACE;
  return SCMOE_OK;
}

// Experts with kept rows take pool slots in expert order, so the packed rows (ordered by
// expert) are the segments of the slots in slot order.  Returns the number of slots in use,
// or -1 when there are more than `pool_experts`; offs_c (if given) receives their segment bounds.
static int offload_plan(const int32_t* counts, int E, int pool_experts, int* slot_expert, int32_t* offs_c) {
  int m = 0;
  if (offs_c) offs_c[0] = 0;
  for (int e = 0; e < E; ++e) {
    if (counts[e] > 0) {
      if (m == pool_experts) return -1;
      slot_expert[m] = e;
      if (offs_c) offs_c[m + 1] = offs_c[m] + counts[e];
      ++m;
    }
  }
  return m;
}

extern "C" int scmoe_offload_begin(const scmoe_desc* D, const void* x_prev, int64_t ld_prev, const scmoe_weights* W,
                                   void* expert_pool, int32_t pool_experts, int32_t async_copy, int32_t* host_plan,
                                   void* workspace, size_t ws_bytes, void* stream_main, void* stream_copy) {
  SCMOE_TRY(check_offload(D, W, expert_pool, pool_experts, async_copy, host_plan, workspace, ws_bytes));
  if (D->T == 0) return SCMOE_OK;
  if (!x_prev) return SCMOE_ERR_NULL;
  if (!view_ok(x_prev, ld_prev, D->d, D->dtype)) return SCMOE_ERR_SHAPE;
  const LayerWs w = carve(D, workspace, true);
  const OffloadPool pool = carve_pool(D, expert_pool, pool_experts);
  hipStream_t sm = static_cast<hipStream_t>(stream_main);
  hipStream_t sc = static_cast<hipStream_t>(stream_copy);
  const bool async = async_copy == 1 && stream_copy != nullptr && sc != sm;
  const size_t eb = elem_bytes(D->dtype);
  const int E = D->E;

  // 1. Expert selection on the preceding-layer representation: known this early, so the
  //    migration below moves exactly the experts that will run (nothing is predicted).
  SCMOE_TRY(gate_topk(x_prev, ld_prev, D->dtype, W->W_g, W->bias, D->T, D->d, E, D->k, D->normalize,
                      w.expert_idx, w.gate_w, nullptr, sm));
  const bool gol = gather_on_load(D);
  SCMOE_TRY(dispatch(x_prev, ld_prev, D->dtype, w.expert_idx, D->T, D->d, E, D->k, D->capacity, w.counts,
                     w.offsets, w.dst_row, w.src_token, gol ? nullptr : w.x_perm, D->d, w.disp_ws,
                     w.disp_bytes, sm, nullptr));
  hipError_t he = hipMemcpyAsync(host_plan, w.counts, static_cast<size_t>(E) * 4, hipMemcpyDeviceToHost, sm);
  if (he != hipSuccess) return hip_fail(he);
  EventPair* ev = nullptr;
  if (async) {
    SCMOE_TRY(get_events(&ev));
    he = hipEventRecord(ev->fork, sm);          // everything that used the pool before is older than this
    if (he != hipSuccess) return hip_fail(he);
  }
  he = hipStreamSynchronize(sm);                // the host needs the counts to issue the copies
  if (he != hipSuccess) return hip_fail(he);

  // 2. Plan and migration.
  int32_t* offs_c = host_plan + E;
  int slot_expert[SCMOE_MAX_EXPERTS];
  const int m = offload_plan(host_plan, E, pool_experts, slot_expert, offs_c);
  if (m < 0) return SCMOE_ERR_WORKSPACE;        // more experts selected than the pool holds
  hipStream_t cs = async ? sc : sm;
  if (async) {
    he = hipStreamWaitEvent(sc, ev->fork, 0);
    if (he != hipSuccess) return hip_fail(he);
  }
  const size_t w_bytes = static_cast<size_t>(D->F) * D->d * eb;
  for (int s = 0; s < m; ++s) {
    const size_t e = static_cast<size_t>(slot_expert[s]);
    he = hipMemcpyAsync(pool.W1 + s * w_bytes, static_cast<const unsigned char*>(W->W1) + e * w_bytes, w_bytes,
                        hipMemcpyHostToDevice, cs);
    if (he != hipSuccess) return hip_fail(he);
    he = hipMemcpyAsync(pool.W2 + s * w_bytes, static_cast<const unsigned char*>(W->W2) + e * w_bytes, w_bytes,
                        hipMemcpyHostToDevice, cs);
    if (he != hipSuccess) return hip_fail(he);
    if (W->b1) {
      he = hipMemcpyAsync(pool.b1 + static_cast<size_t>(s) * D->F, W->b1 + e * D->F, static_cast<size_t>(D->F) * 4,
                          hipMemcpyHostToDevice, cs);
      if (he != hipSuccess) return hip_fail(he);
    }
    if (W->b2) {
      he = hipMemcpyAsync(pool.b2 + static_cast<size_t>(s) * D->d, W->b2 + e * D->d, static_cast<size_t>(D->d) * 4,
                          hipMemcpyHostToDevice, cs);
      if (he != hipSuccess) return hip_fail(he);
    }
  }
  he = hipMemcpyAsync(w.offsets_c, offs_c, static_cast<size_t>(m + 1) * 4, hipMemcpyHostToDevice, cs);
  if (he != hipSuccess) return hip_fail(he);
  return SCMOE_OK;
}

extern "C" int scmoe_offload_finish(const scmoe_desc* D, const void* x_prev, int64_t ld_prev, const void* x_cur,
                                    int64_t ld_cur, const scmoe_weights* W, void* expert_pool, int32_t pool_experts,
                                    int32_t async_copy, const int32_t* host_plan, void* y, int64_t ldy,
                                    void* workspace, size_t ws_bytes, void* stream_main, void* stream_copy) {
  SCMOE_TRY(check_offload(D, W, expert_pool, pool_experts, async_copy, host_plan, workspace, ws_bytes));
  if (D->T == 0) return SCMOE_OK;
  if (!x_prev || !x_cur || !y) return SCMOE_ERR_NULL;
  if (!view_ok(x_prev, ld_prev, D->d, D->dtype) || !view_ok(x_cur, ld_cur, D->d, D->dtype) ||
      !view_ok(y, ldy, D->d, D->dtype))
    return SCMOE_ERR_SHAPE;
  const LayerWs w = carve(D, workspace, true);
  const OffloadPool pool = carve_pool(D, expert_pool, pool_experts);
  hipStream_t sm = static_cast<hipStream_t>(stream_main);
  hipStream_t sc = static_cast<hipStream_t>(stream_copy);
  const bool async = async_copy == 1 && stream_copy != nullptr && sc != sm;
  const int E = D->E;
  int slot_expert[SCMOE_MAX_EXPERTS];
  const int m = offload_plan(host_plan, E, pool_experts, slot_expert, nullptr);
  if (m < 0) return SCMOE_ERR_WORKSPACE;
  hipError_t he;
  EventPair* ev = nullptr;
  if (async) {
    SCMOE_TRY(get_events(&ev));
    he = hipEventRecord(ev->join, sc);          // behind the copies that scmoe_offload_begin put on this stream
    if (he != hipSuccess) return hip_fail(he);
  }

  // 3. Shared expert on the current-layer representation: resident; under asynchronous
  //    migration it runs while the copies are still arriving.
  hipLaunchKernelGGL(set_pair, dim3(1), dim3(64), 0, sm, w.offsets_shared, 0, D->T);
  SCMOE_TRY(launch_status());
  FfnArgs se{};
  se.x = x_cur; se.ldx = ld_cur; se.offsets = w.offsets_shared;
  se.max_rows = D->T; se.E = 1; se.d = D->d; se.F = D->F;
  se.W1 = W->W1s; se.ldw1 = D->d; se.b1 = W->b1s;
  se.W2 = W->W2s; se.ldw2 = D->F; se.b2 = W->b2s;
  se.hidden = w.hidden_s; se.ldh = w.ldh; se.gelu_mode = D->gelu_mode;
  se.scratch = w.scratch_bytes ? w.scratch_s : nullptr; se.scratch_bytes = w.scratch_bytes;
  se.y = w.s; se.ldy = D->d;
  SCMOE_TRY(expert_ffn_any(se, D->dtype, sm));
  if (D->cg_mode != SCMOE_CG_NONE)
    SCMOE_TRY(coef_gate(x_cur, ld_cur, D->dtype, W->W_cg, D->cg_mode, D->T, D->d, w.coef, sm));

  // 4. Routed experts from the pool, then decode and merge.
  if (async) {
    he = hipStreamWaitEvent(sm, ev->join, 0);
    if (he != hipSuccess) return hip_fail(he);
  }
  if (m > 0) {
    const bool gol = gather_on_load(D);
    FfnArgs a{};
    a.x = gol ? x_prev : w.x_perm;
    a.ldx = gol ? ld_prev : D->d;
    a.gather = gol ? w.src_token : nullptr;
    a.x_rows = D->T;
    a.offsets = w.offsets_c;
    a.max_rows = static_cast<int>(packed_rows(D->T, E, D->k, D->capacity));
    a.E = m; a.d = D->d; a.F = D->F;
    a.W1 = pool.W1; a.ldw1 = D->d; a.b1 = W->b1 ? pool.b1 : nullptr;
    a.W2 = pool.W2; a.ldw2 = D->F; a.b2 = W->b2 ? pool.b2 : nullptr;
    a.hidden = w.hidden; a.ldh = w.ldh; a.y = w.y_perm; a.ldy = D->d; a.gelu_mode = D->gelu_mode;
    a.scratch = w.scratch_bytes ? w.scratch_r : nullptr; a.scratch_bytes = w.scratch_bytes;
    SCMOE_TRY(expert_ffn_any(a, D->dtype, sm));
  }
  return combine(w.y_perm, D->d, D->dtype, w.dst_row, w.gate_w, D->T, D->d, D->k, w.s, D->d, nullptr, 0,
                 D->cg_mode != SCMOE_CG_NONE ? w.coef : nullptr, y, ldy, sm);
}

extern "C" int scmoe_layer_forward_offload(const scmoe_desc* D, const void* x_prev, int64_t ld_prev,
                                           const void* x_cur, int64_t ld_cur, const scmoe_weights* W,
                                           void* expert_pool, int32_t pool_experts, int32_t async_copy,
                                           int32_t* host_plan, void* y, int64_t ldy, void* workspace,
                                           size_t ws_bytes, void* stream_main, void* stream_copy) {
  // every argument check of both halves comes before anything is enqueued
  SCMOE_TRY(check_offload(D, W, expert_pool, pool_experts, async_copy, host_plan, workspace, ws_bytes));
  if (D->T == 0) return SCMOE_OK;
  if (!x_prev || !x_cur || !y) return SCMOE_ERR_NULL;
  if (!view_ok(x_prev, ld_prev, D->d, D->dtype) || !view_ok(x_cur, ld_cur, D->d, D->dtype) ||
      !view_ok(y, ldy, D->d, D->dtype))
    return SCMOE_ERR_SHAPE;
  SCMOE_TRY(scmoe_offload_begin(D, x_prev, ld_prev, W, expert_pool, pool_experts, async_copy, host_plan, workspace,
                                ws_bytes, stream_main, stream_copy));
  return scmoe_offload_finish(D, x_prev, ld_prev, x_cur, ld_cur, W, expert_pool, pool_experts, async_copy, host_plan,
                              y, ldy, workspace, ws_bytes, stream_main, stream_copy);
}

extern "C" int moe_topk_layer_forward(const scmoe_desc* D, const void* x, int64_t ldx,
                                      const scmoe_weights* W, void* y, int64_t ldy,
                                      const scmoe_routing_out* routing, void* workspace,
                                      size_t ws_bytes, void* stream) {
  SCMOE_TRY(check_desc(D, 1, SCMOE_MAX_TOPK));
  SCMOE_TRY(check_weights(D, W, false));
  if (D->T == 0) return SCMOE_OK;
  if (!x || !y || !workspace) return SCMOE_ERR_NULL;
  if (!view_ok(x, ldx, D->d, D->dtype) || !view_ok(y, ldy, D->d, D->dtype) || !aligned16(workspace))
    return SCMOE_ERR_SHAPE;
  const LayerWs w = carve(D, workspace, false);
  if (ws_bytes < w.total) return SCMOE_ERR_WORKSPACE;
  hipStream_t sm = static_cast<hipStream_t>(stream);
  // Top-1 on the tiled MFMA path with y apart from x: the second GEMM decodes in its epilogue
  // (y[src_token[r]] = gate weight x row; dropped tokens' rows are zeroed by a kernel of their
  // own), no y_perm round trip and no combine launch.
  const unsigned char* x0 = static_cast<const unsigned char*>(x);
  const unsigned char* y0 = static_cast<const unsigned char*>(y);
  const size_t eb = elem_bytes(D->dtype);
  const bool apart = x0 + static_cast<size_t>(D->T) * ldx * eb <= y0 || y0 + static_cast<size_t>(D->T) * ldy * eb <= x0;
  const bool fused = D->k == 1 && gather_on_load(D) && apart &&
                     !gemm_skinny_fits(static_cast<int>(packed_rows(D->T, D->E, D->k, D->capacity)), D->E);
  if (fused) {
    SCMOE_TRY(routed_chain(D, x, ldx, W, w, sm, y, ldy, nullptr, nullptr, nullptr, nullptr, true));
    return copy_routing(D, w, routing, sm);
  }
  SCMOE_TRY(routed_chain(D, x, ldx, W, w, sm));
  SCMOE_TRY(combine(w.y_perm, D->d, D->dtype, w.dst_row, w.gate_w, D->T, D->d, D->k, nullptr, 0, nullptr, 0,
                    nullptr, y, ldy, sm));
  return copy_routing(D, w, routing, sm);
}

extern "C" int moe_top2_layer_forward(const scmoe_desc* D, const void* x, int64_t ldx,
                                      const scmoe_weights* W, void* y, int64_t ldy,
                                      const scmoe_routing_out* routing, void* workspace,
                                      size_t ws_bytes, void* stream) {
  if (D && D->k != 2) return SCMOE_ERR_ARG;
  return moe_topk_layer_forward(D, x, ldx, W, y, ldy, routing, workspace, ws_bytes, stream);
}
