/*
 * scmoe.h — C ABI of the MI355X (gfx950) ScMoE forward-pass library.
 *
 * One shortcut-connected MoE block (ScMoE paper, Sec. 3.1, Eq. (7)):
 *
 *     y = SE(x_cur) + sum_i G(x_prev)_i * E_i(x_prev)        (+ x_cur if a residual is passed)
 *
 * split into the operators of the expert-parallel workflow (Sec. 2.2): gate routing,
 * input encode (= dispatch permutation), expert computation, output decode (= combine).
 * On one GPU the two All-to-All steps of that workflow are the identity.
 *
 * Conventions that hold for every entry point
 * -------------------------------------------
 *  - Every pointer is a DEVICE pointer unless its comment says "host".  All buffers are
 *    owned by the caller; the library allocates and frees no device memory and keeps no
 *    pointer after it returns.
 *  - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Argument checks
 *    run synchronously on the host; kernels are enqueued on the stream and the call returns
 *    without synchronising.
 *  - The return value is a status code (SCMOE_OK == 0).  On an error nothing is launched (one
 *    exception, stated at the entry: the expert pool of the offload calls turning out too
 *    small).  No exception and no abort crosses the boundary.
 *  - Matrices are row-major.  `ld*` arguments are row strides in ELEMENTS.
 *  - `dtype` (SCMOE_F32 or SCMOE_BF16) is the storage type of activations and of the FFN
 *    weight matrices.  Gate weights W_g, gate bias, FFN biases, gate_w and probs are
 *    always fp32; indices, counts and offsets are int32.
 *  - bf16 buffers must be 16-byte aligned with row strides that are multiples of 8
 *    elements; fp32 buffers 16-byte aligned with strides that are multiples of 4.
 *    d and F must be multiples of 8.  Violations give SCMOE_ERR_SHAPE.
 *  - T == 0 is legal everywhere (no-op, SCMOE_OK).
 */
#ifndef SCMOE_H
#define SCMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  SCMOE_OK = 0,
  SCMOE_ERR_NULL = 1,      /* a required pointer is NULL                         */
  SCMOE_ERR_SHAPE = 2,     /* a size, stride or alignment is outside the contract */
  SCMOE_ERR_DTYPE = 3,     /* dtype is neither SCMOE_F32 nor SCMOE_BF16           */
  SCMOE_ERR_WORKSPACE = 4, /* the workspace passed is too small                   */
  SCMOE_ERR_HIP = 5,       /* a HIP call failed; see scmoe_last_hip_error()       */
  SCMOE_ERR_ARG = 6        /* an option value (mode flag, k, ...) is not supported */
};

enum { SCMOE_F32 = 0, SCMOE_BF16 = 1 };

/* GELU flavour of the expert MLPs.  The paper only says the experts are MLPs (Sec. 2.1);
 * the exact erf form 0.5 v (1 + erf(v / sqrt 2)) is the default reading. */
enum { SCMOE_GELU_ERF = 0, SCMOE_GELU_TANH = 1 };

/* How the shared expert's output and the routed output are merged (Sec. 5.2):
 * direct add (Eq. (6)), CG-1 (Eq. (14)-(15)), CG-2 (Eq. (16)-(17)). */
enum { SCMOE_CG_NONE = 0, SCMOE_CG_1 = 1, SCMOE_CG_2 = 2 };

/* Upper limit on the number of experts accepted by the gate and dispatch kernels. */
#define SCMOE_MAX_EXPERTS 64
/* Upper limit on k, the routed experts per token (the paper's layers use 1, 2 and 3). */
#define SCMOE_MAX_TOPK 4

/* Shape and options of one layer.  Plain data, host memory, read during the call only. */
typedef struct scmoe_desc {
  int32_t T;         /* tokens                                                        */
  int32_t d;         /* model width                                                   */
  int32_t F;         /* FFN hidden width                                              */
  int32_t E;         /* routed experts, 1..SCMOE_MAX_EXPERTS                          */
  int32_t k;         /* routed experts per token, 1..min(E, SCMOE_MAX_TOPK).  ScMoE
                        proper uses 1; 2 with the shared expert is ScMoE-2; the standard
                        layers of Table 4 use 2 and 3                                  */
  int32_t capacity;  /* C: rows an expert accepts; >= T*k means unbounded             */
  int32_t dtype;     /* SCMOE_F32 / SCMOE_BF16                                        */
  int32_t gelu_mode; /* SCMOE_GELU_ERF / SCMOE_GELU_TANH                              */
  int32_t normalize; /* gate weights: 0 = softmax over all E logits evaluated at the
                        selected experts; 1 = softmax over the k selected logits only
                        (Eq. (2) taken literally; for k = 1 that weight is 1)          */
  int32_t cg_mode;   /* SCMOE_CG_NONE / SCMOE_CG_1 / SCMOE_CG_2                        */
} scmoe_desc;

/* Weights of one layer.  Host struct of device pointers. */
typedef struct scmoe_weights {
  const float* W_g;  /* [d, E] gate matrix of Eq. (4), fp32                            */
  const float* bias; /* [E] deterministic additive gate term in the slot of Eq. (4)'s
                        epsilon, or NULL                                               */
  const void* W1;    /* [E, F, d] first linear layer of every routed expert ([out,in]) */
  const float* b1;   /* [E, F] or NULL                                                 */
  const void* W2;    /* [E, d, F] second linear layer ([out,in])                       */
  const float* b2;   /* [E, d] or NULL                                                 */
  const void* W1s;   /* [F, d] shared expert (unused by moe_topk_layer_forward)        */
  const float* b1s;  /* [F] or NULL                                                    */
  const void* W2s;   /* [d, F]                                                         */
  const float* b2s;  /* [d] or NULL                                                    */
  const float* W_cg; /* [1, d] (CG-1) or [2, d] (CG-2), fp32; NULL when cg_mode == 0   */
  int64_t ld_w1;     /* row stride, in elements, of W1 and W1s (>= d; 0 means d).  Expert e
                        of W1 starts at element e * F * ld_w1                          */
  int64_t ld_w2;     /* row stride, in elements, of W2 and W2s (>= F; 0 means F).  Expert e
                        of W2 starts at element e * d * ld_w2                          */
} scmoe_weights;

/* Optional copies of the routing state of a layer call.  Each member may be NULL. */
typedef struct scmoe_routing_out {
  int32_t* expert_idx; /* [T*k]                                                       */
  float* gate_w;       /* [T*k]                                                       */
  int32_t* counts;     /* [E]                                                         */
  int32_t* offsets;    /* [E+1]                                                       */
  int32_t* dst_row;    /* [T*k]                                                       */
  int32_t* src_token;  /* [min(T*k, E*C)]                                             */
} scmoe_routing_out;

/* Text for a status code.  Host, static storage. */
const char* scmoe_status_string(int status);

/* hipError_t (as int) of the most recent SCMOE_ERR_HIP on the calling thread. */
int scmoe_last_hip_error(void);

/* Tuning knob, process-wide and the only state the library keeps between calls (one atomic
 * integer, read once per launch; no environment variable is consulted): tile configuration of
 * the bf16 grouped GEMM behind scmoe_expert_ffn and the layer calls.  Meant for benchmarks and
 * tests; a call that races with a change of the knob uses the old or the new value.
 * 0 (default) = chosen per launch: 256x256x64 tiles,
 * 8 waves, 2 LDS stages, or 128x128 tiles, 2 waves, when the larger tiles would not give
 * every compute unit one (128x128x32, or 128x128x64 with 4 waves and 3 stages when even those
 * are fewer than the compute units); 1 = always 256x256x32, 8 waves, 4 stages; 2 = always
 * 128x128x32; 3 = always 128x128x64.
 * Results agree to bf16 rounding of the same fp32 sums; only speed differs.  Other values
 * give SCMOE_ERR_ARG. */
int scmoe_set_gemm_variant(int32_t variant);

/* Row stride (in elements) that staggers the rows of a GEMM operand of `width` columns:
 * `width` itself, or `width` plus 128 bytes of padding when the dense stride is a multiple
 * of 512 bytes.  With every operand and the output at power-of-two strides, all workgroups
 * reach the same cache channels in step; staggering any one of the matrices breaks that up
 * (measured +19 % on a dense 32768 x 8192 x 2048 bf16 product with no bias).  The layer
 * calls lay out their intermediate `hidden` this way, which is enough for them; the helper
 * is for callers of scmoe_expert_ffn, who own `hidden`, and for weight strides if wanted.
 * Host only; `ld` is a host pointer. */
int scmoe_padded_ld(int32_t width, int32_t dtype, int64_t* ld);

/* Capacity from a capacity factor (Tables 8-9 give only the factor): C = ceil(cf*k*T/E),
 * the ceiling taken after removing rounding noise of the double product.  Host only.
 * `C` is a host pointer. */
int scmoe_capacity(int32_t T, int32_t E, int32_t k, double cf, int32_t* C);

/*
 * Gate routing, top-1 (Eq. (2)-(4) with k = 1 and epsilon = 0; ScMoE applies it to the
 * preceding-layer representation, Sec. 3.1).
 *
 *   logit[t,e] = fp32 chain  acc = 0; for i = 0..d-1: acc = fma(x[t,i], W_g[i,e], acc);
 *                then  + bias[e]  (one rounded add; skipped when bias == NULL)
 *   expert_idx[t] = argmax_e logit[t,e], lowest e on ties, a NaN never wins
 *   gate_w[t]     = softmax(logit[t,:])[expert_idx[t]]   (normalize == 0)
 *                 = 1                                    (normalize == 1)
 *   probs[t,:]    = softmax(logit[t,:])                  (optional, may be NULL)
 *
 * The ascending-i single-FMA chain is part of the contract: it fixes the logits bit for
 * bit and with them the routing.  x: [T, d] with stride ldx, dtype as given (bf16 is
 * widened exactly).  W_g: [d, E] fp32, E <= SCMOE_MAX_EXPERTS; any 4-byte aligned address is
 * accepted, a 16-byte aligned one takes the faster kernel (the results are the same).
 */
int scmoe_gate_top1(const void* x, int64_t ldx, int32_t dtype, const float* W_g,
                    const float* bias, int32_t T, int32_t d, int32_t E, int32_t normalize,
                    int32_t* expert_idx, float* gate_w, float* probs, void* stream);

/*
 * Gate routing, top-2 (Eq. (2)-(4) with k = 2), used by the standard MoE layer that the
 * paper takes as its baseline.  Same logits as above.  expert_idx[t,0] is the arg max,
 * expert_idx[t,1] the arg max among the remaining experts (lowest index on ties; needs
 * E >= 2).  normalize == 1: gate_w[t,:] = softmax over the two selected logits (Eq. (2));
 * normalize == 0: the two entries of the full softmax.
 * expert_idx, gate_w: [T, 2] row-major.
 */
int scmoe_gate_top2(const void* x, int64_t ldx, int32_t dtype, const float* W_g,
                    const float* bias, int32_t T, int32_t d, int32_t E, int32_t normalize,
                    int32_t* expert_idx, float* gate_w, float* probs, void* stream);

/*
 * Gate routing for any k in 1..min(E, SCMOE_MAX_TOPK) (Eq. (2)-(4); k = 3 is the standard
 * top-3 layer that Table 4 compares ScMoE-2 with).  Same logits as above.  expert_idx[t,j]
 * is the arg max among the experts not listed in expert_idx[t,0..j-1] (lowest index on ties,
 * a NaN never wins), so a row lists the k largest logits in descending order.
 * normalize == 1: gate_w[t,:] = softmax over the k selected logits; normalize == 0: their
 * entries of the full softmax.  expert_idx, gate_w: [T, k] row-major.  k = 1 and k = 2 give
 * exactly what scmoe_gate_top1 / scmoe_gate_top2 give.  SCMOE_ERR_ARG for k outside
 * 1..SCMOE_MAX_TOPK, SCMOE_ERR_SHAPE for k > E.
 */
int scmoe_gate_topk(const void* x, int64_t ldx, int32_t dtype, const float* W_g,
                    const float* bias, int32_t T, int32_t d, int32_t E, int32_t k,
                    int32_t normalize, int32_t* expert_idx, float* gate_w, float* probs,
                    void* stream);

/* Bytes of workspace scmoe_dispatch needs.  `out` is a host pointer. */
int scmoe_dispatch_workspace_bytes(int32_t T, int32_t E, int32_t k, size_t* out);

/*
 * Input encode (Sec. 2.2): the capacity-bounded permutation of token rows into contiguous
 * per-expert segments.
 *
 * Items are the (token t, choice j) pairs, ordered by (j, t): every first choice comes
 * before any second choice, every second before any third, and so on.  The slot of an item inside its expert e is the number of
 * earlier items routed to e; the item is kept iff slot < capacity.
 *
 *   counts[e]        = min(#items routed to e, capacity)
 *   offsets[0..E]    = exclusive prefix sum of counts; offsets[E] = K, the kept items
 *   dst_row[t*k + j] = offsets[e] + slot if kept, else -1
 *   src_token[r]     = t for the item stored in packed row r, r < K (entries >= K are
 *                      left untouched)
 *   x_perm[r, :]     = x[src_token[r], :]   (raw row copy; may be NULL to skip the copy)
 *
 * expert_idx: [T*k], values in [0, E) — values outside that range are treated as
 * dropped.  src_token and x_perm must have room for min(T*k, E*capacity) rows.
 * The result is deterministic (a stable counting sort), not dependent on scheduling.
 */
int scmoe_dispatch(const void* x, int64_t ldx, int32_t dtype, const int32_t* expert_idx,
                   int32_t T, int32_t d, int32_t E, int32_t k, int32_t capacity,
                   int32_t* counts, int32_t* offsets, int32_t* dst_row, int32_t* src_token,
                   void* x_perm, int64_t ld_perm, void* workspace, size_t ws_bytes,
                   void* stream);

/*
 * scmoe_dispatch for callers that cannot allocate or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without the
 * workspace, same results bit for bit.  The scratch is a static device array inside the
 * library of scmoe_dispatch_static_max_bytes bytes (2 MiB; each GPU the library runs on holds
 * one until the process ends); the call allocates and frees nothing.  A call that would need
 * more (scmoe_dispatch_workspace_bytes(T, E, k) above that size, i.e. T * k * E beyond about
 * 67 million) gives SCMOE_ERR_WORKSPACE and launches nothing.  All calls on one GPU share
 * the array: calls that may overlap in time on one GPU (different streams, different host
 * threads) race and must be ordered by the caller.
 */
int scmoe_dispatch_static(const void* x, int64_t ldx, int32_t dtype, const int32_t* expert_idx,
                          int32_t T, int32_t d, int32_t E, int32_t k, int32_t capacity,
                          int32_t* counts, int32_t* offsets, int32_t* dst_row,
                          int32_t* src_token, void* x_perm, int64_t ld_perm, void* stream);

/* Size in bytes of the static scratch behind scmoe_dispatch_static.  `out` is a host pointer. */
int scmoe_dispatch_static_max_bytes(size_t* out);

/*
 * Expert computation (Eq. (1); the experts are two-layer MLPs, Sec. 2.1) as a grouped
 * GEMM over packed segments:
 *
 *   for e in 0..E-1, r in [offsets[e], offsets[e+1]):
 *       hidden[r, :] = GELU(W1[e] . x_perm[r, :] + b1[e])
 *       y_perm[r, :] = W2[e] . hidden[r, :] + b2[e]
 *
 * offsets: [E+1] on the DEVICE (read by the kernels, never by the host); offsets[E] must
 * not exceed max_rows, the number of rows x_perm / hidden / y_perm hold (rows past
 * offsets[E] are not touched).  W1: [E, F, d] with row stride ldw1 (expert e starts at
 * element e * F * ldw1), W2: [E, d, F] with row stride ldw2, in `dtype`; b1 [E, F],
 * b2 [E, d] fp32 or NULL.  hidden: caller scratch [max_rows, F] in `dtype`, row stride ldh.
 * All strides are in elements, multiples of 8, and at least the row width.
 * bf16: fp32 accumulation, hidden and y_perm rounded to bf16 (RNE) on store.
 * workspace: optional device scratch of scmoe_expert_ffn_workspace_bytes bytes (16-byte
 * aligned).  With it the bf16 kernels cut the tiles of the last, partly filled round of
 * workgroups along K and add the parts up in a fixed order (results stay run-to-run
 * identical; they may differ in the last bit from a call without workspace).  NULL, or
 * fewer bytes than asked for: that round runs unsplit.  Calls that may overlap in time
 * need separate workspaces.
 * max_rows <= 64, or max_rows <= 16 E and max_rows <= 1024 (decode steps; bf16, d and F
 * multiples of 64): the call
 * is bound by reading the weights, and a weight-streaming kernel replaces the tiled one; up to
 * 64 rows and with a workspace it cuts K into parts so that the whole chip streams (parts
 * summed in a fixed order).
 * hidden with a row stride of scmoe_padded_ld(F) instead of F is worth about 15 % of the
 * first GEMM when F * 2 bytes is a large power of two.
 * With E = 1 and offsets = {0, T} this is the dense MLP used for the shared expert
 * (Eq. (6)).
 */
int scmoe_expert_ffn(const void* x_perm, int64_t ld_perm, int32_t dtype,
                     const int32_t* offsets, int32_t max_rows, int32_t E, int32_t d,
                     int32_t F, const void* W1, int64_t ldw1, const float* b1,
                     const void* W2, int64_t ldw2, const float* b2, void* hidden,
                     int64_t ldh, void* y_perm, int64_t ldy, int32_t gelu_mode,
                     void* workspace, size_t ws_bytes, void* stream);

/* Bytes of optional scratch scmoe_expert_ffn can use for these widths (0 when the shape
 * takes a path that needs none).  `out` is a host pointer. */
int scmoe_expert_ffn_workspace_bytes(int32_t dtype, int32_t d, int32_t F, size_t* out);

/*
 * Output decode (Sec. 2.2) fused with the merge of Eq. (6)/(7):
 *
 *   y[t,:] = c0[t] * base[t,:] + c1[t] * sum_j gate_w[t*k+j] * y_perm[dst_row[t*k+j], :]
 *            + residual[t,:]
 *
 * Terms with dst_row == -1 are skipped (a dropped token's expert output is exactly 0).
 * base (the shared expert's output) and residual may each be NULL.  c0 = c1 = 1 unless a
 * coefficient gate is given: coef != NULL holds [T, 2] fp32 pairs (c0, c1) as produced by
 * scmoe_coef_gate.  Arithmetic in fp32; y is rounded once on store.  y may alias base or
 * residual when the strides match.
 */
int scmoe_combine(const void* y_perm, int64_t ldyp, int32_t dtype, const int32_t* dst_row,
                  const float* gate_w, int32_t T, int32_t d, int32_t k, const void* base,
                  int64_t ldbase, const void* residual, int64_t ldres, const float* coef,
                  void* y, int64_t ldy, void* stream);

/*
 * Coefficient gate (Sec. 5.2).  CG-1, Eq. (14): c0 = sigmoid(W_cg . x), c1 = 1.
 * CG-2, Eq. (16): (c0, c1) = softmax(W_cg . x) with W_cg of two rows.  The dot products
 * are fp32 sums (no bit-exact contract; they feed no integer decision).
 * x: [T, d]; W_cg: [1, d] or [2, d] fp32; coef: [T, 2] fp32.
 */
int scmoe_coef_gate(const void* x, int64_t ldx, int32_t dtype, const float* W_cg,
                    int32_t cg_mode, int32_t T, int32_t d, float* coef, void* stream);

/* Bytes of workspace a layer call needs for `desc`.  `desc`, `out`: host pointers. */
int scmoe_workspace_bytes(const scmoe_desc* desc, size_t* out);

/*
 * One ScMoE block forward (Eq. (7); module form: without the residual unless given):
 *
 *   y = SE(x_cur) + sum_i G(x_prev)_i E_i(x_prev)
 *
 * = gate(x_prev) -> dispatch -> expert_ffn -> combine(base = SE(x_cur)).
 * The shared expert depends on x_cur only and the routed chain on x_prev only (Sec. 3.2):
 * with stream_aux != NULL the shared expert's GEMMs are enqueued on stream_aux and the
 * routed chain on stream_main, forked and joined with events.  Where the output decode is fused
 * into the routed experts' second GEMM (bf16 MFMA path, k = 1, y apart from the inputs) the join
 * sits in front of that second GEMM only: gate, encode and the routed first GEMM run beside the
 * shared expert; otherwise the whole routed chain does and the join sits in front of the
 * combine kernel.  With stream_aux == NULL
 * everything runs in order on stream_main (and, on the bf16 MFMA path, the first GEMMs of the
 * shared and the routed experts share one launch).  The result is ready on stream_main.
 * (Measured on one MI355X: kernels of a few thousand tokens and more fill the chip and a second
 * stream gains nothing; up to about 4096 tokens it saves 5-13 % of the call.)
 * desc->k = 1 is ScMoE; desc->k = 2 routes two experts per token on x_prev (ScMoE-2,
 * appendix "more activated experts"); larger k up to SCMOE_MAX_TOPK follows the same rule.
 * With desc->cg_mode != 0 the coefficient gate reads x_cur.
 * residual may be NULL.  routing may be NULL.  y may be the buffer of x_prev, x_cur or
 * residual (same pointer and row stride; any other overlap is not supported): the call then
 * takes a path that has read a row before it writes it.  No host synchronisation happens inside, no
 * memory is allocated and no memset is enqueued, so the call can be captured in a HIP graph
 * (after one ordinary call on the device, which creates the events and sets kernel attributes).
 * Reproducibility: the routing is the same in every mode; y is the same bits for the same
 * call repeated, but one- and two-stream calls may differ in the last bit (the tiles of a
 * GEMM that are cut along K depend on what shares its launch).
 */
int scmoe_layer_forward(const scmoe_desc* desc, const void* x_prev, int64_t ld_prev,
                        const void* x_cur, int64_t ld_cur, const scmoe_weights* w,
                        const void* residual, int64_t ldres, void* y, int64_t ldy,
                        const scmoe_routing_out* routing, void* workspace, size_t ws_bytes,
                        void* stream_main, void* stream_aux);

/* Bytes of the device pool that receives migrated experts: room for `pool_experts` experts
 * (W1, W2, b1, b2 of each).  `desc`, `out`: host pointers. */
int scmoe_offload_pool_bytes(const scmoe_desc* desc, int32_t pool_experts, size_t* out);

/*
 * ScMoE block forward with the gate-routed experts offloaded to host memory and migrated on
 * demand (Sec. 5.3 "expert offloading", appendix A.3): the shared expert and the gate stay
 * on the GPU; because ScMoE selects experts from the preceding-layer representation, the
 * selection is known before the current layer's computation starts, and exactly the selected
 * experts are copied host -> device (determinate migration, nothing is predicted) while the
 * shared expert runs.
 *
 *   w->W1, w->W2, w->b1, w->b2   HOST pointers ([E,F,d], [E,d,F], [E,F], [E,d]; dense;
 *                                pinned memory is needed for the copies to overlap);
 *   all other members of w       device pointers as in scmoe_layer_forward;
 *   expert_pool                  device, 256-byte aligned, scmoe_offload_pool_bytes bytes;
 *   host_plan                    host scratch of 2*E + 1 int32 (pinned recommended); on return
 *                                [0, E) holds the kept rows per expert;
 *   async_copy                   1: copies on stream_copy, overlapped with the shared expert
 *                                ("Offload-Async"); 0: copies on stream_main in front of the
 *                                shared expert ("Offload", blocking migration).
 *
 * The call synchronises stream_main once on the host (the host reads the per-expert counts to
 * issue the copies).  SCMOE_ERR_WORKSPACE if more experts are selected than the pool holds:
 * that is known only once the counts are on the host, so for this one error gate routing and
 * input encode HAVE run and stream_main HAS been synchronised when the call returns (nothing
 * else is enqueued); every other error is found before anything is launched.
 * Result: the same from call to call; equal to scmoe_layer_forward's on the same inputs up
 * to rounding (the two launch their GEMMs differently, see there).
 * This call is scmoe_offload_begin followed at once by scmoe_offload_finish: only the shared
 * expert is then available to hide the copies behind.  Callers with work of their own to put
 * in between (the attention and MLP of the block pair, Sec. 5.3) use the two calls below.
 */
int scmoe_layer_forward_offload(const scmoe_desc* desc, const void* x_prev, int64_t ld_prev,
                                const void* x_cur, int64_t ld_cur, const scmoe_weights* w,
                                void* expert_pool, int32_t pool_experts, int32_t async_copy,
                                int32_t* host_plan, void* y, int64_t ldy, void* workspace,
                                size_t ws_bytes, void* stream_main, void* stream_copy);

/*
 * The two halves of scmoe_layer_forward_offload (same arguments, same meaning).
 *
 * scmoe_offload_begin: gate routing and input encode on x_prev, the per-expert counts to
 * host_plan, one host synchronisation of stream_main, then the copies of exactly the selected
 * experts into the pool are ISSUED (on stream_copy behind an event when async_copy = 1, else on
 * stream_main) and the call returns.  Whatever the caller enqueues on stream_main after it runs
 * while the experts migrate: this window between "selection known" and "experts needed" is the
 * mechanism of Sec. 5.3 / appendix A.3.  SCMOE_ERR_WORKSPACE as described above.
 *
 * scmoe_offload_finish: the shared expert on x_cur, then (behind the copies) the routed
 * experts from the pool, output decode and merge into y.  Must follow a scmoe_offload_begin
 * with the same desc, weights, pool, host_plan, workspace and streams; between the two calls
 * the caller must leave the workspace, the pool and host_plan alone (they carry the routing
 * and the migrating experts) and must enqueue nothing on stream_copy.  No host synchronisation.
 */
int scmoe_offload_begin(const scmoe_desc* desc, const void* x_prev, int64_t ld_prev,
                        const scmoe_weights* w, void* expert_pool, int32_t pool_experts,
                        int32_t async_copy, int32_t* host_plan, void* workspace, size_t ws_bytes,
                        void* stream_main, void* stream_copy);
int scmoe_offload_finish(const scmoe_desc* desc, const void* x_prev, int64_t ld_prev,
                         const void* x_cur, int64_t ld_cur, const scmoe_weights* w,
                         void* expert_pool, int32_t pool_experts, int32_t async_copy,
                         const int32_t* host_plan, void* y, int64_t ldy, void* workspace,
                         size_t ws_bytes, void* stream_main, void* stream_copy);

/*
 * Standard top-k MoE layer on the current-layer representation (Eq. (1)-(4); k = 2 is the
 * baseline the paper compares with, Fig. 2(a)):  y = sum_j gate_w[t,j] E_{idx[t,j]}(x[t]).
 * desc->k in 1..min(E, SCMOE_MAX_TOPK); k = 3 is the standard top-3 layer of Table 4, which
 * has the compute volume of ScMoE-2.  Shared-expert members of `w` are ignored.
 */
int moe_topk_layer_forward(const scmoe_desc* desc, const void* x, int64_t ldx,
                           const scmoe_weights* w, void* y, int64_t ldy,
                           const scmoe_routing_out* routing, void* workspace,
                           size_t ws_bytes, void* stream);

/* The k = 2 case of moe_topk_layer_forward under the name the baseline is known by. */
int moe_top2_layer_forward(const scmoe_desc* desc, const void* x, int64_t ldx,
                           const scmoe_weights* w, void* y, int64_t ldy,
                           const scmoe_routing_out* routing, void* workspace,
                           size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SCMOE_H */
