// Input encode (ScMoE paper Sec. 2.2): capacity-bounded stable permutation of token rows
// into per-expert segments.  On one GPU this replaces "encode + All-to-All dispatch".
//
// Items are (token t, choice j) pairs in the order i = j*T + t, so every first choice is
// ranked before any second choice, every second before any third, and so on.  The slot of an item is the number of earlier items of
// the same expert.  Positions come from counting (ballot / popcount / prefix sums), never
// from the arrival order of atomics, so the permutation is reproducible bit for bit.
//
//   hist : per block of 256 items, items per expert            -> blockhist[nblk, E]
//   scan : exclusive prefix over blocks, counts, offsets       -> blockbase[nblk, E]
//   rank : slot = blockbase + waves before + lanes before      -> dst_row, src_token
//   rows : x_perm[r, :] = x[src_token[r], :] for r < offsets[E]
#include "common.hpp"

namespace scmoe {

constexpr int DISP_BLOCK = 256;

// Scratch of scmoe_dispatch_static, the entry point that allocates nothing: the block
// histograms and block bases that scmoe_dispatch keeps in the caller's workspace live in this
// array instead.  Every device that loads the library holds its own copy until the process
// ends.  In host code the name stands for the symbol, not for a device address: the address
// on the current device comes from hipGetSymbolAddress (static_scratch below) and only that
// pointer is handed to kernels.
constexpr size_t DISPATCH_STATIC_BYTES = size_t(2) << 20;
static __device__ __align__(256) unsigned char scratch[DISPATCH_STATIC_BYTES];

__device__ __forceinline__ int item_expert(const int32_t* __restrict__ expert_idx, int i, int n,
                                           int T, int k, int E, int* t_out, int* j_out) {
  if (i >= n) return -1;
  const int j = i / T;
  const int t = i - j * T;
  *t_out = t;
  *j_out = j;
  const int e = expert_idx[static_cast<int64_t>(t) * k + j];
  return (e >= 0 && e < E) ? e : -1;
}

__global__ __launch_bounds__(DISP_BLOCK) void dispatch_hist(const int32_t* __restrict__ expert_idx,
                                                           int T, int k, int E,
                                                           int32_t* __restrict__ blockhist) {
  __shared__ int hist[SCMOE_MAX_EXPERTS];
  const int tid = threadIdx.x;
  if (tid < E) hist[tid] = 0;
  __syncthreads();
  int t, j;
  const int e = item_expert(expert_idx, blockIdx.x * DISP_BLOCK + tid, T * k, T, k, E, &t, &j);
  if (e >= 0) atomicAdd(&hist[e], 1);  // integer counts: the sum does not depend on order
  __syncthreads();
  if (tid < E) blockhist[static_cast<int64_t>(blockIdx.x) * E + tid] = hist[tid];
}

// One workgroup of four waves.  Each wave takes experts wave, wave+4, ...; its lanes take 64
// consecutive blocks at a time and a shuffle scan gives the exclusive prefix over blocks.
__global__ __launch_bounds__(256) void dispatch_scan(const int32_t* __restrict__ blockhist, int nblk,
                                                     int E, int capacity,
                                                     int32_t* __restrict__ blockbase,
                                                     int32_t* __restrict__ counts,
                                                     int32_t* __restrict__ offsets, const ScanChores ch) {
  __shared__ int cnt[SCMOE_MAX_EXPERTS];
  if (ch.pair != nullptr && threadIdx.x == 0) {
    ch.pair[0] = 0;
    ch.pair[1] = ch.pair_hi;
  }
  for (int i = threadIdx.x; i < ch.nzero; i += blockDim.x) {
    if (ch.zero_a != nullptr) ch.zero_a[i] = 0;
    if (ch.zero_b != nullptr) ch.zero_b[i] = 0;
  }
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  for (int e = wave; e < E; e += 4) {
    int run = 0;
    for (int b0 = 0; b0 < nblk; b0 += 64) {
      const int b = b0 + lane;
      const int h = (b < nblk) ? blockhist[static_cast<int64_t>(b) * E + e] : 0;
      int incl = h;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const int up = __shfl_up(incl, off, 64);
        if (lane >= off) incl += up;
      }
      if (b < nblk) blockbase[static_cast<int64_t>(b) * E + e] = run + incl - h;
      run += __shfl(incl, 63, 64);
    }
    if (lane == 0) {
      const int c = run < capacity ? run : capacity;
      cnt[e] = c;
      counts[e] = c;
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0;
    for (int q = 0; q < E; ++q) {
      offsets[q] = run;
      run += cnt[q];
    }
    offsets[E] = run;
  }
}

__global__ __launch_bounds__(DISP_BLOCK) void dispatch_rank(
    const int32_t* __restrict__ expert_idx, int T, int k, int E, int capacity,
    const int32_t* __restrict__ blockbase, const int32_t* __restrict__ offsets,
    int32_t* __restrict__ dst_row, int32_t* __restrict__ src_token) {
  __shared__ int wavecnt[DISP_BLOCK / 64][SCMOE_MAX_EXPERTS];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  for (int c = tid; c < (DISP_BLOCK / 64) * SCMOE_MAX_EXPERTS; c += DISP_BLOCK) (&wavecnt[0][0])[c] = 0;
  __syncthreads();
  int t = 0, j = 0;
  const int e = item_expert(expert_idx, blockIdx.x * DISP_BLOCK + tid, T * k, T, k, E, &t, &j);
  const bool valid = e >= 0;
  // lanes of this wave that hold the same expert (an emulated "match any")
  unsigned long long same = __ballot(valid);
  for (int b = 0; (1 << b) < E; ++b) {
    const unsigned long long bal = __ballot(valid && ((e >> b) & 1));
    same &= ((e >> b) & 1) ? bal : ~bal;
  }
  const unsigned long long below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  const int before = __popcll(same & below);
  if (valid && before == 0) wavecnt[wave][e] = __popcll(same);
  __syncthreads();
  const int i = blockIdx.x * DISP_BLOCK + tid;
  if (i < T * k) {
    int out = -1;
    if (valid) {
      int slot = blockbase[static_cast<int64_t>(blockIdx.x) * E + e] + before;
      for (int w = 0; w < wave; ++w) slot += wavecnt[w][e];
      if (slot < capacity) {
        out = offsets[e] + slot;
        src_token[out] = t;
      }
    }
    dst_row[static_cast<int64_t>(t) * k + j] = out;
  }
}

// hist + scan + rank in ONE workgroup of 16 waves for calls of at most DISP_SMALL_ITEMS items
// (decode steps), where three dependent launches cost more than the work: the items are
// walked in chunks of 1024 (a lane keeps the experts of its items in registers), once to
// count and once to rank; same results as the three kernels.  (Measured: 5 us less per layer
// call up to 1024 tokens, even at 2048; with 8 or 16 chunks one workgroup takes 10-17 us
// longer than the three kernels.)
constexpr int DISP_SMALL_THREADS = 1024;
constexpr int DISP_SMALL_CHUNKS = 2;
constexpr int DISP_SMALL_ITEMS = DISP_SMALL_THREADS * DISP_SMALL_CHUNKS;

__global__ __launch_bounds__(DISP_SMALL_THREADS) void dispatch_small(
    const int32_t* __restrict__ expert_idx, int T, int k, int E, int capacity, int32_t* __restrict__ counts,
    int32_t* __restrict__ offsets, int32_t* __restrict__ dst_row, int32_t* __restrict__ src_token,
    const ScanChores ch) {
  constexpr int NW = DISP_SMALL_THREADS / 64;
  __shared__ int wcnt[NW][SCMOE_MAX_EXPERTS];     // items per (wave, expert) of the current chunk
  __shared__ int seen[SCMOE_MAX_EXPERTS];         // items per expert: all (first pass) / in earlier chunks (second)
  __shared__ int offs[SCMOE_MAX_EXPERTS + 1];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  if (ch.pair != nullptr && tid == 0) {
    ch.pair[0] = 0;
    ch.pair[1] = ch.pair_hi;
  }
  for (int i = tid; i < ch.nzero; i += DISP_SMALL_THREADS) {
    if (ch.zero_a != nullptr) ch.zero_a[i] = 0;
    if (ch.zero_b != nullptr) ch.zero_b[i] = 0;
  }
  const int n = T * k;
  const int nchunk = (n + DISP_SMALL_THREADS - 1) / DISP_SMALL_THREADS;
  if (tid < SCMOE_MAX_EXPERTS) seen[tid] = 0;
  __syncthreads();
  // lanes of this wave that hold the same expert as this lane, and how many of them come before it
  auto match = [&](int e, bool valid, int& before, int& total) {
    unsigned long long same = __ballot(valid);
    for (int b = 0; (1 << b) < E; ++b) {
      const unsigned long long bal = __ballot(valid && ((e >> b) & 1));
      same &= ((e >> b) & 1) ? bal : ~bal;
    }
    const unsigned long long below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    before = __popcll(same & below);
    total = __popcll(same);
  };
  int ev[DISP_SMALL_CHUNKS];
#pragma unroll
  for (int q = 0; q < DISP_SMALL_CHUNKS; ++q) {
    ev[q] = -1;
    if (q < nchunk) {
      int t, j;
      ev[q] = item_expert(expert_idx, q * DISP_SMALL_THREADS + tid, n, T, k, E, &t, &j);
      int before, total;
      match(ev[q], ev[q] >= 0, before, total);
      if (ev[q] >= 0 && before == 0) atomicAdd(&seen[ev[q]], total);   // integer counts: order does not matter
    }
  }
  __syncthreads();
  if (tid == 0) {
    int run = 0;
    for (int e = 0; e < E; ++e) {
      const int c = seen[e] < capacity ? seen[e] : capacity;
      counts[e] = c;
      offsets[e] = run;
      offs[e] = run;
      run += c;
    }
    offsets[E] = run;
    offs[E] = run;
  }
  __syncthreads();
  if (tid < SCMOE_MAX_EXPERTS) seen[tid] = 0;
#pragma unroll
  for (int q = 0; q < DISP_SMALL_CHUNKS; ++q) {
    if (q < nchunk) {
      for (int c = tid; c < NW * SCMOE_MAX_EXPERTS; c += DISP_SMALL_THREADS) (&wcnt[0][0])[c] = 0;
      __syncthreads();
      const int e = ev[q];
      const bool valid = e >= 0;
      int before, total;
      match(e, valid, before, total);
      if (valid && before == 0) wcnt[wave][e] = total;
      __syncthreads();
      const int i = q * DISP_SMALL_THREADS + tid;
      if (i < n) {
        const int j = i / T;
        const int t = i - j * T;
        int out = -1;
        if (valid) {
          int slot = seen[e] + before;
          for (int w = 0; w < wave; ++w) slot += wcnt[w][e];
          if (slot < capacity) {
            out = offs[e] + slot;
            src_token[out] = t;
          }
        }
        dst_row[static_cast<int64_t>(t) * k + j] = out;
      }
      __syncthreads();
      if (tid < E) {
        int add = 0;
        for (int w = 0; w < NW; ++w) add += wcnt[w][tid];
        seen[tid] += add;
      }
      // (the next chunk's clearing of wcnt comes after a barrier of its own: see below)
      __syncthreads();
    }
  }
}

// x_perm[r, :] = x[src_token[r], :], 16 bytes per lane, one wave per row.
__global__ __launch_bounds__(256) void gather_rows(const unsigned char* __restrict__ x, int64_t ldx_bytes,
                                                   const int32_t* __restrict__ src_token,
                                                   const int32_t* __restrict__ offsets, int E,
                                                   int row_bytes, unsigned char* __restrict__ x_perm,
                                                   int64_t ldp_bytes) {
  const int K = offsets[E];
  const int lane = threadIdx.x & 63;
  const int wave = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  const int nwaves = gridDim.x * (blockDim.x >> 6);
  for (int r = wave; r < K; r += nwaves) {
    const int src = src_token[r];
    const unsigned char* s = x + static_cast<int64_t>(src) * ldx_bytes;
    unsigned char* q = x_perm + static_cast<int64_t>(r) * ldp_bytes;
    for (int c = lane * 16; c < row_bytes; c += 64 * 16 * 4) {
      uint4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (c + u * 1024 < row_bytes) v[u] = *reinterpret_cast<const uint4*>(s + c + u * 1024);
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (c + u * 1024 < row_bytes) *reinterpret_cast<uint4*>(q + c + u * 1024) = v[u];
    }
  }
}

static inline int disp_nblk(int T, int k) {
  const int64_t n = static_cast<int64_t>(T) * k;
  return static_cast<int>((n + DISP_BLOCK - 1) / DISP_BLOCK);
}

size_t dispatch_ws_bytes(int T, int E, int k) {
  // blockhist + blockbase, each [nblk, E] int32, rounded up to 256 bytes
  const size_t one = static_cast<size_t>(disp_nblk(T, k)) * static_cast<size_t>(E) * sizeof(int32_t);
  return ((2 * one + 255) / 256) * 256;
}

int dispatch(const void* x, int64_t ldx, int dtype, const int32_t* expert_idx, int T, int d, int E,
             int k, int capacity, int32_t* counts, int32_t* offsets, int32_t* dst_row,
             int32_t* src_token, void* x_perm, int64_t ld_perm, void* workspace, size_t ws_bytes,
             hipStream_t stream, const ScanChores* chores) {
  if (!dtype_ok(dtype)) return SCMOE_ERR_DTYPE;
  if (T < 0 || E < 1 || E > SCMOE_MAX_EXPERTS || capacity < 0) return SCMOE_ERR_SHAPE;
  if (k < 1 || k > SCMOE_MAX_TOPK) return SCMOE_ERR_ARG;
  if (static_cast<int64_t>(T) * k > 0x7fffffffLL) return SCMOE_ERR_SHAPE;
  if (!counts || !offsets) return SCMOE_ERR_NULL;
  if (T > 0 && (!expert_idx || !dst_row || !src_token)) return SCMOE_ERR_NULL;
  if (x_perm != nullptr) {
    if (d <= 0 || (d % 8) != 0) return SCMOE_ERR_SHAPE;
    if (T > 0 && !x) return SCMOE_ERR_NULL;
    if (T > 0 && (!view_ok(x, ldx, d, dtype) || !view_ok(x_perm, ld_perm, d, dtype))) return SCMOE_ERR_SHAPE;
  }
  if (ws_bytes < dispatch_ws_bytes(T, E, k)) return SCMOE_ERR_WORKSPACE;
  if (T > 0 && !workspace) return SCMOE_ERR_NULL;
  const int nblk = disp_nblk(T, k);
  const bool small = static_cast<int64_t>(T) * k <= DISP_SMALL_ITEMS;
  if (small) {
    hipLaunchKernelGGL(dispatch_small, dim3(1), dim3(DISP_SMALL_THREADS), 0, stream, expert_idx, T, k, E, capacity,
                       counts, offsets, dst_row, src_token, chores ? *chores : ScanChores{});
  } else {
    int32_t* blockhist = static_cast<int32_t*>(workspace);
    int32_t* blockbase = blockhist + static_cast<size_t>(nblk) * E;
    hipLaunchKernelGGL(dispatch_hist, dim3(nblk), dim3(DISP_BLOCK), 0, stream, expert_idx, T, k, E, blockhist);
    hipLaunchKernelGGL(dispatch_scan, dim3(1), dim3(256), 0, stream, blockhist, nblk, E, capacity, blockbase,
                       counts, offsets, chores ? *chores : ScanChores{});
    hipLaunchKernelGGL(dispatch_rank, dim3(nblk), dim3(DISP_BLOCK), 0, stream, expert_idx, T, k, E, capacity,
                       blockbase, offsets, dst_row, src_token);
  }
  if (nblk > 0) {
    if (x_perm != nullptr) {
      const int64_t max_rows = static_cast<int64_t>(T) * k;
      int blocks = static_cast<int>((max_rows + 3) / 4);
      if (blocks > 4096) blocks = 4096;
      const int eb = elem_bytes(dtype);
      hipLaunchKernelGGL(gather_rows, dim3(blocks), dim3(256), 0, stream, static_cast<const unsigned char*>(x),
                         ldx * eb, src_token, offsets, E, d * eb, static_cast<unsigned char*>(x_perm),
                         ld_perm * eb);
    }
  }
  return launch_status();
}

}  // namespace scmoe

extern "C" int scmoe_dispatch_workspace_bytes(int32_t T, int32_t E, int32_t k, size_t* out) {
  if (!out) return SCMOE_ERR_NULL;
  if (T < 0 || E < 1 || E > SCMOE_MAX_EXPERTS) return SCMOE_ERR_SHAPE;
  if (k < 1 || k > SCMOE_MAX_TOPK) return SCMOE_ERR_ARG;
  *out = scmoe::dispatch_ws_bytes(T, E, k);
  return SCMOE_OK;
}

// Device address of `scratch` on the current device, looked up once per device.
static int static_scratch(void** out) {
  constexpr int MAXDEV = 64;
  static std::atomic<void*> ptrs[MAXDEV];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return scmoe::hip_fail(e);
  if (dev < 0 || dev >= MAXDEV) return SCMOE_ERR_ARG;
  void* p = ptrs[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scmoe::scratch));
    if (e != hipSuccess) return scmoe::hip_fail(e);
    if (p == nullptr) return SCMOE_ERR_HIP;
    ptrs[dev].store(p, std::memory_order_release);     // (two threads may both look it up: same address)
  }
  *out = p;
  return SCMOE_OK;
}

extern "C" int scmoe_dispatch_static_max_bytes(size_t* out) {
  if (!out) return SCMOE_ERR_NULL;
  *out = scmoe::DISPATCH_STATIC_BYTES;
  return SCMOE_OK;
}

extern "C" int scmoe_dispatch_static(const void* x, int64_t ldx, int32_t dtype, const int32_t* expert_idx,
                                     int32_t T, int32_t d, int32_t E, int32_t k, int32_t capacity,
                                     int32_t* counts, int32_t* offsets, int32_t* dst_row,
                                     int32_t* src_token, void* x_perm, int64_t ld_perm, void* stream) {
  if (T < 0 || E < 1 || E > SCMOE_MAX_EXPERTS) return SCMOE_ERR_SHAPE;
  if (k < 1 || k > SCMOE_MAX_TOPK) return SCMOE_ERR_ARG;
  if (static_cast<int64_t>(T) * k > 0x7fffffffLL) return SCMOE_ERR_SHAPE;
  if (scmoe::dispatch_ws_bytes(T, E, k) > scmoe::DISPATCH_STATIC_BYTES) return SCMOE_ERR_WORKSPACE;
  void* ws = nullptr;
  const int st = static_scratch(&ws);
  if (st != SCMOE_OK) return st;
  // The kernels write every scratch entry they later read (the block histograms, then the block
  // bases), so nothing has to be cleared between calls.
  return scmoe::dispatch(x, ldx, dtype, expert_idx, T, d, E, k, capacity, counts, offsets, dst_row, src_token,
                         x_perm, ld_perm, ws, scmoe::DISPATCH_STATIC_BYTES, static_cast<hipStream_t>(stream),
                         nullptr);
}

extern "C" int scmoe_dispatch(const void* x, int64_t ldx, int32_t dtype, const int32_t* expert_idx,
                              int32_t T, int32_t d, int32_t E, int32_t k, int32_t capacity,
                              int32_t* counts, int32_t* offsets, int32_t* dst_row,
                              int32_t* src_token, void* x_perm, int64_t ld_perm, void* workspace,
                              size_t ws_bytes, void* stream) {
  return scmoe::dispatch(x, ldx, dtype, expert_idx, T, d, E, k, capacity, counts, offsets, dst_row,
                         src_token, x_perm, ld_perm, workspace, ws_bytes, static_cast<hipStream_t>(stream), nullptr);
}
