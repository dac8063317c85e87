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
// Up to 131072 items the first three are one launch (dispatch_onepass).
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

// hist + scan + rank in ONE launch for calls of at most DISP1_MAX_ITEMS items (every workload of
// the paper's tables, and decode steps), where three dependent launches cost more than the work.
// Nothing is handed from workgroup to workgroup: a workgroup owns a block of 1024 consecutive
// items and counts, by itself, the items of every expert in the whole call and in the blocks
// before its own, walking all expert indices (128 KB at 32768 items: they come from the L2).
// The walk is what the kernel costs, so it is made of few instructions per 64 items:
//  * E <= 16: a lane adds 1 << 4e into a 64-bit register of sixteen 4-bit counters (one item per
//    lane and vector, so 15 vectors fit before the nibbles are spread into two registers of
//    8-bit counters: fine up to 255 vectors per wave; the indices of 32 vectors are requested
//    at a time); the 64 lanes' and 16 waves' counters are
//    added up once at the end (wave e sums expert e).
//  * E > 16: one ballot per bit of the expert index per vector; lane L keeps the count of expert L.
// Integer counts only, so the permutation is the same bit for bit as the three kernels'.  No
// scratch memory, no atomics, no waiting.
constexpr int DISP1_THREADS = 1024;
constexpr int DISP1_WAVES = DISP1_THREADS / 64;
constexpr int DISP1_MAX_ITEMS = 131072;
constexpr int DISP1_ROUND = 32;                 // 64-item vectors whose loads are in flight together

template <bool NIB, int K>
__global__ __launch_bounds__(DISP1_THREADS) void dispatch_onepass(
    const int32_t* __restrict__ expert_idx, int T, int E, int capacity, int32_t* __restrict__ counts,
    int32_t* __restrict__ offsets, int32_t* __restrict__ dst_row, int32_t* __restrict__ src_token,
    const ScanChores ch) {
  constexpr int NW = DISP1_WAVES;
  constexpr int k = K;
  static_assert(DISP1_MAX_ITEMS / 64 / NW <= 255 && NW >= 16, "8-bit counters per lane; a wave per expert in the sum");
  // NIB: [0 = whole call, 1 = before this block][wave][lane] -> four words of 8-bit counters
  // (expert e: word (e & 1) * 2 + (e >> 3), byte (e >> 1) & 3); else [.][wave][lane = expert] counts.
  __shared__ int cw[2][NW][64][NIB ? 4 : 1];
  __shared__ int wown[NW][64];     // items per expert in the wave's own 64 items of the block; then their prefix over waves
  __shared__ int tot_s[64];        // items of expert e in the whole call
  __shared__ int seg[64];          // offsets[e]
  __shared__ int bef[64];          // items of expert e before this block
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  if (blockIdx.x == 0) {
    if (ch.pair != nullptr && tid == 0) {
      ch.pair[0] = 0;
      ch.pair[1] = ch.pair_hi;
    }
    for (int i = tid; i < ch.nzero; i += DISP1_THREADS) {
      if (ch.zero_a != nullptr) ch.zero_a[i] = 0;
      if (ch.zero_b != nullptr) ch.zero_b[i] = 0;
    }
  }
  const int n = T * k;
  const int nvec = (n + 63) >> 6;
  const int vb = blockIdx.x * NW;                 // first 64-item vector of this block
  const int i0 = vb * 64;                         // first item of this block
  int nb = 0;
  while ((1 << nb) < E) ++nb;
  // items of this wave's 64 whose expert is `lane` (lanes >= E count nothing that is used), and
  // the lanes that hold the same expert as this lane
  auto count64 = [&](int e, unsigned long long& same) {
    const bool valid = e >= 0;
    unsigned long long mine = __ballot(valid);
    same = mine;
    for (int b = 0; b < nb; ++b) {
      const unsigned long long bal = __ballot(valid && ((e >> b) & 1));
      mine &= ((lane >> b) & 1) ? bal : ~bal;
      same &= ((e >> b) & 1) ? bal : ~bal;
    }
    return __popcll(mine);
  };
  // The walk goes through expert_idx in memory order, 64 entries per wave and step: entry
  // f = t * k + j is item j * T + t.  With k = 1 that is the item order, a vector lies before the
  // block or not as a whole, and "before this block" is a copy of the counters taken when the
  // walk reaches the block; with k > 1 a lane adds to a second set of counters when its item
  // comes before the block's first one.
  constexpr unsigned long long M4 = 0x0f0f0f0f0f0f0f0full;
  unsigned long long nib = 0, lo = 0, hi = 0;     // NIB: 4-bit counters since the last spread; 8-bit counters (even, odd experts)
  unsigned long long b_nib = 0, b_lo = 0, b_hi = 0;
  int tot = 0, before = 0;                        // !NIB
  bool snapped = false;                           // k = 1: the counters as they were when the walk reached this block
  for (int v0 = wave; v0 < nvec; v0 += NW * DISP1_ROUND) {
    int ev[DISP1_ROUND];
#pragma unroll
    for (int u = 0; u < DISP1_ROUND; ++u) {
      const int f = (v0 + u * NW) * 64 + lane;
      const int ee = expert_idx[f < n ? f : 0];    // (n > 0 here; entries past the end re-read entry 0)
      ev[u] = (f < n && ee >= 0 && ee < E) ? ee : -1;
    }
#pragma unroll
    for (int u = 0; u < DISP1_ROUND; ++u) {
      const int v = v0 + u * NW;
      if (v < nvec) {                              // wave-uniform
        bool early = false;                        // k > 1: this lane's item comes before the block
        if constexpr (K == 1) {
          if (v >= vb && !snapped) {
            snapped = true;
            b_nib = nib; b_lo = lo; b_hi = hi;
            before = tot;
          }
        } else {
          const int f = v * 64 + lane;
          early = (f % K) * T + f / K < i0;
        }
        if constexpr (NIB) {
          const unsigned long long inc = static_cast<unsigned long long>(ev[u] >= 0) << ((ev[u] & 15) * 4);
          nib += inc;
          if (K > 1) b_nib += early ? inc : 0ull;
        } else {
          unsigned long long same;
          tot += count64(ev[u], same);
          if (K > 1) before += count64(early ? ev[u] : -1, same);
        }
      }
      if (NIB && (u % 15 == 14 || u == DISP1_ROUND - 1)) {   // before a 4-bit counter can overflow
        lo += nib & M4;
        hi += (nib >> 4) & M4;
        nib = 0;
        if (K > 1) {
          b_lo += b_nib & M4;
          b_hi += (b_nib >> 4) & M4;
          b_nib = 0;
        }
      }
    }
  }
  if (K == 1 && !snapped) {                        // every vector of this wave lies before the block
    b_nib = 0; b_lo = lo; b_hi = hi;
    before = tot;
  }
  if constexpr (NIB) {
    b_lo += b_nib & M4;
    b_hi += (b_nib >> 4) & M4;
    cw[0][wave][lane][0] = static_cast<int>(lo); cw[0][wave][lane][1] = static_cast<int>(lo >> 32);
    cw[0][wave][lane][2] = static_cast<int>(hi); cw[0][wave][lane][3] = static_cast<int>(hi >> 32);
    cw[1][wave][lane][0] = static_cast<int>(b_lo); cw[1][wave][lane][1] = static_cast<int>(b_lo >> 32);
    cw[1][wave][lane][2] = static_cast<int>(b_hi); cw[1][wave][lane][3] = static_cast<int>(b_hi >> 32);
  } else {
    cw[0][wave][lane][0] = tot;
    cw[1][wave][lane][0] = before;
  }
  // this thread's own item
  const int i = (vb + wave) * 64 + lane;
  int t = i, j = 0, e = -1;
  if constexpr (K == 1) {
    if (i < n) e = expert_idx[i];
    if (e >= E) e = -1;
  } else {
    e = item_expert(expert_idx, i, n, T, k, E, &t, &j);
  }
  unsigned long long same;
  wown[wave][lane] = count64(e, same);
  const unsigned long long below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  const int rank = __popcll(same & below);
  __syncthreads();
  if constexpr (NIB) {
    if (wave < E) {                                // wave e adds up expert e: 16 waves x 64 lanes of 8-bit counters
      const int word = (wave & 1) * 2 + (wave >> 3), shift = ((wave >> 1) & 3) * 8;
      int st = 0, sb = 0;
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        st += (cw[0][w][lane][word] >> shift) & 255;
        sb += (cw[1][w][lane][word] >> shift) & 255;
      }
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) {
        st += __shfl_xor(st, off, 64);
        sb += __shfl_xor(sb, off, 64);
      }
      if (lane == 0) {
        tot_s[wave] = st;
        bef[wave] = sb;
      }
    }
    __syncthreads();
  }
  if (wave == 0) {
    int tt = 0, bb = 0;
    if constexpr (NIB) {
      tt = lane < E ? tot_s[lane] : 0;
    } else {
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        tt += cw[0][w][lane][0];
        bb += cw[1][w][lane][0];
      }
      bef[lane] = bb;
    }
    const int c = (lane < E) ? (tt < capacity ? tt : capacity) : 0;
    int incl = c;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int up = __shfl_up(incl, off, 64);
      if (lane >= off) incl += up;
    }
    seg[lane] = incl - c;
    if (blockIdx.x == 0 && lane < E) {
      counts[lane] = c;
      offsets[lane] = incl - c;
      if (lane == E - 1) offsets[E] = incl;
    }
  } else if (wave == 1) {
    int run = 0;                                   // exclusive prefix of the own-vector counts over the waves
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const int c = wown[w][lane];
      wown[w][lane] = run;
      run += c;
    }
  }
  __syncthreads();
  if (i < n) {
    int out = -1;
    if (e >= 0) {
      const int slot = bef[e] + wown[wave][e] + rank;
      if (slot < capacity) {
        out = seg[e] + slot;
        src_token[out] = t;
      }
    }
    dst_row[static_cast<int64_t>(t) * k + j] = out;
  }
}

// x_perm[r, :] = x[src_token[r], :], 16 bytes per lane, one wave per row, up to four pieces of a
// row per lane in flight.  The loads are unconditional (a lane past the end of the row re-reads
// its last piece and does not store): with loads under a condition the compiler kept the four
// pieces in LDS instead of registers.
__global__ __launch_bounds__(256) void gather_rows(const unsigned char* __restrict__ x, int64_t ldx_bytes,
                                                   const int32_t* __restrict__ src_token,
                                                   const int32_t* __restrict__ offsets, int E,
                                                   int row_bytes, unsigned char* __restrict__ x_perm,
                                                   int64_t ldp_bytes) {
  const int K = offsets[E];
  const int lane = threadIdx.x & 63;
  const int wave = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  const int nwaves = gridDim.x * (blockDim.x >> 6);
  const int last = row_bytes - 16;
  for (int r = wave; r < K; r += nwaves) {
    const int src = src_token[r];
    const unsigned char* s = x + static_cast<int64_t>(src) * ldx_bytes;
    unsigned char* q = x_perm + static_cast<int64_t>(r) * ldp_bytes;
    for (int c = lane * 16; c < row_bytes; c += 64 * 16 * 4) {
      const int c1 = c + 1024, c2 = c + 2048, c3 = c + 3072;
      const uint4 v0 = *reinterpret_cast<const uint4*>(s + c);
      const uint4 v1 = *reinterpret_cast<const uint4*>(s + (c1 < last ? c1 : last));
      const uint4 v2 = *reinterpret_cast<const uint4*>(s + (c2 < last ? c2 : last));
      const uint4 v3 = *reinterpret_cast<const uint4*>(s + (c3 < last ? c3 : last));
      *reinterpret_cast<uint4*>(q + c) = v0;
      if (c1 < row_bytes) *reinterpret_cast<uint4*>(q + c1) = v1;
      if (c2 < row_bytes) *reinterpret_cast<uint4*>(q + c2) = v2;
      if (c3 < row_bytes) *reinterpret_cast<uint4*>(q + c3) = v3;
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
  const int64_t items = static_cast<int64_t>(T) * k;
  if (items <= DISP1_MAX_ITEMS) {
    const int blocks = items > 0 ? static_cast<int>((items + DISP1_THREADS - 1) / DISP1_THREADS) : 1;
    const ScanChores sc = chores ? *chores : ScanChores{};
#define SCMOE_ONEPASS(NIB, K)                                                                                    \
  hipLaunchKernelGGL((dispatch_onepass<NIB, K>), dim3(blocks), dim3(DISP1_THREADS), 0, stream, expert_idx, T, E, \
                     capacity, counts, offsets, dst_row, src_token, sc)
    if (E <= 16) {
      switch (k) {
        case 1: SCMOE_ONEPASS(true, 1); break;
        case 2: SCMOE_ONEPASS(true, 2); break;
        case 3: SCMOE_ONEPASS(true, 3); break;
        default: SCMOE_ONEPASS(true, 4); break;
      }
    } else {
      switch (k) {
        case 1: SCMOE_ONEPASS(false, 1); break;
        case 2: SCMOE_ONEPASS(false, 2); break;
        case 3: SCMOE_ONEPASS(false, 3); break;
        default: SCMOE_ONEPASS(false, 4); break;
      }
    }
#undef SCMOE_ONEPASS
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
