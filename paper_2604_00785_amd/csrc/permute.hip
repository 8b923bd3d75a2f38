// Stages 2-3 of Algorithm 1 (token counting, index generation) and the Stage-4
// gather, as an atomics-free stable counting sort:
//
//   count   every workgroup owns PERM_CHUNK consecutive (token, slot) pairs and
//           counts them per local expert; each wave finds, with one ballot per
//           bit of the expert id, the lanes of a 64-pair batch that chose the
//           same expert, and the lowest lane of each such group adds the group
//           size to the wave's own LDS row: no atomic anywhere.  -> block_hist[e][b]
//   scan    one workgroup turns block_hist, read in expert-major order, into
//           exclusive prefix sums: the first row of every (expert, workgroup)
//           cell, and expert_offsets.  This is the paper's
//           partial_cum_token_counts / cum_token_counts at workgroup granularity.
//   place   every workgroup recounts its pairs, derives each wave's first row
//           per expert, and ranks pairs inside a batch by the popcount of the
//           lower lanes that chose the same expert -> slot_row, row_token.
//   rows    one wave per token copies x[t] to its (up to k) grouped rows with
//           16-byte accesses: x is read once, xp is written in full rows.
#include "common.h"

namespace {

constexpr int PERM_THREADS = 256;
constexpr int PERM_WAVES = PERM_THREADS / MOE_WAVE;
constexpr int PERM_ITERS = 1;                                  // 64-pair batches per wave
constexpr int PERM_CHUNK = PERM_WAVES * PERM_ITERS * MOE_WAVE;  // pairs per workgroup

__device__ __forceinline__ uint64_t lanemask_lt() {
  const int lane = threadIdx.x % MOE_WAVE;
  return lane == 0 ? 0ull : (~0ull >> (64 - lane));
}

// For every lane, the mask of lanes of its 64-pair batch that chose the same local expert: the
// AND over the bits of the expert id of "lanes whose bit equals mine" (one ballot per bit, so
// log2(e_count) steps whatever the number of distinct experts).  Lanes with e < 0 get 0.
__device__ __forceinline__ uint64_t same_expert_mask(int e, int nbits) {
  uint64_t m = __ballot(e >= 0);
  for (int b = 0; b < nbits; ++b) {
    const uint64_t set = __ballot((e >> b) & 1);
    m &= ((e >> b) & 1) ? set : ~set;
  }
  return e >= 0 ? m : 0ull;
}

// Counts this wave's pairs per local expert into cnt[] (one LDS row per wave).
// le[it] receives the local expert id of the lane's pair in batch `it`, or -1.
__device__ __forceinline__ void count_wave(const int32_t* __restrict__ topk_idx, int n, int e_begin, int e_count,
                                           int nbits, int first, int* cnt, int le[PERM_ITERS]) {
  const int lane = threadIdx.x % MOE_WAVE;
#pragma unroll
  for (int it = 0; it < PERM_ITERS; ++it) {
    const int idx = first + it * MOE_WAVE + lane;
    int e = -1;
    if (idx < n) {
      e = topk_idx[idx] - e_begin;
      if (e < 0 || e >= e_count) e = -1;
    }
    le[it] = e;
    const uint64_t m = same_expert_mask(e, nbits);
    // the lowest lane of every group adds the group's size: one writer per expert and batch
    if (m != 0 && lane == __builtin_ctzll(m)) cnt[e] += __builtin_popcountll(m);
    __builtin_amdgcn_wave_barrier();
  }
}

__global__ __launch_bounds__(PERM_THREADS) void permute_count_kernel(const int32_t* __restrict__ topk_idx, int n,
                                                                     int e_begin, int e_count, int nbits, int nblocks,
                                                                     int32_t* __restrict__ block_hist) {
  __shared__ int wcnt[PERM_WAVES][MOE_MAX_EXPERTS];
  const int tid = threadIdx.x, w = tid / MOE_WAVE;
  for (int e = tid; e < e_count; e += PERM_THREADS) {
#pragma unroll
    for (int v = 0; v < PERM_WAVES; ++v) wcnt[v][e] = 0;
  }
  __syncthreads();
  int le[PERM_ITERS];
  count_wave(topk_idx, n, e_begin, e_count, nbits, blockIdx.x * PERM_CHUNK + w * PERM_ITERS * MOE_WAVE, wcnt[w], le);
  __syncthreads();
  for (int e = tid; e < e_count; e += PERM_THREADS) {
    int s = 0;
#pragma unroll
    for (int v = 0; v < PERM_WAVES; ++v) s += wcnt[v][e];
    block_hist[static_cast<size_t>(e) * nblocks + blockIdx.x] = s;
  }
}

// In-place exclusive scan of block_hist (length e_count*nblocks, padded to a multiple of 4 by the
// workspace rounding) by one workgroup of 1024 threads: 4096 elements per sweep with 16-byte
// accesses, a shuffle scan inside each wave, the 16 wave totals through LDS, a running carry.
__global__ __launch_bounds__(1024) void permute_scan_kernel(int32_t* __restrict__ block_hist, int e_count, int nblocks,
                                                            int32_t* __restrict__ expert_offsets) {
  __shared__ int wsum[16];
  const int tid = threadIdx.x, lane = tid % MOE_WAVE, w = tid / MOE_WAVE;
  const int N = e_count * nblocks;
  int carry = 0;
  for (int base = 0; base < N; base += 4096) {
    const int i = base + tid * 4;
    int4 v = make_int4(0, 0, 0, 0);
    if (i < N) v = *reinterpret_cast<const int4*>(block_hist + i);
    if (i + 1 >= N) v.y = 0;
    if (i + 2 >= N) v.z = 0;
    if (i + 3 >= N) v.w = 0;
    const int s = v.x + v.y + v.z + v.w;
    int inc = s;
#pragma unroll
    for (int d = 1; d < MOE_WAVE; d <<= 1) {
      const int o = __shfl_up(inc, d, MOE_WAVE);
      if (lane >= d) inc += o;
    }
    if (lane == MOE_WAVE - 1) wsum[w] = inc;
    __syncthreads();
    int before = 0, total = 0;
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int t = wsum[q];
      if (q < w) before += t;
      total += t;
    }
    __syncthreads();
    int4 o;
    o.x = carry + before + inc - s;
    o.y = o.x + v.x;
    o.z = o.y + v.y;
    o.w = o.z + v.z;
    if (i < N) {
      *reinterpret_cast<int4*>(block_hist + i) = o;
      const int r[4] = {o.x, o.y, o.z, o.w};
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (i + j < N && (i + j) % nblocks == 0) expert_offsets[(i + j) / nblocks] = r[j];
    }
    carry += total;
  }
  if (tid == 0) expert_offsets[e_count] = carry;
}

__global__ __launch_bounds__(PERM_THREADS) void permute_place_kernel(const int32_t* __restrict__ topk_idx, int n, int k,
                                                                     int e_begin, int e_count, int nbits, int nblocks,
                                                                     const int32_t* __restrict__ block_base,
                                                                     int32_t* __restrict__ row_token,
                                                                     int32_t* __restrict__ slot_row,
                                                                     const float* __restrict__ topk_w,
                                                                     float* __restrict__ row_weight) {
  __shared__ int wcnt[PERM_WAVES][MOE_MAX_EXPERTS];
  const int tid = threadIdx.x, w = tid / MOE_WAVE, lane = tid % MOE_WAVE;
  for (int e = tid; e < e_count; e += PERM_THREADS) {
#pragma unroll
    for (int v = 0; v < PERM_WAVES; ++v) wcnt[v][e] = 0;
  }
  __syncthreads();
  int le[PERM_ITERS];
  const int first = blockIdx.x * PERM_CHUNK + w * PERM_ITERS * MOE_WAVE;
  count_wave(topk_idx, n, e_begin, e_count, nbits, first, wcnt[w], le);
  __syncthreads();
  // counts -> first row of each wave for each expert
  for (int e = tid; e < e_count; e += PERM_THREADS) {
    int base = block_base[static_cast<size_t>(e) * nblocks + blockIdx.x];
#pragma unroll
    for (int v = 0; v < PERM_WAVES; ++v) {
      const int c = wcnt[v][e];
      wcnt[v][e] = base;
      base += c;
    }
  }
  __syncthreads();
  int* next = wcnt[w];
  const uint64_t lt = lanemask_lt();
#pragma unroll
  for (int it = 0; it < PERM_ITERS; ++it) {
    const int idx = first + it * MOE_WAVE + lane;
    const int e = le[it];
    int row = -1;
    const uint64_t m = same_expert_mask(e, nbits);
    if (m != 0) {
      const int base = next[e];                      // every lane of the group reads the same counter
      row = base + __builtin_popcountll(m & lt);
      __builtin_amdgcn_wave_barrier();
      if (lane == __builtin_ctzll(m)) next[e] = base + __builtin_popcountll(m);
    }
    __builtin_amdgcn_wave_barrier();
    if (idx < n) {
      slot_row[idx] = row;
      if (row >= 0) {
        row_token[row] = idx / k;
        if (row_weight != nullptr) row_weight[row] = topk_w[idx];   // the row's gate weight, for callers that fold it into h
      }
    }
  }
}

// xp[slot_row[t,i]] = x[t] for every local slot; one wave per token.
template <int VPT>
__global__ __launch_bounds__(256) void permute_rows_kernel(const uint4* __restrict__ x, const int32_t* __restrict__ slot_row,
                                                           int T, int k, int chunks /* d/8 */, uint4* __restrict__ xp) {
  const int lane = threadIdx.x % MOE_WAVE;
  const int t = blockIdx.x * (256 / MOE_WAVE) + threadIdx.x / MOE_WAVE;
  if (t >= T) return;
  const uint4* src = x + static_cast<size_t>(t) * chunks;
  for (int c0 = 0; c0 < chunks; c0 += MOE_WAVE * VPT) {
    uint4 v[VPT];
#pragma unroll
    for (int j = 0; j < VPT; ++j) {
      const int c = c0 + j * MOE_WAVE + lane;
      if (c < chunks) v[j] = src[c];
    }
    for (int i = 0; i < k; ++i) {
      const int row = slot_row[static_cast<size_t>(t) * k + i];
      if (row < 0) continue;
      uint4* dst = xp + static_cast<size_t>(row) * chunks;
#pragma unroll
      for (int j = 0; j < VPT; ++j) {
        const int c = c0 + j * MOE_WAVE + lane;
        if (c < chunks) dst[c] = v[j];
      }
    }
  }
}

inline int perm_blocks(int T, int k) {
  const long long n = static_cast<long long>(T) * k;
  return static_cast<int>((n + PERM_CHUNK - 1) / PERM_CHUNK);
}

}  // namespace

extern "C" size_t moe_permute_workspace_bytes(int T, int k, int e_count) {
  if (T <= 0 || k <= 0 || e_count <= 0) return 0;
  const size_t cells = static_cast<size_t>(e_count) * perm_blocks(T, k);
  return (cells * sizeof(int32_t) + 16 + 255) & ~static_cast<size_t>(255);   // + one 16-byte access of slack
}

namespace {
int permute_impl(const moe_bf16* x, const int32_t* topk_idx, const float* topk_w, int T, int d, int E_total, int k,
                 int e_begin, int e_count, int32_t* expert_offsets, int32_t* row_token, int32_t* slot_row,
                 float* row_weight, moe_bf16* xp, void* ws, size_t ws_bytes, void* stream) {
  // xp == NULL: index generation only (for callers that let the GEMMs gather the rows); x is not read then
  if (!topk_idx || !expert_offsets || !row_token || !slot_row || !ws || (xp && !x)) return MOE_ERR_INVALID;
  if (T <= 0 || d <= 0 || d % 8 != 0 || E_total <= 0 || k <= 0 || k > E_total) return MOE_ERR_INVALID;
  if (e_begin < 0 || e_count <= 0 || e_begin + e_count > E_total || e_count > MOE_MAX_EXPERTS) return MOE_ERR_INVALID;
  if (static_cast<long long>(T) * k > 0x7FFFFFFFll / 2) return MOE_ERR_INVALID;
  if ((xp && (!moe_aligned16(x) || !moe_aligned16(xp))) || !moe_aligned16(ws) || !moe_aligned16(topk_idx) ||
      !moe_aligned16(slot_row) || !moe_aligned16(row_token) || !moe_aligned16(expert_offsets))
    return MOE_ERR_INVALID;
  if (ws_bytes < moe_permute_workspace_bytes(T, k, e_count)) return MOE_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int n = T * k, nb = perm_blocks(T, k);
  int nbits = 0;
  while ((1 << nbits) < e_count) ++nbits;
  int32_t* block_hist = static_cast<int32_t*>(ws);
  MOE_LAUNCH("permute_count", permute_count_kernel, dim3(nb), dim3(PERM_THREADS), 0, s, topk_idx, n, e_begin, e_count,
             nbits, nb, block_hist);
  MOE_LAUNCH("permute_scan", permute_scan_kernel, dim3(1), dim3(1024), 0, s, block_hist, e_count, nb, expert_offsets);
  MOE_LAUNCH("permute_place", permute_place_kernel, dim3(nb), dim3(PERM_THREADS), 0, s, topk_idx, n, k, e_begin,
             e_count, nbits, nb, static_cast<const int32_t*>(block_hist), row_token, slot_row, topk_w, row_weight);
  if (!xp) return moe_check_launch();
  const int chunks = d / 8;
  dim3 grid((T + 3) / 4), block(256);
  const uint4* xs = reinterpret_cast<const uint4*>(x);
  uint4* xd = reinterpret_cast<uint4*>(xp);
  if (chunks <= 64)
    MOE_LAUNCH("permute_rows", permute_rows_kernel<1>, grid, block, 0, s, xs, static_cast<const int32_t*>(slot_row), T, k, chunks, xd);
  else if (chunks <= 128)
    MOE_LAUNCH("permute_rows", permute_rows_kernel<2>, grid, block, 0, s, xs, static_cast<const int32_t*>(slot_row), T, k, chunks, xd);
  else
    MOE_LAUNCH("permute_rows", permute_rows_kernel<4>, grid, block, 0, s, xs, static_cast<const int32_t*>(slot_row), T, k, chunks, xd);
  return moe_check_launch();
}
}  // namespace

extern "C" int moe_permute(const moe_bf16* x, const int32_t* topk_idx, int T, int d, int E_total, int k, int e_begin,
                           int e_count, int32_t* expert_offsets, int32_t* row_token, int32_t* slot_row, moe_bf16* xp,
                           void* ws, size_t ws_bytes, void* stream) {
  return permute_impl(x, topk_idx, nullptr, T, d, E_total, k, e_begin, e_count, expert_offsets, row_token, slot_row,
                      nullptr, xp, ws, ws_bytes, stream);
}

extern "C" int moe_permute_gate(const int32_t* topk_idx, const float* topk_w, int T, int E_total, int k, int e_begin,
                                int e_count, int32_t* expert_offsets, int32_t* row_token, int32_t* slot_row,
                                float* row_weight, void* ws, size_t ws_bytes, void* stream) {
  if (!topk_w || !row_weight || !moe_aligned16(topk_w) || !moe_aligned16(row_weight)) return MOE_ERR_INVALID;
  return permute_impl(nullptr, topk_idx, topk_w, T, 8, E_total, k, e_begin, e_count, expert_offsets, row_token,
                      slot_row, row_weight, nullptr, ws, ws_bytes, stream);
}

// ---------------------------------------------------------------------------------------------
// moe_permute for callers that cannot provide a workspace: the [expert][workgroup] histogram table
// lives in a device array that is part of the library image (every GPU the library runs on holds
// its own copy until the process ends).
namespace {
constexpr size_t STATIC_WS_BYTES = 1u << 20;       // 262144 table cells (the headline shape needs 16384)
static __device__ __align__(256) unsigned char scratch[STATIC_WS_BYTES];

constexpr int STATIC_WS_MAX_DEVICES = 64;
void* g_scratch_addr[STATIC_WS_MAX_DEVICES];        // device address of `scratch` on each device, once looked up

// Device address of this device's copy of `scratch` (the array's name is only a host-side handle).
// Looked up on the first call on a device, with that device current; concurrent first calls store
// the same value.
void* scratch_address() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= STATIC_WS_MAX_DEVICES) {
    (void)hipGetLastError();
    return nullptr;
  }
  void* p = __atomic_load_n(&g_scratch_addr[dev], __ATOMIC_ACQUIRE);
  if (p != nullptr) return p;
  if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
    (void)hipGetLastError();
    return nullptr;
  }
  __atomic_store_n(&g_scratch_addr[dev], p, __ATOMIC_RELEASE);
  return p;
}
}  // namespace

extern "C" size_t moe_permute_static_ws_capacity(void) { return STATIC_WS_BYTES; }

extern "C" int moe_permute_static_ws(const moe_bf16* x, const int32_t* topk_idx, int T, int d, int E_total, int k,
                                     int e_begin, int e_count, int32_t* expert_offsets, int32_t* row_token,
                                     int32_t* slot_row, moe_bf16* xp, void* stream) {
  // sizes first: a shape whose table does not fit is refused before anything else is looked at
  if (T <= 0 || k <= 0 || e_count <= 0 || e_count > MOE_MAX_EXPERTS) return MOE_ERR_INVALID;
  if (static_cast<long long>(T) * k > 0x7FFFFFFFll / 2) return MOE_ERR_INVALID;
  if (moe_permute_workspace_bytes(T, k, e_count) > STATIC_WS_BYTES) return MOE_ERR_WORKSPACE;
  void* ws = scratch_address();
  if (ws == nullptr) return MOE_ERR_LAUNCH;
  // every table cell the scan reads is written by the counting kernel of the same call first, so
  // nothing has to be cleared between calls
  return permute_impl(x, topk_idx, nullptr, T, d, E_total, k, e_begin, e_count, expert_offsets, row_token, slot_row,
                      nullptr, xp, ws, STATIC_WS_BYTES, stream);
}
