// Stages 2-3 of Algorithm 1 (token counting, index generation) and the Stage-4
// gather, as an atomics-free stable counting sort:
//
//   count   every workgroup owns PERM_CHUNK consecutive (token, slot) pairs and
//           counts them per local expert; each wave counts its own quarter with
//           ballots (one pass per distinct expert in a 64-pair batch) into its
//           own LDS row, so there is no atomic anywhere.  -> block_hist[e][b]
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
constexpr int PERM_ITERS = 4;                                  // 64-pair batches per wave
constexpr int PERM_CHUNK = PERM_WAVES * PERM_ITERS * MOE_WAVE;  // pairs per workgroup

__device__ __forceinline__ uint64_t lanemask_lt() {
  const int lane = threadIdx.x % MOE_WAVE;
  return lane == 0 ? 0ull : (~0ull >> (64 - lane));
}

// Counts this wave's pairs per local expert into cnt[] (one LDS row per wave).
// le[it] receives the local expert id of the lane's pair in batch `it`, or -1.
__device__ __forceinline__ void count_wave(const int32_t* __restrict__ topk_idx, int n, int e_begin, int e_count,
                                           int first, int* cnt, int le[PERM_ITERS]) {
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
    uint64_t active = __ballot(e >= 0);
    while (active) {
      const int leader = __builtin_ctzll(active);
      const int e0 = __shfl(e, leader, MOE_WAVE);
      const uint64_t m = __ballot(e == e0);
      if (lane == leader) cnt[e0] += __builtin_popcountll(m);
      active &= ~m;
    }
  }
}

__global__ __launch_bounds__(PERM_THREADS) void permute_count_kernel(const int32_t* __restrict__ topk_idx, int n,
                                                                     int e_begin, int e_count, int nblocks,
                                                                     int32_t* __restrict__ block_hist) {
  __shared__ int wcnt[PERM_WAVES][MOE_MAX_EXPERTS];
  const int tid = threadIdx.x, w = tid / MOE_WAVE;
  for (int i = tid; i < PERM_WAVES * MOE_MAX_EXPERTS; i += PERM_THREADS) (&wcnt[0][0])[i] = 0;
  __syncthreads();
  int le[PERM_ITERS];
  count_wave(topk_idx, n, e_begin, e_count, blockIdx.x * PERM_CHUNK + w * PERM_ITERS * MOE_WAVE, wcnt[w], le);
  __syncthreads();
  for (int e = tid; e < e_count; e += PERM_THREADS) {
    int s = 0;
#pragma unroll
    for (int v = 0; v < PERM_WAVES; ++v) s += wcnt[v][e];
    block_hist[static_cast<size_t>(e) * nblocks + blockIdx.x] = s;
  }
}

// In-place exclusive scan of block_hist (length e_count*nblocks) by one workgroup.
__global__ __launch_bounds__(1024) void permute_scan_kernel(int32_t* __restrict__ block_hist, int e_count, int nblocks,
                                                            int32_t* __restrict__ expert_offsets) {
  __shared__ int sums[1024];
  const int tid = threadIdx.x;
  const int N = e_count * nblocks;
  const int per = (N + 1023) / 1024;
  const int lo = tid * per, hi = min(N, lo + per);
  int s = 0;
  for (int i = lo; i < hi; ++i) s += block_hist[i];
  sums[tid] = s;
  __syncthreads();
  // Hillis-Steele inclusive scan over the 1024 partial sums
  for (int off = 1; off < 1024; off <<= 1) {
    int v = tid >= off ? sums[tid - off] : 0;
    __syncthreads();
    sums[tid] += v;
    __syncthreads();
  }
  int run = sums[tid] - s;  // exclusive prefix of this thread's segment
  for (int i = lo; i < hi; ++i) {
    const int c = block_hist[i];
    block_hist[i] = run;
    if (i % nblocks == 0) expert_offsets[i / nblocks] = run;
    run += c;
  }
  if (tid == 1023) expert_offsets[e_count] = sums[1023];
}

__global__ __launch_bounds__(PERM_THREADS) void permute_place_kernel(const int32_t* __restrict__ topk_idx, int n, int k,
                                                                     int e_begin, int e_count, int nblocks,
                                                                     const int32_t* __restrict__ block_base,
                                                                     int32_t* __restrict__ row_token,
                                                                     int32_t* __restrict__ slot_row) {
  __shared__ int wcnt[PERM_WAVES][MOE_MAX_EXPERTS];
  const int tid = threadIdx.x, w = tid / MOE_WAVE, lane = tid % MOE_WAVE;
  for (int i = tid; i < PERM_WAVES * MOE_MAX_EXPERTS; i += PERM_THREADS) (&wcnt[0][0])[i] = 0;
  __syncthreads();
  int le[PERM_ITERS];
  const int first = blockIdx.x * PERM_CHUNK + w * PERM_ITERS * MOE_WAVE;
  count_wave(topk_idx, n, e_begin, e_count, first, wcnt[w], le);
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
    uint64_t active = __ballot(e >= 0);
    while (active) {
      const int leader = __builtin_ctzll(active);
      const int e0 = __shfl(e, leader, MOE_WAVE);
      const uint64_t m = __ballot(e == e0);
      const int base = next[e0];
      __builtin_amdgcn_wave_barrier();
      if (e == e0) row = base + __builtin_popcountll(m & lt);
      if (lane == leader) next[e0] = base + __builtin_popcountll(m);
      __builtin_amdgcn_wave_barrier();
      active &= ~m;
    }
    if (idx < n) {
      slot_row[idx] = row;
      if (row >= 0) row_token[row] = idx / k;
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
  return (cells * sizeof(int32_t) + 255) & ~static_cast<size_t>(255);
}

extern "C" int moe_permute(const moe_bf16* x, const int32_t* topk_idx, int T, int d, int E_total, int k, int e_begin,
                           int e_count, int32_t* expert_offsets, int32_t* row_token, int32_t* slot_row, moe_bf16* xp,
                           void* ws, size_t ws_bytes, void* stream) {
  if (!x || !topk_idx || !expert_offsets || !row_token || !slot_row || !xp || !ws) return MOE_ERR_INVALID;
  if (T <= 0 || d <= 0 || d % 8 != 0 || E_total <= 0 || k <= 0 || k > E_total) return MOE_ERR_INVALID;
  if (e_begin < 0 || e_count <= 0 || e_begin + e_count > E_total || e_count > MOE_MAX_EXPERTS) return MOE_ERR_INVALID;
  if (static_cast<long long>(T) * k > 0x7FFFFFFFll / 2) return MOE_ERR_INVALID;
  if (!moe_aligned16(x) || !moe_aligned16(xp) || !moe_aligned16(ws) || !moe_aligned16(topk_idx) ||
      !moe_aligned16(slot_row) || !moe_aligned16(row_token) || !moe_aligned16(expert_offsets))
    return MOE_ERR_INVALID;
  if (ws_bytes < moe_permute_workspace_bytes(T, k, e_count)) return MOE_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int n = T * k, nb = perm_blocks(T, k);
  int32_t* block_hist = static_cast<int32_t*>(ws);
  MOE_LAUNCH("permute_count", permute_count_kernel, dim3(nb), dim3(PERM_THREADS), 0, s, topk_idx, n, e_begin, e_count,
             nb, block_hist);
  MOE_LAUNCH("permute_scan", permute_scan_kernel, dim3(1), dim3(1024), 0, s, block_hist, e_count, nb, expert_offsets);
  MOE_LAUNCH("permute_place", permute_place_kernel, dim3(nb), dim3(PERM_THREADS), 0, s, topk_idx, n, k, e_begin,
             e_count, nb, static_cast<const int32_t*>(block_hist), row_token, slot_row);
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
