// Pieces that the routing kernel and the index-generation kernels share: how a run of (token, slot)
// pairs is cut into chunks, and how a wave counts a batch of 64 pairs per local expert without atomics.
#pragma once
#include "common.h"

constexpr int PERM_THREADS = 256;
constexpr int PERM_WAVES = PERM_THREADS / MOE_WAVE;

// Pairs of a chunk that wave w owns: the chunk is cut into PERM_WAVES runs of whole 64-pair batches,
// in order, so that wave order is pair order.
__device__ __forceinline__ int perm_wave_span(int chunk) {
  return ((chunk + PERM_WAVES * MOE_WAVE - 1) / (PERM_WAVES * MOE_WAVE)) * MOE_WAVE;
}

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

// Adds this wave's share of a chunk to cnt[] (the wave's own LDS row): local(i) is the local expert
// of the chunk's pair i, or -1.  The lowest lane of every group of equal experts adds the group's
// size: one writer per expert and batch, no atomic.
template <typename Local>
__device__ __forceinline__ void count_wave_span(int chunk, int nbits, int* cnt, Local local) {
  const int lane = threadIdx.x % MOE_WAVE, w = threadIdx.x / MOE_WAVE;
  const int span = perm_wave_span(chunk);
  const int lo = w * span, hi = min(chunk, lo + span);
  for (int first = lo; first < hi; first += MOE_WAVE) {
    const int i = first + lane;
    const int e = i < hi ? local(i) : -1;
    const uint64_t m = same_expert_mask(e, nbits);
    if (m != 0 && lane == __builtin_ctzll(m)) cnt[e] += __builtin_popcountll(m);
    __builtin_amdgcn_wave_barrier();
  }
}

// Most rows the [chunk][expert] table may have.  Every placing workgroup sums all of them, so the table is
// kept near 16384 cells (64 KB); with few local experts that allows many short chunks (one routing pass
// each), with many experts no fewer than 256 (128 beyond 128 experts) however large the table gets.
inline int perm_max_chunks(int e_count) {
  if (e_count > 128) return 128;
  const int by_cells = 16384 / e_count;
  return by_cells < 256 ? 256 : (by_cells > 4096 ? 4096 : by_cells);
}

// Launches Stage 1 with the per-chunk expert counts as a by-product (route.hip); hist has room for hist_cells
// counts.  Returns false if the shape does not fit the fused kernel (the caller then routes and counts with
// two launches).
bool moe_launch_route_count(const float* logits, int T, int E, int k, int renormalize, int e_begin, int e_count,
                            int nbits, int32_t* topk_idx, float* topk_w, int32_t* hist, size_t hist_cells, int* chunk,
                            int* nblocks, hipStream_t s);
