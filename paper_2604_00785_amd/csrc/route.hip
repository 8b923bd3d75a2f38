// Stage 1 of Algorithm 1: Softmax over the experts, then TopK.
//
// A group of G lanes (G a power of two, 8..64) owns one token and keeps
// ceil(E/G) logits per lane in registers.  Selection runs on the logits (the
// softmax is monotone): each logit becomes a 64-bit key
//   (order-preserving image of the fp32 value) << 32 | (0xFFFFFFFF - expert)
// so that an unsigned maximum picks the largest value and, among equal values,
// the lowest expert id.  k rounds of a butterfly maximum over the group pick the
// k winners; the owner of a winner retires its key.  Gates are exp(l - max)
// divided by the sum over all experts, or over the winners when renormalising.
//
// When the index generation of Stages 2-3 follows in the same call, a workgroup routes a chunk of
// tokens (one or more passes of 256 / G tokens) and counts its winners per local expert straight from
// the registers that hold them: the [chunk][expert] table of the counting sort is then a by-product
// of the routing and the pairs need not be read back for it.
#include "perm_common.h"

namespace {

__device__ __forceinline__ uint32_t ordered_bits(float v) {
  v += 0.0f;  // -0.0 -> +0.0 so the two zeros tie
  uint32_t u = __float_as_uint(v);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ uint64_t shfl_xor_u64(uint64_t v, int mask) {
  uint32_t lo = static_cast<uint32_t>(v), hi = static_cast<uint32_t>(v >> 32);
  lo = __shfl_xor(lo, mask, MOE_WAVE);
  hi = __shfl_xor(hi, mask, MOE_WAVE);
  return (static_cast<uint64_t>(hi) << 32) | lo;
}

// The maximum of a 64-bit key over a group of G lanes, in every lane of the group.  Partners inside a row
// of 16 lanes come through DPP lane permutations (no LDS round trip): neighbour, other pair of the quad,
// then the mirrored lane of the 8- and 16-lane halves (by then all lanes of the smaller unit agree, so the
// mirror is as good as the XOR partner); beyond a row, through the crossbar.
template <int CTRL> __device__ __forceinline__ uint64_t dpp_u64(uint64_t v) {
  const int lo = __builtin_amdgcn_update_dpp(0, static_cast<int>(static_cast<uint32_t>(v)), CTRL, 0xF, 0xF, false);
  const int hi = __builtin_amdgcn_update_dpp(0, static_cast<int>(static_cast<uint32_t>(v >> 32)), CTRL, 0xF, 0xF, false);
  return (static_cast<uint64_t>(static_cast<uint32_t>(hi)) << 32) | static_cast<uint32_t>(lo);
}
template <int G> __device__ __forceinline__ uint64_t group_max_u64(uint64_t best) {
  auto take = [&](uint64_t o) { best = o > best ? o : best; };
  if constexpr (G >= 2) take(dpp_u64<0xB1>(best));     // quad_perm [1,0,3,2]
  if constexpr (G >= 4) take(dpp_u64<0x4E>(best));     // quad_perm [2,3,0,1]
  if constexpr (G >= 8) take(dpp_u64<0x141>(best));    // row_half_mirror
  if constexpr (G >= 16) take(dpp_u64<0x140>(best));   // row_mirror
  if constexpr (G >= 32) take(shfl_xor_u64(best, 16));
  if constexpr (G >= 64) take(shfl_xor_u64(best, 32));
  return best;
}

// COUNT: also write hist[blockIdx.x][local expert] = winners of this workgroup's tokens per local expert.
template <int G, int VPL, bool COUNT>
__global__ __launch_bounds__(256) void route_kernel(const float* __restrict__ logits, int T, int E, int k,
                                                    int renormalize, int32_t* __restrict__ topk_idx,
                                                    float* __restrict__ topk_w, int passes, int e_begin, int e_count,
                                                    int nbits, int32_t* __restrict__ hist) {
  constexpr int GROUPS_PER_BLOCK = 256 / G;
  __shared__ int wcnt[COUNT ? PERM_WAVES : 1][COUNT ? MOE_MAX_EXPERTS : 1];   // per wave: winners per local expert
  const int tid = threadIdx.x;
  const int gl = tid % G;  // lane inside the group
  if constexpr (COUNT) {
    for (int e = tid; e < e_count; e += 256) {
#pragma unroll
      for (int v = 0; v < PERM_WAVES; ++v) wcnt[v][e] = 0;
    }
    __syncthreads();
  }

  auto load_row = [&](int pass, float (&val)[VPL]) {
    const int t = (blockIdx.x * passes + pass) * GROUPS_PER_BLOCK + tid / G;
    const int tt = t < T ? t : T - 1;  // idle groups shadow the last token and store nothing
#pragma unroll
    for (int j = 0; j < VPL; ++j) {
      const int e = gl + j * G;
      val[j] = e < E ? logits[static_cast<size_t>(tt) * E + e] : 0.f;
    }
  };
  float nxt[VPL];
  load_row(0, nxt);

  for (int pass = 0; pass < passes; ++pass) {
    const int t = (blockIdx.x * passes + pass) * GROUPS_PER_BLOCK + tid / G;
    const bool live = t < T;
    uint64_t key[VPL];
    float val[VPL];
#pragma unroll
    for (int j = 0; j < VPL; ++j) {
      const int e = gl + j * G;
      val[j] = nxt[j];
      // padding keys lie below every real key (real keys have a non-zero low word or high bit)
      key[j] = e < E ? (static_cast<uint64_t>(ordered_bits(val[j])) << 32) | (0xFFFFFFFFu - static_cast<uint32_t>(e)) : 0;
    }
    if (pass + 1 < passes) load_row(pass + 1, nxt);   // the next pass's logits arrive during this pass's selection

    // full-softmax denominator pieces need the row maximum, which is winner 0
    int my_idx[VPL];   // winner i is kept by lane i % G in slot i / G
    float my_val[VPL];
#pragma unroll
    for (int j = 0; j < VPL; ++j) { my_idx[j] = 0; my_val[j] = 0.f; }
    float row_max = 0.f;

    for (int i = 0; i < k; ++i) {
      uint64_t best = key[0];
#pragma unroll
      for (int j = 1; j < VPL; ++j) best = key[j] > best ? key[j] : best;
      best = group_max_u64<G>(best);
      const int e = static_cast<int>(0xFFFFFFFFu - static_cast<uint32_t>(best));
      // the owner retires the key and publishes the value
      float v = 0.f;
#pragma unroll
      for (int j = 0; j < VPL; ++j) {
        if (gl + j * G == e) { v = val[j]; key[j] = 0; }
      }
      // exactly one lane of the group holds v != 0-initialised; share it
      const int owner = e % G;
      v = __shfl(v, (tid / G) * G % MOE_WAVE + owner, MOE_WAVE);
      if (i == 0) row_max = v;
      if (gl == i % G) {
#pragma unroll
        for (int j = 0; j < VPL; ++j)
          if (j == i / G) { my_idx[j] = e; my_val[j] = v; }
      }
    }

    // denominator
    float part = 0.f;
    if (renormalize) {
#pragma unroll
      for (int j = 0; j < VPL; ++j)
        if (gl + j * G < k) part += expf(my_val[j] - row_max);
    } else {
#pragma unroll
      for (int j = 0; j < VPL; ++j)
        if (gl + j * G < E) part += expf(val[j] - row_max);
    }
#pragma unroll
    for (int m = 1; m < G; m <<= 1) part += __shfl_xor(part, m, MOE_WAVE);
    const float inv = 1.0f / part;

#pragma unroll
    for (int j = 0; j < VPL; ++j) {
      const int i = gl + j * G;
      if (i < k) {
        if (live) {
          topk_idx[static_cast<size_t>(t) * k + i] = my_idx[j];
          topk_w[static_cast<size_t>(t) * k + i] = expf(my_val[j] - row_max) * inv;
        }
      }
    }
    if constexpr (COUNT) {
      // The winners are counted where they are: slot j of the wave's lanes is one batch of up to 64 pairs (lane gl
      // of a group holds winner gl + j G), counted with the ballots of the counting sort; the lowest lane of every
      // group of equal experts adds the group's size to the wave's own LDS row.
      int* cnt = wcnt[tid / MOE_WAVE];
      const int lane = tid % MOE_WAVE;
#pragma unroll
      for (int j = 0; j < VPL; ++j) {
        if (j * G < k) {   // uniform: some lane holds a winner in this slot
          int le = (live && gl + j * G < k) ? my_idx[j] - e_begin : -1;
          if (le < 0 || le >= e_count) le = -1;
          const uint64_t m = same_expert_mask(le, nbits);
          if (m != 0 && lane == __builtin_ctzll(m)) cnt[le] += __builtin_popcountll(m);
          __builtin_amdgcn_wave_barrier();
        }
      }
    }
  }

  if constexpr (COUNT) {
    __syncthreads();
    for (int e = tid; e < e_count; e += 256) {
      int s = 0;
#pragma unroll
      for (int v = 0; v < PERM_WAVES; ++v) s += wcnt[v][e];
      hist[static_cast<size_t>(blockIdx.x) * e_count + e] = s;
    }
  }
}

template <int G, int VPL>
void launch_route(const float* logits, int T, int E, int k, int renorm, int32_t* idx, float* w, hipStream_t s) {
  const int groups = 256 / G;
  dim3 grid((T + groups - 1) / groups), block(256);
  MOE_LAUNCH("route", (route_kernel<G, VPL, false>), grid, block, 0, s, logits, T, E, k, renorm, idx, w, 1, 0, 0, 0,
             static_cast<int32_t*>(nullptr));
}

// Tokens per workgroup: whole passes of 256 / G tokens; as few passes as keep the chunks at perm_max_chunks
// or fewer and the [chunk][expert] table inside the workspace the caller gave (a workspace of the minimum
// size holds one table row per 256 pairs, which can mean several passes when k is small).
template <int G, int VPL>
bool launch_route_count(const float* logits, int T, int E, int k, int renorm, int e_begin, int e_count, int nbits,
                        int32_t* idx, float* w, int32_t* hist, size_t hist_cells, int* chunk, int* nblocks, hipStream_t s) {
  const int groups = 256 / G;
  const long long rows_fit = static_cast<long long>(hist_cells / static_cast<size_t>(e_count));
  const long long max_chunks = rows_fit < perm_max_chunks(e_count) ? rows_fit : perm_max_chunks(e_count);
  if (max_chunks < 1) return false;
  const long long cap = groups * max_chunks;
  const int passes = static_cast<int>((T + cap - 1) / cap);
  if (static_cast<long long>(passes) * groups * k > 0x3FFFFFFF) return false;
  const int tokens = passes * groups;
  *chunk = tokens * k;
  *nblocks = (T + tokens - 1) / tokens;
  MOE_LAUNCH("route_count", (route_kernel<G, VPL, true>), dim3(*nblocks), dim3(256), 0, s, logits, T, E, k, renorm, idx, w,
             passes, e_begin, e_count, nbits, hist);
  return true;
}

}  // namespace

bool moe_launch_route_count(const float* logits, int T, int E, int k, int renormalize, int e_begin, int e_count,
                            int nbits, int32_t* topk_idx, float* topk_w, int32_t* hist, size_t hist_cells, int* chunk,
                            int* nblocks, hipStream_t s) {
  if (E > MOE_MAX_EXPERTS) return false;
#define MOE_ROUTE_COUNT(G, VPL) \
  launch_route_count<G, VPL>(logits, T, E, k, renormalize, e_begin, e_count, nbits, topk_idx, topk_w, hist, hist_cells, chunk, \
                             nblocks, s)
  // eight logits per lane where the expert count allows: twice the tokens per pass of the plain launch, so
  // that one pass already fills a chunk at the usual shapes (a second pass would run after the first)
  if (E <= 8) return MOE_ROUTE_COUNT(8, 1);
  if (E <= 16) return MOE_ROUTE_COUNT(8, 2);
  if (E <= 32) return MOE_ROUTE_COUNT(8, 4);
  if (E <= 64) return MOE_ROUTE_COUNT(8, 8);
  if (E <= 128) return MOE_ROUTE_COUNT(16, 8);
  if (E <= 256) return MOE_ROUTE_COUNT(32, 8);
  return MOE_ROUTE_COUNT(64, 8);
#undef MOE_ROUTE_COUNT
}

extern "C" int moe_route(const float* logits, int T, int E, int k, int renormalize, int32_t* topk_idx,
                         float* topk_w, void* stream) {
  if (!logits || !topk_idx || !topk_w) return MOE_ERR_INVALID;
  if (T <= 0 || E <= 0 || k <= 0 || k > E || E > MOE_MAX_EXPERTS) return MOE_ERR_INVALID;
  if (!moe_aligned16(logits) || !moe_aligned16(topk_idx) || !moe_aligned16(topk_w)) return MOE_ERR_INVALID;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int r = renormalize != 0;
  // the same lane groups as the counting variant, so that both give the same bits (the order of the
  // sums in the softmax denominator follows the group shape)
  if (E <= 8) launch_route<8, 1>(logits, T, E, k, r, topk_idx, topk_w, s);
  else if (E <= 16) launch_route<8, 2>(logits, T, E, k, r, topk_idx, topk_w, s);
  else if (E <= 32) launch_route<8, 4>(logits, T, E, k, r, topk_idx, topk_w, s);
  else if (E <= 64) launch_route<8, 8>(logits, T, E, k, r, topk_idx, topk_w, s);
  else if (E <= 128) launch_route<16, 8>(logits, T, E, k, r, topk_idx, topk_w, s);
  else if (E <= 256) launch_route<32, 8>(logits, T, E, k, r, topk_idx, topk_w, s);
  else launch_route<64, 8>(logits, T, E, k, r, topk_idx, topk_w, s);
  return moe_check_launch();
}
