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
#include "common.h"

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

template <int G, int VPL>
__global__ __launch_bounds__(256) void route_kernel(const float* __restrict__ logits, int T, int E, int k,
                                                    int renormalize, int32_t* __restrict__ topk_idx,
                                                    float* __restrict__ topk_w) {
  constexpr int GROUPS_PER_BLOCK = 256 / G;
  const int tid = threadIdx.x;
  const int gl = tid % G;  // lane inside the group
  const int t = blockIdx.x * GROUPS_PER_BLOCK + tid / G;
  const bool live = t < T;
  const int tt = live ? t : T - 1;  // idle groups shadow the last token and store nothing

  uint64_t key[VPL];
  float val[VPL];
#pragma unroll
  for (int j = 0; j < VPL; ++j) {
    const int e = gl + j * G;
    if (e < E) {
      val[j] = logits[static_cast<size_t>(tt) * E + e];
      key[j] = (static_cast<uint64_t>(ordered_bits(val[j])) << 32) | (0xFFFFFFFFu - static_cast<uint32_t>(e));
    } else {
      val[j] = 0.f;
      key[j] = 0;  // below every real key (real keys have a non-zero low word or high bit)
    }
  }

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
#pragma unroll
    for (int m = 1; m < G; m <<= 1) {
      uint64_t o = shfl_xor_u64(best, m);
      best = o > best ? o : best;
    }
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

  if (live) {
#pragma unroll
    for (int j = 0; j < VPL; ++j) {
      const int i = gl + j * G;
      if (i < k) {
        topk_idx[static_cast<size_t>(t) * k + i] = my_idx[j];
        topk_w[static_cast<size_t>(t) * k + i] = expf(my_val[j] - row_max) * inv;
      }
    }
  }
}

template <int G, int VPL>
void launch_route(const float* logits, int T, int E, int k, int renorm, int32_t* idx, float* w, hipStream_t s) {
  const int groups = 256 / G;
  dim3 grid((T + groups - 1) / groups), block(256);
  MOE_LAUNCH("route", (route_kernel<G, VPL>), grid, block, 0, s, logits, T, E, k, renorm, idx, w);
}

}  // namespace

extern "C" int moe_route(const float* logits, int T, int E, int k, int renormalize, int32_t* topk_idx,
                         float* topk_w, void* stream) {
  if (!logits || !topk_idx || !topk_w) return MOE_ERR_INVALID;
  if (T <= 0 || E <= 0 || k <= 0 || k > E || E > MOE_MAX_EXPERTS) return MOE_ERR_INVALID;
  if (!moe_aligned16(logits) || !moe_aligned16(topk_idx) || !moe_aligned16(topk_w)) return MOE_ERR_INVALID;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int r = renormalize != 0;
  if (E <= 8) launch_route<8, 1>(logits, T, E, k, r, topk_idx, topk_w, s);
  else if (E <= 16) launch_route<16, 1>(logits, T, E, k, r, topk_idx, topk_w, s);
  else if (E <= 32) launch_route<32, 1>(logits, T, E, k, r, topk_idx, topk_w, s);
  else if (E <= 64) launch_route<16, 4>(logits, T, E, k, r, topk_idx, topk_w, s);
  else if (E <= 128) launch_route<32, 4>(logits, T, E, k, r, topk_idx, topk_w, s);
  else if (E <= 256) launch_route<64, 4>(logits, T, E, k, r, topk_idx, topk_w, s);
  else launch_route<64, 8>(logits, T, E, k, r, topk_idx, topk_w, s);
  return moe_check_launch();
}
