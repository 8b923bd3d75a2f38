// The router of Stage 1 of Algorithm 1 (logits = Router(input), a Linear layer without bias) and
// the derivative of Stage 1: through the renormalisation, TopK and Softmax back to the logits,
// and through the Linear layer to its weight and to the layer input.  The paper leaves the
// derivative to autograd; the formulas are the chain rule written out (see moe_route_bwd).
//
// moe_router_fwd   logits[T,E] = x[T,d] . Wr[E,d]^T with fp32 router weights and bf16 activations.
//   A wave owns a 32-token x 32-expert block and feeds v_mfma_f32_32x32x16_bf16 straight from global
//   memory (both operands are contiguous along d, the reduction).  The fp32 weights are split in
//   registers into three bf16 terms (w = hi + mid + lo exactly to 24 bits); x * hi, x * mid and
//   x * lo are exact in fp32, so the result has fp32 accuracy at bf16 matrix-core speed.
// moe_route_bwd    one group of G lanes per token, like moe_route: recomputes the softmax, forms the
//   gradient of the k chosen probabilities, scatters it by expert through LDS.
// moe_router_bwd   dx[T,d] += dlogits[T,E] . Wr[E,d]   (matrix cores, both operands split into two bf16
//                  terms; the weights pass through LDS and the transposing LDS load)
//                  dWr[E,d] = dlogits^T . x            (matrix cores, dlogits split into three bf16
//                  terms; token chunks -> partial sums in the workspace -> one deterministic
//                  reduction; no atomics)
#include "common.h"

namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// ------------------------------------------------------------------ router forward
// three bf16 terms of eight fp32 values; each residual is exact in fp32
__device__ __forceinline__ void split3(const float (&w)[8], bf16x8_t& hi, bf16x8_t& mid, bf16x8_t& lo) {
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const __bf16 h = static_cast<__bf16>(w[i]);
    const float r1 = w[i] - static_cast<float>(h);
    const __bf16 m = static_cast<__bf16>(r1);
    const float r2 = r1 - static_cast<float>(m);
    hi[i] = h;
    mid[i] = m;
    lo[i] = static_cast<__bf16>(r2);
  }
}

constexpr int RF_WAVES = 8;   // waves per workgroup: they share one block of logits and split the reduction
constexpr int RF_UNROLL = 2;  // reduction steps whose loads a wave has in flight together
constexpr int RF_TB = 2;      // 32-token blocks per workgroup: a weight fragment is split once and used for both

__global__ __launch_bounds__(64 * RF_WAVES) void router_fwd_kernel(const uint16_t* __restrict__ x,
                                                                   const float* __restrict__ Wr, int T, int d,
                                                                   int E, float* __restrict__ logits) {
  __shared__ float s_part[RF_WAVES - 1][RF_TB * 16][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int e_blocks = (E + 31) / 32;
  const int t0 = (blockIdx.x / e_blocks) * (32 * RF_TB), e0 = (blockIdx.x % e_blocks) * 32;
  const int lrow = lane & 31, lgrp = lane >> 5;
  int er = e0 + lrow;  if (er > E - 1) er = E - 1;     // rows past the end shadow the last one
  const float* wb = Wr + static_cast<size_t>(er) * d + lgrp * 8;
  const uint16_t* xa[RF_TB];
#pragma unroll
  for (int b = 0; b < RF_TB; ++b) {
    int tr = t0 + b * 32 + lrow;  if (tr > T - 1) tr = T - 1;
    xa[b] = x + static_cast<size_t>(tr) * d + lgrp * 8;
  }
  // Three independent accumulation chains per token block (one per weight term), so that consecutive
  // MFMAs do not wait for each other.  Wave w takes a contiguous eighth of the 16-wide reduction
  // steps.  The kernel is bound by what it pulls through the L2: the weights are read once per
  // workgroup, so a workgroup covers two token blocks with each weight fragment it loads and splits.
  f32x16_t acc[RF_TB][3];
#pragma unroll
  for (int b = 0; b < RF_TB; ++b)
#pragma unroll
    for (int m = 0; m < 3; ++m)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[b][m][r] = 0.f;
  const int nsteps = d / 16;
  auto mma = [&](const bf16x8_t (&a)[RF_TB], const f32x4& w0, const f32x4& w1) __attribute__((always_inline)) {
    const float wa[8] = {w0[0], w0[1], w0[2], w0[3], w1[0], w1[1], w1[2], w1[3]};
    bf16x8_t hi, mid, lo;
    split3(wa, hi, mid, lo);
    // operand order (weights, activations) gives a lane 4 consecutive experts of one token
#pragma unroll
    for (int b = 0; b < RF_TB; ++b) {
      acc[b][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lo, a[b], acc[b][0], 0, 0, 0);
      acc[b][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(mid, a[b], acc[b][1], 0, 0, 0);
      acc[b][2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hi, a[b], acc[b][2], 0, 0, 0);
    }
  };
  const int per_wave = (nsteps + RF_WAVES - 1) / RF_WAVES;
  int st = wave * per_wave;
  const int st_end = min(nsteps, st + per_wave);
  for (; st + RF_UNROLL <= st_end; st += RF_UNROLL) {
    bf16x8_t a[RF_UNROLL][RF_TB];
    f32x4 w0[RF_UNROLL], w1[RF_UNROLL];
#pragma unroll
    for (int u = 0; u < RF_UNROLL; ++u) {
      const int k = (st + u) * 16;
#pragma unroll
      for (int b = 0; b < RF_TB; ++b) a[u][b] = *reinterpret_cast<const bf16x8_t*>(xa[b] + k);
      w0[u] = *reinterpret_cast<const f32x4*>(wb + k);
      w1[u] = *reinterpret_cast<const f32x4*>(wb + k + 4);
    }
#pragma unroll
    for (int u = 0; u < RF_UNROLL; ++u) mma(a[u], w0[u], w1[u]);
  }
  for (; st < st_end; ++st) {
    const int k = st * 16;
    bf16x8_t a[RF_TB];
#pragma unroll
    for (int b = 0; b < RF_TB; ++b) a[b] = *reinterpret_cast<const bf16x8_t*>(xa[b] + k);
    const f32x4 w0 = *reinterpret_cast<const f32x4*>(wb + k), w1 = *reinterpret_cast<const f32x4*>(wb + k + 4);
    mma(a, w0, w1);
  }
  f32x16_t sum[RF_TB];
#pragma unroll
  for (int b = 0; b < RF_TB; ++b)
#pragma unroll
    for (int r = 0; r < 16; ++r) sum[b][r] = (acc[b][0][r] + acc[b][1][r]) + acc[b][2][r];   // smallest terms first
  // the partial sums of the waves are added in wave order
  if (wave > 0) {
#pragma unroll
    for (int b = 0; b < RF_TB; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) s_part[wave - 1][b * 16 + r][lane] = sum[b][r];
  }
  __syncthreads();
  if (wave != 0) return;
#pragma unroll
  for (int w = 0; w < RF_WAVES - 1; ++w)
#pragma unroll
    for (int b = 0; b < RF_TB; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) sum[b][r] += s_part[w][b * 16 + r][lane];
  // sum[b][4q+c] = (token t0 + 32 b + lrow, expert e0 + q*8 + lgrp*4 + c)
#pragma unroll
  for (int b = 0; b < RF_TB; ++b) {
    const int t = t0 + b * 32 + lrow;
    if (t < T) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int e = e0 + q * 8 + lgrp * 4;
        float* o = logits + static_cast<size_t>(t) * E + e;
        if (e + 3 < E && (E & 3) == 0) {
          *reinterpret_cast<f32x4*>(o) = f32x4{sum[b][4 * q], sum[b][4 * q + 1], sum[b][4 * q + 2], sum[b][4 * q + 3]};
        } else {
#pragma unroll
          for (int c = 0; c < 4; ++c)
            if (e + c < E) o[c] = sum[b][4 * q + c];
        }
      }
    }
  }
}

// ------------------------------------------------------------------ softmax / top-k backward
template <int G, int VPL>
__global__ __launch_bounds__(256) void route_bwd_kernel(const float* __restrict__ logits,
                                                        const int32_t* __restrict__ topk_idx,
                                                        const float* __restrict__ dgate, int T, int E, int k,
                                                        int renormalize, float* __restrict__ dlogits) {
  constexpr int GROUPS = 256 / G;
  extern __shared__ float s_dp[];   // [GROUPS][E]: gradient of the probabilities, by expert
  const int tid = threadIdx.x;
  const int gl = tid % G, grp = tid / G;
  const int t = blockIdx.x * GROUPS + grp;
  const bool live = t < T;
  const int tt = live ? t : T - 1;
  float* dp = s_dp + grp * E;

  float val[VPL];
  float m = -INFINITY;
#pragma unroll
  for (int j = 0; j < VPL; ++j) {
    const int e = gl + j * G;
    val[j] = e < E ? logits[static_cast<size_t>(tt) * E + e] : -INFINITY;
    m = fmaxf(m, val[j]);
    if (e < E) dp[e] = 0.f;
  }
#pragma unroll
  for (int s = 1; s < G; s <<= 1) m = fmaxf(m, __shfl_xor(m, s, MOE_WAVE));
  float p[VPL], sum = 0.f;
#pragma unroll
  for (int j = 0; j < VPL; ++j) {
    p[j] = gl + j * G < E ? expf(val[j] - m) : 0.f;
    sum += p[j];
  }
#pragma unroll
  for (int s = 1; s < G; s <<= 1) sum += __shfl_xor(sum, s, MOE_WAVE);
  const float inv = 1.0f / sum;
#pragma unroll
  for (int j = 0; j < VPL; ++j) p[j] *= inv;

  // the chosen probabilities s_i and the gradient of the gates, slot i on lane i % G
  float S = 0.f, dot = 0.f;
  for (int i = gl; i < k; i += G) {
    const int e = topk_idx[static_cast<size_t>(tt) * k + i];
    const float s_i = expf(logits[static_cast<size_t>(tt) * E + e] - m) * inv;
    S += s_i;
    dot += dgate[static_cast<size_t>(tt) * k + i] * s_i;
  }
#pragma unroll
  for (int s = 1; s < G; s <<= 1) { S += __shfl_xor(S, s, MOE_WAVE); dot += __shfl_xor(dot, s, MOE_WAVE); }
  // renormalised: w_i = s_i / S, dL/ds_i = (dgate_i - sum_j dgate_j w_j) / S ; otherwise dL/ds_i = dgate_i
  const float invS = renormalize ? 1.0f / S : 1.0f;
  const float shift = renormalize ? dot * invS : 0.f;
  __syncthreads();                       // dp is zeroed
  float c = 0.f;                         // sum_i dL/ds_i * s_i
  for (int i = gl; i < k; i += G) {
    const int e = topk_idx[static_cast<size_t>(tt) * k + i];
    const float s_i = expf(logits[static_cast<size_t>(tt) * E + e] - m) * inv;
    const float ds = (dgate[static_cast<size_t>(tt) * k + i] - shift) * invS;
    dp[e] = ds;                          // a token's experts are distinct
    c += ds * s_i;
  }
#pragma unroll
  for (int s = 1; s < G; s <<= 1) c += __shfl_xor(c, s, MOE_WAVE);
  __syncthreads();
  if (live) {
#pragma unroll
    for (int j = 0; j < VPL; ++j) {
      const int e = gl + j * G;
      if (e < E) dlogits[static_cast<size_t>(t) * E + e] = p[j] * (dp[e] - c);
    }
  }
}

template <int G, int VPL>
void launch_route_bwd(const float* logits, const int32_t* idx, const float* dgate, int T, int E, int k, int renorm,
                      float* dlogits, hipStream_t s) {
  const int groups = 256 / G;
  dim3 grid((T + groups - 1) / groups), block(256);
  MOE_LAUNCH("route_bwd", (route_bwd_kernel<G, VPL>), grid, block, groups * E * sizeof(float), s, logits, idx, dgate,
             T, E, k, renorm, dlogits);
}

// ------------------------------------------------------------------ router backward
// dx += dlogits . Wr on the matrix cores.  A workgroup owns 128 columns and 128 tokens: its block of
// the weights is split once into two bf16 terms (hi + mid: 16 significant bits, far more than the
// bf16 result keeps) and kept in LDS as it lies in memory, experts as rows, to be read with the
// transposing LDS load; dlogits goes from global memory straight into registers (eight consecutive
// experts per lane) and is split the same way; the three products hi*hi, hi*mid, mid*hi are
// accumulated.  Results are staged per wave in LDS so that dx is read and written 16 bytes per lane.
constexpr int DX_COLS = 128;      // columns per workgroup: 4 waves x 32
constexpr int DX_TOK = 32;        // tokens per MFMA block
constexpr int DX_BLOCKS = 4;      // token blocks per workgroup
constexpr int DX_EXP = 64;        // experts per LDS stage
constexpr int DX_WROW = DX_COLS * 2;      // bytes of an expert row of a weight term
constexpr int DX_OROW = 36;               // floats per token row of a wave's output stage (padded)

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// 16-byte pieces of a row are XOR-swizzled with 4 * (row & 3): the four rows that 16 lanes of a
// transposing read touch then fall into different bank groups
__device__ __forceinline__ int tr_piece(int row, int piece) { return piece ^ ((row & 3) << 2); }

// two bf16 terms of eight fp32 values
__device__ __forceinline__ void split2(const float (&w)[8], bf16x8_t& hi, bf16x8_t& mid) {
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const __bf16 h = static_cast<__bf16>(w[i]);
    hi[i] = h;
    mid[i] = static_cast<__bf16>(w[i] - static_cast<float>(h));
  }
}

__global__ __launch_bounds__(256, 2) void router_bwd_dx_kernel(const float* __restrict__ dlogits,
                                                            const float* __restrict__ Wr, int T, int d, int E,
                                                            uint16_t* __restrict__ dx) {
  // grid: (column blocks of 128, token chunks of 128)
  __shared__ __attribute__((aligned(16))) unsigned char s_w[2][DX_EXP * DX_WROW];
  __shared__ __attribute__((aligned(16))) float s_o[4][DX_TOK * DX_OROW];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c_base = blockIdx.x * DX_COLS, t_base = blockIdx.y * (DX_TOK * DX_BLOCKS);
  const int lrow = lane & 31, kg = lane >> 5;
  // weight fragment address: within 16 lanes, lane i names expert row i / 4 and four columns
  // 4 * (i % 4) of the wave's 32; lane l of the 16 receives rows 0..3 of column l
  const int fi = lane & 15;
  const int fcol = wave * 32 + ((lane >> 4) & 1) * 16 + 4 * (fi & 3);
  const int frow = kg * 8 + (fi >> 2);
  const int wfrag = frow * DX_WROW + tr_piece(frow, fcol >> 3) * 16 + (fcol & 7) * 2;

  f32x16_t acc[DX_BLOCKS];
#pragma unroll
  for (int b = 0; b < DX_BLOCKS; ++b)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[b][r] = 0.f;

  // what dx holds so far is requested now and needed only at the end: after the output stage lane l
  // owns 16 consecutive columns (l % 2) of token l / 2 of each block
  const int ot = lane >> 1, oc = (lane & 1) * 16;
  const int col = c_base + wave * 32 + oc;
  u32x4 old[DX_BLOCKS][2];
#pragma unroll
  for (int b = 0; b < DX_BLOCKS; ++b) {
    const int t = t_base + b * DX_TOK + ot;
    if (t < T && col < d) {
      const u32x4* p = reinterpret_cast<const u32x4*>(dx + static_cast<size_t>(t) * d + col);
      old[b][0] = p[0];
      old[b][1] = p[1];
    } else {
      old[b][0] = u32x4{0u, 0u, 0u, 0u};
      old[b][1] = u32x4{0u, 0u, 0u, 0u};
    }
  }

  for (int e_base = 0; e_base < E; e_base += DX_EXP) {
    __syncthreads();   // the previous stage has been read
    // stage the weights: thread -> expert row tid / 4 (64 rows), pieces tid % 4 + 4 h of 16 (8 columns each)
    {
      const int er = tid >> 2, e = e_base + er;
#pragma unroll
      for (int h = 0; h < 4; ++h) {
        const int piece = h * 4 + (tid & 3), c = c_base + piece * 8;
        float w[8];
        if (e < E && c < d) {
          const f32x4 w0 = *reinterpret_cast<const f32x4*>(Wr + static_cast<size_t>(e) * d + c);
          const f32x4 w1 = *reinterpret_cast<const f32x4*>(Wr + static_cast<size_t>(e) * d + c + 4);
#pragma unroll
          for (int j = 0; j < 4; ++j) { w[j] = w0[j]; w[4 + j] = w1[j]; }
        } else {
#pragma unroll
          for (int j = 0; j < 8; ++j) w[j] = 0.f;
        }
        bf16x8_t hi, mid;
        split2(w, hi, mid);
        const int off = er * DX_WROW + tr_piece(er, piece) * 16;
        *reinterpret_cast<bf16x8_t*>(s_w[0] + off) = hi;
        *reinterpret_cast<bf16x8_t*>(s_w[1] + off) = mid;
      }
    }
    __syncthreads();
    // one 16-expert sub-step of token block b: three MFMAs on the fragments of sub-step ss
    auto mma3 = [&](int b_, int ss, const float (&gv)[8]) __attribute__((always_inline)) {
      bf16x8_t ghi, gmid;
      split2(gv, ghi, gmid);
      union { s16x4 h[2]; bf16x8_t v; } whi, wmid;
      const unsigned char* wf = s_w[0] + wfrag + ss * 16 * DX_WROW;
      whi.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(wf));
      whi.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(wf + 4 * DX_WROW));
      wmid.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(wf + DX_EXP * DX_WROW));
      wmid.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(wf + DX_EXP * DX_WROW + 4 * DX_WROW));
      // (gradient, weight): a lane ends up with one column and 16 tokens; smallest terms first
      acc[b_] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gmid, whi.v, acc[b_], 0, 0, 0);
      acc[b_] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ghi, wmid.v, acc[b_], 0, 0, 0);
      acc[b_] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ghi, whi.v, acc[b_], 0, 0, 0);
    };
    if ((E & 7) == 0) {
      // Every group of eight experts is whole or absent.  All four sub-steps are run; a group past the
      // last expert reads the last eight experts again and meets zero weight rows.  Several workgroups
      // share a compute unit and hide each other's load latency.
      f32x4 cur[4][2];
      auto fetch = [&](int b_, f32x4 (&dst)[4][2]) __attribute__((always_inline)) {
        const int t = t_base + b_ * DX_TOK + lrow;
        const float* row = dlogits + static_cast<size_t>(t < T ? t : T - 1) * E;   // rows past the end are not stored
#pragma unroll
        for (int ss = 0; ss < 4; ++ss) {
          int e = e_base + ss * 16 + kg * 8;
          if (e > E - 8) e = E - 8;
          dst[ss][0] = *reinterpret_cast<const f32x4*>(row + e);
          dst[ss][1] = *reinterpret_cast<const f32x4*>(row + e + 4);
        }
      };
#pragma unroll
      for (int b = 0; b < DX_BLOCKS; ++b) {
        fetch(b, cur);
#pragma unroll
        for (int ss = 0; ss < 4; ++ss) {
          const float gv[8] = {cur[ss][0][0], cur[ss][0][1], cur[ss][0][2], cur[ss][0][3],
                               cur[ss][1][0], cur[ss][1][1], cur[ss][1][2], cur[ss][1][3]};
          mma3(b, ss, gv);
        }
      }
    } else {
      const int nss = min(DX_EXP, E - e_base + 15) / 16;   // 16-expert sub-steps that hold an expert
#pragma unroll
      for (int b = 0; b < DX_BLOCKS; ++b) {
        const int t = t_base + b * DX_TOK + lrow;
        const int tc = t < T ? t : T - 1;   // rows past the end are computed and not stored
        const float* g = dlogits + static_cast<size_t>(tc) * E + e_base + kg * 8;
        for (int ss = 0; ss < nss; ++ss) {
          const int e = e_base + ss * 16 + kg * 8;
          float gv[8];
#pragma unroll
          for (int j = 0; j < 8; ++j) gv[j] = e + j < E ? g[ss * 16 + j] : 0.f;
          mma3(b, ss, gv);
        }
      }
    }
  }
  // acc[b][4q+c] = (token t_base + 32 b + 8 q + 4 kg + c, column c_base + 32 wave + lane % 32).
  // Through the wave's own stage: afterwards lane l owns 16 consecutive columns (l % 2) of token l / 2.
  float* so = s_o[wave];
#pragma unroll
  for (int b = 0; b < DX_BLOCKS; ++b) {
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int r = 0; r < 16; ++r) so[(8 * (r >> 2) + 4 * kg + (r & 3)) * DX_OROW + lrow] = acc[b][r];
    __builtin_amdgcn_wave_barrier();
    const int t = t_base + b * DX_TOK + ot;
    if (t < T && col < d) {
      float v[16];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const f32x4 q = *reinterpret_cast<const f32x4*>(so + ot * DX_OROW + oc + 4 * j);
        v[4 * j] = q[0]; v[4 * j + 1] = q[1]; v[4 * j + 2] = q[2]; v[4 * j + 3] = q[3];
      }
      u32x4* p = reinterpret_cast<u32x4*>(dx + static_cast<size_t>(t) * d + col);
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        u32x4 o;
#pragma unroll
        for (int j = 0; j < 4; ++j)
          o[j] = pack_bf16(bf16lo(old[b][h][j]) + v[8 * h + 2 * j], bf16hi(old[b][h][j]) + v[8 * h + 2 * j + 1]);
        p[h] = o;
      }
    }
  }
}

// dWr = dlogits^T . x on the matrix cores.  Both operands have the reduction (the tokens) as their
// slow dimension, so both pass through LDS: a stage of 32 tokens of x is kept as it lies in memory
// and read with the transposing LDS load; the same tokens of dlogits are split into three bf16 terms
// (as the weights are in the forward kernel) and stored expert-major, so that a lane reads the eight
// consecutive tokens of its expert with one 16-byte load per term.  The next stage is fetched into
// registers while the current one is multiplied.
constexpr int DW_CHUNK = 256;   // tokens per partial sum
constexpr int DW_COLS = 128;    // columns of x per workgroup: 4 waves x 32
constexpr int DW_EXP = 64;      // experts per workgroup: 2 MFMA row blocks
constexpr int DW_TOK = 32;      // tokens per stage
constexpr int DW_XROW = DW_COLS * 2;        // bytes of a token row of the x stage
constexpr int DW_GROW = DW_TOK * 2 + 16;    // bytes of an expert row of a dlogits term (padded)

__global__ __launch_bounds__(256) void router_bwd_dw_partial_kernel(const float* __restrict__ dlogits,
                                                                    const uint16_t* __restrict__ x, int T, int d,
                                                                    int E, float* __restrict__ part) {
  // grid: (column blocks of 128, token chunks of 256, expert blocks of 64)
  __shared__ __attribute__((aligned(16))) unsigned char s_x[DW_TOK * DW_XROW];
  __shared__ __attribute__((aligned(16))) unsigned char s_g[3][DW_EXP * DW_GROW];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c_base = blockIdx.x * DW_COLS, chunk = blockIdx.y, e_base = blockIdx.z * DW_EXP;
  const int t_lo = chunk * DW_CHUNK, t_hi = min(T, t_lo + DW_CHUNK);

  // loader roles: x -- token row tid / 8, pieces 2 * (tid % 8), +1; dlogits -- token tid / 8, experts 8 * (tid % 8) .. +8
  const int ld_row = tid >> 3, ld_sub = tid & 7;
  u32x4 rx[2];
  float rg[8];
  auto fetch = [&](int tb) __attribute__((always_inline)) {
    const int t = tb + ld_row;
    const int tc = t < T ? t : T - 1;   // rows past the end meet zero gradients below
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int c = c_base + (2 * ld_sub + h) * 8;
      rx[h] = c < d ? *reinterpret_cast<const u32x4*>(x + static_cast<size_t>(tc) * d + c) : u32x4{0u, 0u, 0u, 0u};
    }
    const int e = e_base + ld_sub * 8;
    const float* g = dlogits + static_cast<size_t>(tc) * E + e;
    if (t < t_hi && e + 7 < E && (E & 3) == 0) {
      const f32x4 g0 = *reinterpret_cast<const f32x4*>(g), g1 = *reinterpret_cast<const f32x4*>(g + 4);
#pragma unroll
      for (int j = 0; j < 4; ++j) { rg[j] = g0[j]; rg[4 + j] = g1[j]; }
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) rg[j] = (t < t_hi && e + j < E) ? g[j] : 0.f;
    }
  };
  auto stage = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int h = 0; h < 2; ++h)
      *reinterpret_cast<u32x4*>(s_x + ld_row * DW_XROW + tr_piece(ld_row, 2 * ld_sub + h) * 16) = rx[h];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const __bf16 hi = static_cast<__bf16>(rg[j]);
      const float r1 = rg[j] - static_cast<float>(hi);
      const __bf16 mid = static_cast<__bf16>(r1);
      const __bf16 lo = static_cast<__bf16>(r1 - static_cast<float>(mid));
      const int off = (ld_sub * 8 + j) * DW_GROW + ld_row * 2;
      *reinterpret_cast<__bf16*>(s_g[0] + off) = hi;
      *reinterpret_cast<__bf16*>(s_g[1] + off) = mid;
      *reinterpret_cast<__bf16*>(s_g[2] + off) = lo;
    }
  };

  // fragment addresses.  x: within 16 lanes, lane i names token row i / 4 and four columns 4 * (i % 4) of the
  // wave's 32; lane l of the 16 receives rows 0..3 of column l.  The second read lies 4 rows further, the second
  // 16-token sub-step 16 rows further (the swizzle only depends on row % 4).
  const int fi = lane & 15, kg = lane >> 5;
  const int fcol = wave * 32 + ((lane >> 4) & 1) * 16 + 4 * (fi & 3);
  const int frow = kg * 8 + (fi >> 2);
  const unsigned char* xfrag = s_x + frow * DW_XROW + tr_piece(frow, fcol >> 3) * 16 + (fcol & 7) * 2;
  const int gfrag = (lane & 31) * DW_GROW + kg * 16;   // expert lane % 32 of a block, tokens 8 * kg .. +8

  f32x16_t acc[2][3];   // [expert block][term]: independent chains
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int m = 0; m < 3; ++m)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[b][m][r] = 0.f;

  fetch(t_lo);
  for (int tb = t_lo; tb < t_hi; tb += DW_TOK) {
    __syncthreads();   // the previous stage has been read
    stage();
    __syncthreads();
    if (tb + DW_TOK < t_hi) fetch(tb + DW_TOK);
#pragma unroll
    for (int ss = 0; ss < 2; ++ss) {
      union { s16x4 h[2]; bf16x8_t v; } xb;
      xb.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(xfrag + ss * 16 * DW_XROW));
      xb.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(xfrag + ss * 16 * DW_XROW + 4 * DW_XROW));
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int m = 2; m >= 0; --m) {
          const bf16x8_t ga = *reinterpret_cast<const bf16x8_t*>(s_g[m] + b * 32 * DW_GROW + gfrag + ss * 32);
          // (gradient, activation): a lane ends up with one column and 16 experts
          acc[b][m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ga, xb.v, acc[b][m], 0, 0, 0);
        }
    }
  }
  // acc[b][.][4q+c] = (expert e_base + 32 b + 8 q + 4 (lane / 32) + c, column c_base + 32 wave + lane % 32)
  const int col = c_base + wave * 32 + (lane & 31);
  if (col < d) {
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int e = e_base + 32 * b + 8 * (r >> 2) + 4 * kg + (r & 3);
        if (e < E)
          part[(static_cast<size_t>(chunk) * E + e) * d + col] = (acc[b][2][r] + acc[b][1][r]) + acc[b][0][r];
      }
  }
}

__global__ __launch_bounds__(256) void router_bwd_dw_reduce_kernel(const float* __restrict__ part, int chunks,
                                                                   size_t n, float* __restrict__ dWr) {
  const size_t i = (static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x) * 4;
  if (i >= n) return;
  f32x4 s = {0.f, 0.f, 0.f, 0.f};
  for (int c = 0; c < chunks; ++c) s += *reinterpret_cast<const f32x4*>(part + static_cast<size_t>(c) * n + i);
  *reinterpret_cast<f32x4*>(dWr + i) = s;
}

bool bad_router_dims(int T, int d, int E) { return T <= 0 || d <= 0 || E <= 0 || E > MOE_MAX_EXPERTS || d % 16 != 0; }

}  // namespace

extern "C" int moe_router_fwd(const moe_bf16* x, const float* Wr, int T, int d, int E, float* logits, void* stream) {
  if (!x || !Wr || !logits) return MOE_ERR_INVALID;
  if (bad_router_dims(T, d, E)) return MOE_ERR_INVALID;
  if (!moe_aligned16(x) || !moe_aligned16(Wr) || !moe_aligned16(logits)) return MOE_ERR_INVALID;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const long long blocks = static_cast<long long>((T + 32 * RF_TB - 1) / (32 * RF_TB)) * ((E + 31) / 32);
  dim3 grid(static_cast<unsigned>(blocks)), block(64 * RF_WAVES);
  MOE_LAUNCH("router_fwd", router_fwd_kernel, grid, block, 0, s, x, Wr, T, d, E, logits);
  return moe_check_launch();
}

extern "C" int moe_route_bwd(const float* logits, const int32_t* topk_idx, const float* dgate, int T, int E, int k,
                             int renormalize, float* dlogits, void* stream) {
  if (!logits || !topk_idx || !dgate || !dlogits) return MOE_ERR_INVALID;
  if (T <= 0 || E <= 0 || k <= 0 || k > E || E > MOE_MAX_EXPERTS) return MOE_ERR_INVALID;
  if (!moe_aligned16(logits) || !moe_aligned16(topk_idx) || !moe_aligned16(dgate) || !moe_aligned16(dlogits))
    return MOE_ERR_INVALID;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int r = renormalize != 0;
  if (E <= 8) launch_route_bwd<8, 1>(logits, topk_idx, dgate, T, E, k, r, dlogits, s);
  else if (E <= 16) launch_route_bwd<16, 1>(logits, topk_idx, dgate, T, E, k, r, dlogits, s);
  else if (E <= 32) launch_route_bwd<32, 1>(logits, topk_idx, dgate, T, E, k, r, dlogits, s);
  else if (E <= 64) launch_route_bwd<64, 1>(logits, topk_idx, dgate, T, E, k, r, dlogits, s);
  else if (E <= 128) launch_route_bwd<64, 2>(logits, topk_idx, dgate, T, E, k, r, dlogits, s);
  else if (E <= 256) launch_route_bwd<64, 4>(logits, topk_idx, dgate, T, E, k, r, dlogits, s);
  else launch_route_bwd<64, 8>(logits, topk_idx, dgate, T, E, k, r, dlogits, s);
  return moe_check_launch();
}

extern "C" size_t moe_router_bwd_workspace_bytes(int T, int d, int E) {
  if (T <= 0 || d <= 0 || E <= 0) return 0;
  const size_t chunks = (static_cast<size_t>(T) + DW_CHUNK - 1) / DW_CHUNK;
  return chunks * E * d * sizeof(float);
}

extern "C" int moe_router_bwd(const moe_bf16* x, const float* Wr, const float* dlogits, int T, int d, int E,
                              moe_bf16* dx, float* dWr, void* ws, size_t ws_bytes, void* stream) {
  if (!x || !Wr || !dlogits || !dx || !dWr || !ws) return MOE_ERR_INVALID;
  if (bad_router_dims(T, d, E)) return MOE_ERR_INVALID;
  const void* ptrs[] = {x, Wr, dlogits, dx, dWr, ws};
  for (const void* p : ptrs) if (!moe_aligned16(p)) return MOE_ERR_INVALID;
  if (ws_bytes < moe_router_bwd_workspace_bytes(T, d, E)) return MOE_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  {
    dim3 grid((d + DX_COLS - 1) / DX_COLS, (T + DX_TOK * DX_BLOCKS - 1) / (DX_TOK * DX_BLOCKS)), block(256);
    MOE_LAUNCH("router_bwd_dx", router_bwd_dx_kernel, grid, block, 0, s, dlogits, Wr, T, d, E, dx);
  }
  const int chunks = (T + DW_CHUNK - 1) / DW_CHUNK;
  {
    dim3 grid((d + DW_COLS - 1) / DW_COLS, chunks, (E + DW_EXP - 1) / DW_EXP), block(256);
    MOE_LAUNCH("router_bwd_dw_partial", router_bwd_dw_partial_kernel, grid, block, 0, s, dlogits, x, T, d, E,
               static_cast<float*>(ws));
  }
  {
    const size_t n = static_cast<size_t>(E) * d;
    dim3 grid(static_cast<unsigned>((n / 4 + 255) / 256)), block(256);
    MOE_LAUNCH("router_bwd_dw_reduce", router_bwd_dw_reduce_kernel, grid, block, 0, s, static_cast<const float*>(ws),
               chunks, n, dWr);
  }
  return moe_check_launch();
}
