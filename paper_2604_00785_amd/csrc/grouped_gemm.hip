// Stage 4 of Algorithm 1 (the three Grouped_mm calls around Silu(gate)*up) and
// its derivative, as grouped bf16 MFMA GEMMs: one launch covers every expert.
//
// One workgroup (8 waves) computes one 256x256 output tile with a 64-deep
// K step.  Both operand tiles live in LDS as [256 rows][64 k] bf16 (128 bytes
// per row, 16-byte pieces XOR-swizzled by the row so that both the MFMA
// fragment reads and the fill writes spread over the banks), double-buffered:
// while the MFMAs consume one buffer, the next K step is already in flight from
// global memory into registers and is written to the other buffer afterwards.
// The waves form a 2 (M) x 4 (N) grid; each owns a 128x64 piece = 4x2
// v_mfma_f32_32x32x16_bf16 accumulators (128 fp32 registers per lane).
//
// An operand that is contiguous along K in memory (activations [rows, K],
// forward weights [N, K]) goes to LDS as it is.  An operand that is contiguous
// along the other dimension (weights in dgrad, both operands in wgrad) is
// transposed in registers on its way to LDS: a thread loads a 4 (k) x 8 (n)
// block with four 16-byte loads and writes eight 8-byte K-runs.
//
// Tiles of the row-grouped products are found on the device from
// expert_offsets: a workgroup turns its M-tile number into (expert, first row)
// with a wave-wide prefix sum over ceil(rows_e / 256); experts without rows own
// no tile; rows past an expert's end are clamped on load and masked on store.
#include "common.h"

namespace {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int GEMM_THREADS = 512;
constexpr int TILE_BYTES = BM * BK * 2;              // one operand tile
constexpr int LDS_BYTES = 2 * 2 * TILE_BYTES;        // A and B, double-buffered

enum GemmMode { GATE_UP = 0, DOWN = 1, DGRAD_H = 2, DGRAD_X = 3, WGRAD = 4 };

struct GemmArgs {
  // row-grouped products (modes 0-3)
  const uint16_t* A0;   // [R_cap, K]   activations (phase 0)
  const uint16_t* A1;   // second K phase of DGRAD_X (du), else unused
  const uint16_t* B0;   // weights, stacked over experts
  const uint16_t* B1;   // Wu (GATE_UP: second half of the N tile; DGRAD_X: second K phase)
  const uint16_t* G;    // DGRAD_H epilogue inputs
  const uint16_t* U;
  uint16_t* O0;         // g | yp | dg | dxp | dW
  uint16_t* O1;         // u | du
  uint16_t* O2;         // h
  const int32_t* offsets;
  int E;
  int K;                // reduction length of one phase (modes 0-3)
  int N;                // output columns (per half for GATE_UP)
  int n_tiles;          // column tiles
  int m_tiles_cap;      // upper bound on row tiles (modes 0-3)
  // WGRAD: out[e][M][N] = sum over the expert's rows of A[r][M] * B[r][N]
  int M;
};

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row ^ (row >> 3)) & 7); }

// ---- global -> registers ----------------------------------------------------
// K-contiguous operand: thread covers rows tid/8 + 64*i (i<4), 16-byte piece tid%8.
// K-strided operand: thread covers k rows (tid/32)*4 + j (j<4), columns (tid%32)*8 .. +8.
// Either way a thread stages four 16-byte pieces per operand.
struct Staged { uint4 v[4]; };

__device__ __forceinline__ void store_kc(const Staged& r, char* tile, int tid) {
  const int c = tid & 7;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = (tid >> 3) + 64 * i;
    *reinterpret_cast<uint4*>(tile + row * 128 + swz(row, c) * 16) = r.v[i];
  }
}

__device__ __forceinline__ void store_ks(const Staged& r, char* tile, int tid) {
  const int nb = tid & 31, kq = tid >> 5;
  const int chunk = kq >> 1, half = kq & 1;
  const uint32_t w0[4] = {r.v[0].x, r.v[0].y, r.v[0].z, r.v[0].w};
  const uint32_t w1[4] = {r.v[1].x, r.v[1].y, r.v[1].z, r.v[1].w};
  const uint32_t w2[4] = {r.v[2].x, r.v[2].y, r.v[2].z, r.v[2].w};
  const uint32_t w3[4] = {r.v[3].x, r.v[3].y, r.v[3].z, r.v[3].w};
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const int row = nb * 8 + q;
    const uint32_t sel = (q & 1) ? 0x07060302u : 0x05040100u;
    uint2 o;
    o.x = __builtin_amdgcn_perm(w1[q >> 1], w0[q >> 1], sel);  // k0 (low half), k1 (high half)
    o.y = __builtin_amdgcn_perm(w3[q >> 1], w2[q >> 1], sel);  // k2, k3
    *reinterpret_cast<uint2*>(tile + row * 128 + swz(row, chunk) * 16 + half * 8) = o;
  }
}

template <int MODE>
__global__ __launch_bounds__(GEMM_THREADS) void grouped_gemm_kernel(GemmArgs a) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  __shared__ int s_tile[3];
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 2, wn = wave & 3;

  // ---------------- which tile ------------------------------------------------
  int e, m0, m_end, nt;
  if constexpr (MODE == WGRAD) {
    e = blockIdx.y;
    nt = blockIdx.x % a.n_tiles;
    m0 = (blockIdx.x / a.n_tiles) * BM;   // output row of dW
    m_end = a.M;
  } else {
    nt = blockIdx.x % a.n_tiles;
    const int mt = blockIdx.x / a.n_tiles;
    if (tid == 0) s_tile[0] = -1;
    __syncthreads();
    if (wave == 0) {
      int base = 0;
      for (int e0 = 0; e0 < a.E; e0 += 64) {
        const int ee = e0 + lane;
        const int o0 = ee < a.E ? a.offsets[ee] : 0;
        const int o1 = ee < a.E ? a.offsets[ee + 1] : 0;
        const int tiles = (o1 - o0 + BM - 1) / BM;
        int inc = tiles;
#pragma unroll
        for (int s = 1; s < 64; s <<= 1) {
          const int v = __shfl_up(inc, s, 64);
          if (lane >= s) inc += v;
        }
        const int exc = base + inc - tiles;
        if (mt >= exc && mt < exc + tiles) {
          s_tile[0] = ee;
          s_tile[1] = o0 + (mt - exc) * BM;
          s_tile[2] = o1;
        }
        base += __shfl(inc, 63, 64);
      }
    }
    __syncthreads();
    e = s_tile[0];
    if (e < 0) return;
    m0 = s_tile[1];
    m_end = s_tile[2];
  }
  const int n0 = nt * (MODE == GATE_UP ? BN / 2 : BN);

  // ---------------- operand sources -------------------------------------------
  // A tile rows <-> output rows m0 + r ; B tile rows <-> output columns.
  const uint16_t* pa[4];   // per-thread row pointers (KC) or column pointer (KS, pa[0])
  const uint16_t* pb[4];
  ptrdiff_t a_phase = 0, b_phase = 0;   // element offset added for the second K phase
  int k_lo = 0, k_hi = 0;            // WGRAD: expert's row range (the reduction)
  int nk;
  size_t lda, ldb;

  if constexpr (MODE == WGRAD) {
    k_lo = a.offsets[e];
    k_hi = a.offsets[e + 1];
    nk = (k_hi - k_lo + BK - 1) / BK;
    lda = a.M;
    ldb = a.N;
    const int nb = tid & 31;
    int ca = m0 + nb * 8;  if (ca > a.M - 8) ca = a.M - 8;
    int cb = n0 + nb * 8;  if (cb > a.N - 8) cb = a.N - 8;
    pa[0] = a.A0 + ca;
    pb[0] = a.B0 + cb;
  } else {
    nk = a.K / BK;
    lda = a.K;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int r = m0 + (tid >> 3) + 64 * i;
      if (r > m_end - 1) r = m_end - 1;
      pa[i] = a.A0 + static_cast<size_t>(r) * lda + (tid & 7) * 8;
    }
    if constexpr (MODE == DGRAD_X) { a_phase = a.A1 - a.A0; nk *= 2; }
    if constexpr (MODE == GATE_UP || MODE == DOWN) {
      ldb = a.K;
      const size_t wsz = static_cast<size_t>(a.N) * a.K;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int r = (tid >> 3) + 64 * i;   // LDS row of the B tile
        const uint16_t* w = a.B0;
        int col = n0 + r;
        if constexpr (MODE == GATE_UP) {
          if (r >= BN / 2) { w = a.B1; col = n0 + r - BN / 2; }
        }
        if (col > a.N - 1) col = a.N - 1;
        pb[i] = w + static_cast<size_t>(e) * wsz + static_cast<size_t>(col) * ldb + (tid & 7) * 8;
      }
    } else {  // DGRAD_H / DGRAD_X: weights stored [K][N]
      ldb = a.N;
      const size_t wsz = static_cast<size_t>(a.N) * a.K;
      int cb = n0 + (tid & 31) * 8;
      if (cb > a.N - 8) cb = a.N - 8;
      pb[0] = a.B0 + static_cast<size_t>(e) * wsz + cb;
      if constexpr (MODE == DGRAD_X) b_phase = a.B1 - a.B0;
    }
  }
  constexpr bool A_KS = (MODE == WGRAD);
  constexpr bool B_KS = (MODE == WGRAD || MODE == DGRAD_H || MODE == DGRAD_X);

  Staged ra, rb;

  auto load_tiles = [&](int kt) {
    // K offset inside the phase, and the phase offset
    int kk = kt;
    ptrdiff_t offa = 0, offb = 0;
    if constexpr (MODE == DGRAD_X) {
      const int half = nk >> 1;
      if (kt >= half) { kk = kt - half; offa = a_phase; offb = b_phase; }
    }
    if constexpr (A_KS) {
      const int kq = tid >> 5;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int r = k_lo + kk * BK + kq * 4 + j;
        ra.v[j] = r < k_hi ? *reinterpret_cast<const uint4*>(pa[0] + static_cast<size_t>(r) * lda)
                              : make_uint4(0, 0, 0, 0);
      }
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        ra.v[i] = *reinterpret_cast<const uint4*>(pa[i] + offa + static_cast<size_t>(kk) * BK);
    }
    if constexpr (B_KS) {
      const int kq = tid >> 5;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if constexpr (MODE == WGRAD) {
          const int r = k_lo + kk * BK + kq * 4 + j;
          rb.v[j] = r < k_hi ? *reinterpret_cast<const uint4*>(pb[0] + static_cast<size_t>(r) * ldb)
                                : make_uint4(0, 0, 0, 0);
        } else {
          const int r = kk * BK + kq * 4 + j;
          rb.v[j] = *reinterpret_cast<const uint4*>(pb[0] + offb + static_cast<size_t>(r) * ldb);
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        rb.v[i] = *reinterpret_cast<const uint4*>(pb[i] + static_cast<size_t>(kk) * BK);
    }
  };
  auto store_tiles = [&](int buf) {
    char* ta = lds + buf * 2 * TILE_BYTES;
    char* tb = ta + TILE_BYTES;
    if constexpr (A_KS) store_ks(ra, ta, tid); else store_kc(ra, ta, tid);
    if constexpr (B_KS) store_ks(rb, tb, tid); else store_kc(rb, tb, tid);
  };

  // ---------------- main loop ----------------------------------------------------
  f32x16_t acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int lrow = lane & 31, lgrp = lane >> 5;
  if (nk > 0) {
    load_tiles(0);
    store_tiles(0);
  }
  __syncthreads();
  auto compute = [&](int buf) {
    const char* ta = lds + buf * 2 * TILE_BYTES;
    const char* tb = ta + TILE_BYTES;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8_t fa[4], fb[2];
      const int chunk = ks * 2 + lgrp;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = wm * 128 + i * 32 + lrow;
        fa[i] = *reinterpret_cast<const bf16x8_t*>(ta + row * 128 + swz(row, chunk) * 16);
      }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int row = j * 128 + wn * 32 + lrow;
        fb[j] = *reinterpret_cast<const bf16x8_t*>(tb + row * 128 + swz(row, chunk) * 16);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
  };
  // steady state: the next K step is loaded while this one is multiplied
  for (int kt = 0; kt + 1 < nk; ++kt) {
    load_tiles(kt + 1);
    compute(kt & 1);
    store_tiles((kt + 1) & 1);
    __syncthreads();
  }
  if (nk > 0) compute((nk - 1) & 1);

  // ---------------- epilogue -----------------------------------------------------
  // acc[i][j][r] is element (row, col) of the tile with
  //   row = wm*128 + i*32 + (r/4)*8 + lgrp*4 + r%4,  col = j*128 + wn*32 + lrow.
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = m0 + wm * 128 + i * 32 + (r >> 2) * 8 + lgrp * 4 + (r & 3);
      if (row >= m_end) continue;
      if constexpr (MODE == GATE_UP) {
        const int col = n0 + wn * 32 + lrow;
        if (col < a.N) {
          const float gv = acc[i][0][r], uv = acc[i][1][r];
          const float hv = gv / (1.0f + expf(-gv)) * uv;
          const size_t o = static_cast<size_t>(row) * a.N + col;
          a.O0[o] = f32_to_bf16(gv);
          a.O1[o] = f32_to_bf16(uv);
          a.O2[o] = f32_to_bf16(hv);
        }
      } else {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int col = n0 + j * 128 + wn * 32 + lrow;
          if (col >= a.N) continue;
          const float v = acc[i][j][r];
          if constexpr (MODE == DGRAD_H) {
            const size_t o = static_cast<size_t>(row) * a.N + col;
            const float gv = bf16_to_f32(a.G[o]), uv = bf16_to_f32(a.U[o]);
            const float s = 1.0f / (1.0f + expf(-gv));
            a.O0[o] = f32_to_bf16(v * uv * s * (1.0f + gv * (1.0f - s)));
            a.O1[o] = f32_to_bf16(v * gv * s);
          } else if constexpr (MODE == WGRAD) {
            a.O0[(static_cast<size_t>(e) * a.M + row) * a.N + col] = f32_to_bf16(v);
          } else {
            a.O0[static_cast<size_t>(row) * a.N + col] = f32_to_bf16(v);
          }
        }
      }
    }
  }
}

template <int MODE>
int launch_gemm(const GemmArgs& a, dim3 grid, hipStream_t s, const char* name) {
  static bool configured = false;
  if (!configured) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&grouped_gemm_kernel<MODE>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES) != hipSuccess) {
      (void)hipGetLastError();
      return MOE_ERR_LAUNCH;
    }
    configured = true;
  }
  MOE_LAUNCH(name, grouped_gemm_kernel<MODE>, grid, dim3(GEMM_THREADS), LDS_BYTES, s, a);
  return moe_check_launch();
}

bool bad_gemm_dims(int E, int R_cap, int d, int f) {
  return E <= 0 || E > MOE_MAX_EXPERTS || R_cap <= 0 || d <= 0 || f <= 0 || d % 64 != 0 || f % 64 != 0;
}

inline const uint16_t* U16(const moe_bf16* p) { return p; }

}  // namespace

extern "C" size_t moe_grouped_gemm_bwd_workspace_bytes(int R_cap, int f) {
  if (R_cap <= 0 || f <= 0) return 0;
  const size_t one = (static_cast<size_t>(R_cap) * f * sizeof(moe_bf16) + 255) & ~static_cast<size_t>(255);
  return 2 * one;
}

extern "C" size_t moe_workspace_bytes(int T, int E, int k, int d, int f) {
  (void)d;
  if (T <= 0 || k <= 0 || E <= 0) return 0;
  const size_t p = moe_permute_workspace_bytes(T, k, E);
  const size_t b = moe_grouped_gemm_bwd_workspace_bytes(T * k, f);
  return p > b ? p : b;
}

extern "C" int moe_grouped_gemm_fwd(const moe_bf16* xp, const int32_t* expert_offsets, const moe_bf16* Wg,
                                    const moe_bf16* Wu, const moe_bf16* Wd, int E, int R_cap, int d, int f,
                                    moe_bf16* g, moe_bf16* u, moe_bf16* h, moe_bf16* yp, void* stream) {
  if (!xp || !expert_offsets || !Wg || !Wu || !Wd || !g || !u || !h || !yp) return MOE_ERR_INVALID;
  if (bad_gemm_dims(E, R_cap, d, f)) return MOE_ERR_INVALID;
  const void* ptrs[] = {xp, expert_offsets, Wg, Wu, Wd, g, u, h, yp};
  for (const void* p : ptrs) if (!moe_aligned16(p)) return MOE_ERR_INVALID;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int m_tiles = R_cap / BM + E;

  GemmArgs a{};
  a.offsets = expert_offsets; a.E = E; a.m_tiles_cap = m_tiles;
  // gate | up with the SwiGLU epilogue
  a.A0 = U16(xp); a.B0 = U16(Wg); a.B1 = U16(Wu); a.O0 = g; a.O1 = u; a.O2 = h;
  a.K = d; a.N = f; a.n_tiles = (f + BN / 2 - 1) / (BN / 2);
  int rc = launch_gemm<GATE_UP>(a, dim3(a.n_tiles * m_tiles), s, "gemm_gate_up");
  if (rc != MOE_OK) return rc;
  // down
  GemmArgs b{};
  b.offsets = expert_offsets; b.E = E; b.m_tiles_cap = m_tiles;
  b.A0 = U16(h); b.B0 = U16(Wd); b.O0 = yp;
  b.K = f; b.N = d; b.n_tiles = (d + BN - 1) / BN;
  return launch_gemm<DOWN>(b, dim3(b.n_tiles * m_tiles), s, "gemm_down");
}

extern "C" int moe_grouped_gemm_bwd(const moe_bf16* dyp, const moe_bf16* xp, const moe_bf16* g, const moe_bf16* u,
                                    const moe_bf16* h, const int32_t* expert_offsets, const moe_bf16* Wg,
                                    const moe_bf16* Wu, const moe_bf16* Wd, int E, int R_cap, int d, int f,
                                    moe_bf16* dxp, moe_bf16* dWg, moe_bf16* dWu, moe_bf16* dWd, void* ws,
                                    size_t ws_bytes, void* stream) {
  if (!dyp || !xp || !g || !u || !h || !expert_offsets || !Wg || !Wu || !Wd || !dxp || !dWg || !dWu || !dWd || !ws)
    return MOE_ERR_INVALID;
  if (bad_gemm_dims(E, R_cap, d, f)) return MOE_ERR_INVALID;
  const void* ptrs[] = {dyp, xp, g, u, h, expert_offsets, Wg, Wu, Wd, dxp, dWg, dWu, dWd, ws};
  for (const void* p : ptrs) if (!moe_aligned16(p)) return MOE_ERR_INVALID;
  if (ws_bytes < moe_grouped_gemm_bwd_workspace_bytes(R_cap, f)) return MOE_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int m_tiles = R_cap / BM + E;
  uint16_t* dg = static_cast<uint16_t*>(ws);
  uint16_t* du = reinterpret_cast<uint16_t*>(static_cast<char*>(ws) + moe_grouped_gemm_bwd_workspace_bytes(R_cap, f) / 2);

  // dh = dyp . Wd, then the SwiGLU derivative -> dg, du
  GemmArgs a{};
  a.offsets = expert_offsets; a.E = E; a.m_tiles_cap = m_tiles;
  a.A0 = U16(dyp); a.B0 = U16(Wd); a.G = U16(g); a.U = U16(u); a.O0 = dg; a.O1 = du;
  a.K = d; a.N = f; a.n_tiles = (f + BN - 1) / BN;
  int rc = launch_gemm<DGRAD_H>(a, dim3(a.n_tiles * m_tiles), s, "gemm_dgrad_h");
  if (rc != MOE_OK) return rc;
  // dxp = dg . Wg + du . Wu
  GemmArgs b{};
  b.offsets = expert_offsets; b.E = E; b.m_tiles_cap = m_tiles;
  b.A0 = dg; b.A1 = du; b.B0 = U16(Wg); b.B1 = U16(Wu); b.O0 = dxp;
  b.K = f; b.N = d; b.n_tiles = (d + BN - 1) / BN;
  rc = launch_gemm<DGRAD_X>(b, dim3(b.n_tiles * m_tiles), s, "gemm_dgrad_x");
  if (rc != MOE_OK) return rc;
  // weight gradients: dWd = dyp^T h ; dWg = dg^T xp ; dWu = du^T xp
  struct W { const uint16_t* A; const uint16_t* B; uint16_t* O; int M, N; const char* name; };
  const W jobs[3] = {{U16(dyp), U16(h), dWd, d, f, "gemm_wgrad_down"},
                     {dg, U16(xp), dWg, f, d, "gemm_wgrad_gate"},
                     {du, U16(xp), dWu, f, d, "gemm_wgrad_up"}};
  for (const W& j : jobs) {
    GemmArgs w{};
    w.offsets = expert_offsets; w.E = E;
    w.A0 = j.A; w.B0 = j.B; w.O0 = j.O; w.M = j.M; w.N = j.N;
    w.n_tiles = (j.N + BN - 1) / BN;
    const int mt = (j.M + BM - 1) / BM;
    rc = launch_gemm<WGRAD>(w, dim3(w.n_tiles * mt, E), s, j.name);
    if (rc != MOE_OK) return rc;
  }
  return MOE_OK;
}
