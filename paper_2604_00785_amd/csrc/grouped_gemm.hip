// Stage 4 of Algorithm 1 (the three Grouped_mm calls around Silu(gate)*up) and
// its derivative, as grouped bf16 MFMA GEMMs: one launch covers every expert.
//
// One workgroup (8 waves) computes one 256x256 output tile with a 64-deep
// K step.  Both operand tiles live in LDS as [256 rows][64 k] bf16 (128 bytes
// per row, 16-byte pieces XOR-swizzled by the row so that the MFMA fragment
// reads and the fill writes spread over the banks), double-buffered: while the
// MFMAs consume one buffer, the next K step is fetched into the other one.
// The waves form a 2 (M) x 4 (N) grid; each owns a 128x64 piece = 4x2
// v_mfma_f32_32x32x16_bf16 accumulators (128 fp32 registers per lane).
//
// An operand that is contiguous along K in memory (activations [rows, K],
// forward weights [N, K]) is fetched with direct-to-LDS loads
// (global_load_lds_dwordx4): a wave instruction fills eight 128-byte LDS rows, and
// the swizzle is applied on the global side (which 16-byte piece a lane reads).
// An operand that is contiguous along the other dimension (weights in dgrad,
// both operands in wgrad) is transposed in registers on its way to LDS: a thread
// loads a 4 (k) x 8 (n) block with four 16-byte loads and writes eight 8-byte
// K-runs.
//
// The MFMAs are issued as (weight fragment) x (activation fragment), so a lane
// ends up with four consecutive output COLUMNS of one row.  The epilogue rounds
// to bf16, stages each wave's 128x64 piece in that wave's own 16 KB of LDS and
// writes it out in full 128-byte row segments; the SwiGLU forward and backward
// formulas are applied on the way, on the fp32 accumulators.
//
// Tiles of the row-grouped products are found on the device from
// expert_offsets: a workgroup turns its M-tile number into (expert, first row)
// with a wave-wide prefix sum over ceil(rows_e / 256); experts without rows own
// no tile; rows past an expert's end are clamped on load and masked on store.
#include <type_traits>
#include "common.h"

namespace {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int GEMM_THREADS = 512;
constexpr int TILE_BYTES = BM * BK * 2;              // one operand tile
constexpr int LDS_BYTES = 2 * 2 * TILE_BYTES;        // A and B, double-buffered
constexpr int WAVE_STAGE_BYTES = LDS_BYTES / 8;      // epilogue staging per wave (16 KB)

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
#define GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

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
  int m_tiles_cap;      // upper bound on row tiles (modes 0-3); row tiles of one dW (WGRAD)
  // WGRAD: out[e][M][N] = sum over the expert's rows of A[r][M] * B[r][N]
  int M;
};

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row ^ (row >> 3)) & 7); }

// K-strided operand: a thread stages k rows ks_kq*4 + j (j<4), columns ks_nb*8 .. +8.  Inside a
// group of 32 lanes nb takes 8 values and kq 4, so that one transposing LDS write spreads over
// 16 different 8-byte bank groups, and one global load covers 256 contiguous bytes of 4 rows.
struct Staged { u32x4 v[4]; };
__device__ __forceinline__ int ks_nb(int tid) { return ((tid >> 5) & 3) * 8 + (tid & 7); }
__device__ __forceinline__ int ks_kq(int tid) { return (tid >> 7) * 4 + ((tid >> 3) & 3); }

__device__ __forceinline__ void store_ks(const Staged& r, char* tile, int tid) {
  const int nb = ks_nb(tid), kq = ks_kq(tid);
  const int chunk = kq >> 1, half = kq & 1;
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const int row = nb * 8 + q;
    const uint32_t sel = (q & 1) ? 0x07060302u : 0x05040100u;
    u32x2 o;
    o.x = __builtin_amdgcn_perm(r.v[1][q >> 1], r.v[0][q >> 1], sel);  // k0 (low half), k1 (high half)
    o.y = __builtin_amdgcn_perm(r.v[3][q >> 1], r.v[2][q >> 1], sel);  // k2, k3
    *reinterpret_cast<u32x2*>(tile + row * 128 + swz(row, chunk) * 16 + half * 8) = o;
  }
}

// sigmoid through the hardware exp2 and reciprocal (each about 1 ulp): far inside bf16 rounding.
// exp2 overflows to +inf for very negative g and the reciprocal then returns 0, as it should.
__device__ __forceinline__ float sigmoid_f(float g) {
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g));
}
__device__ __forceinline__ float silu_f(float g) { return g * sigmoid_f(g); }

template <int MODE>
__global__ __launch_bounds__(GEMM_THREADS) void grouped_gemm_kernel(GemmArgs a) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  __shared__ int s_pref[MOE_MAX_EXPERTS + 1];   // exclusive prefix of row tiles per expert (modes 0-3)
  const int tid0 = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid0 >> 6);
  const int wm = wave >> 2, wn = wave & 3;

  // ---------------- tile list ---------------------------------------------------
  // The launch is persistent: gridDim.x workgroups (one per compute unit) walk the tile list.
  // Workgroups are dealt to the 8 XCDs round-robin, so workgroup b takes position
  // (b % 8) * (gridDim.x / 8) + b / 8 of every round: each XCD then works on a run of
  // consecutive tiles (same expert, neighbouring panels) that share its L2.
  int total;
  if constexpr (MODE == WGRAD) {
    total = a.E * a.m_tiles_cap * a.n_tiles;
  } else {
    if (wave == 0) {
      int base = 0;
      for (int e0 = 0; e0 < a.E; e0 += 64) {
        const int lane = tid0 & 63;
        const int ee = e0 + lane;
        const int rows = ee < a.E ? a.offsets[ee + 1] - a.offsets[ee] : 0;
        const int tiles = (rows + BM - 1) / BM;
        int inc = tiles;
#pragma unroll
        for (int s = 1; s < 64; s <<= 1) {
          const int v = __shfl_up(inc, s, 64);
          if (lane >= s) inc += v;
        }
        if (ee < a.E) s_pref[ee] = base + inc - tiles;
        base += __shfl(inc, 63, 64);
      }
      if ((tid0 & 63) == 0) s_pref[a.E] = base;
    }
    __syncthreads();
    total = s_pref[a.E] * a.n_tiles;
  }
  const int per_xcd = gridDim.x >> 3;
  const int first_tile = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);

  for (int tile = first_tile; tile < total; tile += gridDim.x) {
  // the thread id is laundered per tile so that lane-dependent address pieces are recomputed for
  // every tile instead of staying live (and spilling) across the whole loop
  int tid = tid0;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63;
  int e, m0, m_end;
  const int nt = tile % a.n_tiles;
  if constexpr (MODE == WGRAD) {
    const int rest = tile / a.n_tiles;
    e = rest / a.m_tiles_cap;
    m0 = (rest % a.m_tiles_cap) * BM;   // output row of dW
    m_end = a.M;
  } else {
    const int mt = tile / a.n_tiles;
    int lo = 0, hi = a.E;               // last expert whose first tile is <= mt
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (s_pref[mid] <= mt) lo = mid; else hi = mid;
    }
    e = lo;
    m0 = a.offsets[e] + (mt - s_pref[e]) * BM;
    m_end = a.offsets[e + 1];
  }
  const int n0 = nt * (MODE == GATE_UP ? BN / 2 : BN);
  // 32-row fragments of this wave that hold at least one valid row (the others are skipped)
  int nfa = (m_end - m0 - wm * 128 + 31) >> 5;
  nfa = nfa < 0 ? 0 : (nfa > 4 ? 4 : nfa);
  nfa = __builtin_amdgcn_readfirstlane(nfa);

  constexpr bool A_KS = (MODE == WGRAD);
  constexpr bool B_KS = (MODE == WGRAD || MODE == DGRAD_H || MODE == DGRAD_X);

  // ---------------- operand sources -------------------------------------------
  // A tile rows <-> output rows m0 + r ; B tile rows <-> output columns.
  // K-contiguous operands: wave w issues 4 direct-to-LDS loads per K step; load i fills LDS
  // rows (4w+i)*8 .. +8, lane l -> row + l/8, physical piece l%8, i.e. logical piece swz(row, l%8).
  const uint16_t* da[4];
  const uint16_t* db[4];
  const uint16_t* pa = nullptr;   // K-strided operands: this thread's column pointer
  const uint16_t* pb = nullptr;
  ptrdiff_t a_phase = 0, b_phase = 0;   // element offset of the second K phase (DGRAD_X)
  int k_lo = 0, k_hi = 0;               // WGRAD: the expert's row range is the reduction
  int nk;
  size_t lda = 0, ldb = 0;

  if constexpr (MODE == WGRAD) {
    k_lo = a.offsets[e];
    k_hi = a.offsets[e + 1];
    nk = (k_hi - k_lo + BK - 1) / BK;
    lda = a.M;
    ldb = a.N;
    const int nb = ks_nb(tid);
    int ca = m0 + nb * 8;  if (ca > a.M - 8) ca = a.M - 8;
    int cb = n0 + nb * 8;  if (cb > a.N - 8) cb = a.N - 8;
    pa = a.A0 + ca;
    pb = a.B0 + cb;
  } else {
    nk = a.K / BK;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = (wave * 4 + i) * 8 + (lane >> 3);
      const int piece = swz(row, lane & 7);
      int r = m0 + row;
      if (r > m_end - 1) r = m_end - 1;
      da[i] = a.A0 + static_cast<size_t>(r) * a.K + piece * 8;
    }
    if constexpr (MODE == DGRAD_X) { a_phase = a.A1 - a.A0; nk *= 2; }
    const size_t wsz = static_cast<size_t>(a.N) * a.K;
    if constexpr (!B_KS) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = (wave * 4 + i) * 8 + (lane >> 3);   // LDS row of the B tile
        const int piece = swz(row, lane & 7);
        const uint16_t* w = a.B0;
        int col = n0 + row;
        if constexpr (MODE == GATE_UP) {
          if (row >= BN / 2) { w = a.B1; col = n0 + row - BN / 2; }
        }
        if (col > a.N - 1) col = a.N - 1;
        db[i] = w + static_cast<size_t>(e) * wsz + static_cast<size_t>(col) * a.K + piece * 8;
      }
    } else {  // DGRAD_H / DGRAD_X: weights stored [K][N]
      ldb = a.N;
      int cb = n0 + ks_nb(tid) * 8;
      if (cb > a.N - 8) cb = a.N - 8;
      pb = a.B0 + static_cast<size_t>(e) * wsz + cb;
      if constexpr (MODE == DGRAD_X) b_phase = a.B1 - a.B0;
    }
  }

  Staged ra, rb;

  // Starts the fetch of K step kt into LDS buffer `buf`: direct-to-LDS loads land there by
  // themselves; K-strided operands arrive in ra / rb and are written by finish_fetch().
  auto start_fetch = [&](int kt, int buf) {
    int kk = kt;
    ptrdiff_t offa = 0, offb = 0;
    if constexpr (MODE == DGRAD_X) {
      const int half = nk >> 1;
      if (kt >= half) { kk = kt - half; offa = a_phase; offb = b_phase; }
    }
    char* ta = lds + buf * 2 * TILE_BYTES;
    char* tb = ta + TILE_BYTES;
    if constexpr (!A_KS) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        __builtin_amdgcn_global_load_lds(GLOBAL_PTR(da[i] + offa + static_cast<size_t>(kk) * BK),
                                         LDS_PTR(ta + (wave * 4 + i) * 1024), 16, 0, 0);
    }
    if constexpr (!B_KS) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        __builtin_amdgcn_global_load_lds(GLOBAL_PTR(db[i] + static_cast<size_t>(kk) * BK),
                                         LDS_PTR(tb + (wave * 4 + i) * 1024), 16, 0, 0);
    }
    const int kq = ks_kq(tid);
    if constexpr (A_KS) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int r = k_lo + kk * BK + kq * 4 + j;
        ra.v[j] = r < k_hi ? *reinterpret_cast<const u32x4*>(pa + static_cast<size_t>(r) * lda) : u32x4{0, 0, 0, 0};
      }
    }
    if constexpr (B_KS) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if constexpr (MODE == WGRAD) {
          const int r = k_lo + kk * BK + kq * 4 + j;
          rb.v[j] = r < k_hi ? *reinterpret_cast<const u32x4*>(pb + static_cast<size_t>(r) * ldb) : u32x4{0, 0, 0, 0};
        } else {
          const int r = kk * BK + kq * 4 + j;
          rb.v[j] = *reinterpret_cast<const u32x4*>(pb + offb + static_cast<size_t>(r) * ldb);
        }
      }
    }
  };
  auto finish_fetch = [&](int buf) {
    char* ta = lds + buf * 2 * TILE_BYTES;
    char* tb = ta + TILE_BYTES;
    if constexpr (A_KS) store_ks(ra, ta, tid);
    if constexpr (B_KS) store_ks(rb, tb, tid);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // direct-to-LDS loads have landed
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
  int arow[4], brow[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) arow[i] = wm * 128 + i * 32 + lrow;
#pragma unroll
  for (int j = 0; j < 2; ++j) brow[j] = (MODE == GATE_UP) ? j * 128 + wn * 32 + lrow : wn * 64 + j * 32 + lrow;

  // FULL: all four 32-row fragments of the wave are live (the common case, branch-free)
  auto compute = [&](int buf, auto full_tag) {
    constexpr bool FULL = decltype(full_tag)::value;
    const char* ta = lds + buf * 2 * TILE_BYTES;
    const char* tb = ta + TILE_BYTES;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8_t fa[4], fb[2];
      const int chunk = ks * 2 + lgrp;
#pragma unroll
      for (int j = 0; j < 2; ++j)
        fb[j] = *reinterpret_cast<const bf16x8_t*>(tb + brow[j] * 128 + swz(brow[j], chunk) * 16);
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (FULL || i < nfa) fa[i] = *reinterpret_cast<const bf16x8_t*>(ta + arow[i] * 128 + swz(arow[i], chunk) * 16);
      // weight fragment first: the lane then holds 4 consecutive output columns of one row
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (FULL || i < nfa) {
#pragma unroll
          for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
        }
    }
  };

  const int grow0 = m0 + wm * 128;                                   // wave's first output row
  const int gcol0 = n0 + wn * (MODE == GATE_UP ? 32 : 64);           // wave's first output column
  // DGRAD_H: saved g / u rows of one 64-row half of the wave's piece, 16 bytes per lane and pass
  u32x4 pg[8], pu[8];
  auto gu_load = [&](int hh) {
    if constexpr (MODE == DGRAD_H) {
#pragma unroll
      for (int p = 0; p < 8; ++p) {
        const int row = p * 8 + (lane >> 3), piece = lane & 7;
        int gr = grow0 + hh * 64 + row;  if (gr > m_end - 1) gr = m_end - 1;
        int gc = gcol0 + piece * 8;  if (gc > a.N - 8) gc = a.N - 8;
        const size_t o = static_cast<size_t>(gr) * a.N + gc;
        pg[p] = *reinterpret_cast<const u32x4*>(a.G + o);
        pu[p] = *reinterpret_cast<const u32x4*>(a.U + o);
      }
    }
  };

  if (nk > 0) {
    start_fetch(0, 0);
    finish_fetch(0);
  }
  __syncthreads();
  auto main_loop = [&](auto full_tag) {
    for (int kt = 0; kt + 1 < nk; ++kt) {
      start_fetch(kt + 1, (kt + 1) & 1);
      __builtin_amdgcn_sched_barrier(0);     // keep the fetch ahead of the math
      compute(kt & 1, full_tag);
      __builtin_amdgcn_sched_barrier(0);
      finish_fetch((kt + 1) & 1);
      __syncthreads();
    }
    gu_load(0);
    if (nk > 0) compute((nk - 1) & 1, full_tag);
  };
  if (nfa == 4) main_loop(std::true_type{}); else main_loop(std::false_type{});
  __syncthreads();                          // every wave is done with the operand tiles

  // ---------------- epilogue -----------------------------------------------------
  // acc[i][j][4q+c] is the wave's element (row, col) with row = i*32 + lrow and
  // col = j*32 + q*8 + lgrp*4 + c.  The wave stages bf16 rows of 128 bytes in its own
  // 16 KB of LDS (16-byte pieces swizzled by row & 7) and stores 16 bytes per lane.
  char* stage = lds + wave * WAVE_STAGE_BYTES;
  auto quad_addr = [&](int row, int piece) -> char* {
    return stage + row * 128 + ((piece ^ (row & 7)) << 4) + lgrp * 8;
  };
  auto put_quad = [&](int row, int piece, float v0, float v1, float v2, float v3) {
    u32x2 o;
    o.x = pack_bf16(v0, v1);
    o.y = pack_bf16(v2, v3);
    *reinterpret_cast<u32x2*>(quad_addr(row, piece)) = o;
  };
  // stores `rows` staged rows starting at staged row 0 to out (row stride ld); the first
  // `pieces` 16-byte pieces of each row go to columns col0 + piece*8 (pieces = 4 or 8)
  auto flush = [&](uint16_t* out, size_t ld, int first_row, int rows, int piece0, int pieces, int col0, int ncols) {
    const int rpp = 64 / pieces;                    // rows per pass
    for (int p = 0; p < rows / rpp; ++p) {
      const int row = p * rpp + lane / pieces;
      const int piece = lane % pieces;
      const u32x4 v = *reinterpret_cast<const u32x4*>(stage + row * 128 + (((piece0 + piece) ^ (row & 7)) << 4));
      const int gr = first_row + row, gc = col0 + piece * 8;
      if (gr < m_end && gc < ncols) *reinterpret_cast<u32x4*>(out + static_cast<size_t>(gr) * ld + gc) = v;
    }
  };

  if constexpr (MODE == GATE_UP) {
    // pass 1: g in pieces 0-3, u in pieces 4-7
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q)
          put_quad(i * 32 + lrow, j * 4 + q, acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
    __builtin_amdgcn_wave_barrier();
    flush(a.O0, a.N, grow0, 128, 0, 4, gcol0, a.N);
    flush(a.O1, a.N, grow0, 128, 4, 4, gcol0, a.N);
    __builtin_amdgcn_wave_barrier();
    // pass 2: h = silu(g) * u from the fp32 accumulators
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float h[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) h[c] = silu_f(acc[i][0][4 * q + c]) * acc[i][1][4 * q + c];
        put_quad(i * 32 + lrow, q, h[0], h[1], h[2], h[3]);
      }
    __builtin_amdgcn_wave_barrier();
    flush(a.O2, a.N, grow0, 128, 0, 4, gcol0, a.N);
  } else if constexpr (MODE == DGRAD_H) {
    // two halves of 64 rows: g rows at stage[0, 8K), u rows at stage[8K, 16K).  The g/u rows of
    // the first half were requested before the last K step, those of the second half are
    // requested before the first half is processed, so their latency stays hidden.
    char* ustage = stage + WAVE_STAGE_BYTES / 2;
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
      const int first = grow0 + hh * 64;
#pragma unroll
      for (int p = 0; p < 8; ++p) {
        const int row = p * 8 + (lane >> 3), piece = lane & 7;
        const int so = row * 128 + ((piece ^ (row & 7)) << 4);
        *reinterpret_cast<u32x4*>(stage + so) = pg[p];
        *reinterpret_cast<u32x4*>(ustage + so) = pu[p];
      }
      if (hh == 0) gu_load(1);
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int i2 = 0; i2 < 2; ++i2)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int row = i2 * 32 + lrow;
            char* ga = quad_addr(row, j * 4 + q);
            char* ua = ga + WAVE_STAGE_BYTES / 2;
            const u32x2 gq = *reinterpret_cast<const u32x2*>(ga);
            const u32x2 uq = *reinterpret_cast<const u32x2*>(ua);
            const float g4[4] = {bf16lo(gq.x), bf16hi(gq.x), bf16lo(gq.y), bf16hi(gq.y)};
            const float u4[4] = {bf16lo(uq.x), bf16hi(uq.x), bf16lo(uq.y), bf16hi(uq.y)};
            float dg[4], du[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
              const float dh = acc[hh * 2 + i2][j][4 * q + c];
              const float sg = sigmoid_f(g4[c]);
              dg[c] = dh * u4[c] * sg * (1.0f + g4[c] * (1.0f - sg));
              du[c] = dh * g4[c] * sg;
            }
            u32x2 o;
            o.x = pack_bf16(dg[0], dg[1]);  o.y = pack_bf16(dg[2], dg[3]);
            *reinterpret_cast<u32x2*>(ga) = o;
            o.x = pack_bf16(du[0], du[1]);  o.y = pack_bf16(du[2], du[3]);
            *reinterpret_cast<u32x2*>(ua) = o;
          }
      __builtin_amdgcn_wave_barrier();
      for (int p = 0; p < 8; ++p) {
        const int row = p * 8 + (lane >> 3), piece = lane & 7;
        const int so = row * 128 + ((piece ^ (row & 7)) << 4);
        const u32x4 dgv = *reinterpret_cast<const u32x4*>(stage + so);
        const u32x4 duv = *reinterpret_cast<const u32x4*>(ustage + so);
        const int gr = first + row, gc = gcol0 + piece * 8;
        if (gr < m_end && gc < a.N) {
          const size_t o = static_cast<size_t>(gr) * a.N + gc;
          *reinterpret_cast<u32x4*>(a.O0 + o) = dgv;
          *reinterpret_cast<u32x4*>(a.O1 + o) = duv;
        }
      }
      __builtin_amdgcn_wave_barrier();
    }
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q)
          put_quad(i * 32 + lrow, j * 4 + q, acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
    __builtin_amdgcn_wave_barrier();
    uint16_t* out = a.O0;
    if constexpr (MODE == WGRAD) out += static_cast<size_t>(e) * a.M * a.N;
    flush(out, a.N, grow0, 128, 0, 8, gcol0, a.N);
  }
  __syncthreads();   // the staging area becomes operand tiles again
  }  // tile loop
}

// Workgroups of the persistent launch: one per compute unit (the 128 KB of LDS allow no more),
// a multiple of 8 so that every XCD gets the same share, and no more than there can be tiles.
int persistent_grid(long long max_tiles) {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 8) {
      (void)hipGetLastError();
      n = 256;
    }
    cus = n & ~7;
  }
  long long g = (max_tiles + 7) & ~7ll;
  if (g > cus) g = cus;
  if (g < 8) g = 8;
  return static_cast<int>(g);
}

template <int MODE>
int launch_gemm(const GemmArgs& a, long long max_tiles, hipStream_t s, const char* name) {
  const dim3 grid(persistent_grid(max_tiles));
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
  int rc = launch_gemm<GATE_UP>(a, static_cast<long long>(a.n_tiles) * m_tiles, s, "gemm_gate_up");
  if (rc != MOE_OK) return rc;
  // down
  GemmArgs b{};
  b.offsets = expert_offsets; b.E = E; b.m_tiles_cap = m_tiles;
  b.A0 = U16(h); b.B0 = U16(Wd); b.O0 = yp;
  b.K = f; b.N = d; b.n_tiles = (d + BN - 1) / BN;
  return launch_gemm<DOWN>(b, static_cast<long long>(b.n_tiles) * m_tiles, s, "gemm_down");
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
  int rc = launch_gemm<DGRAD_H>(a, static_cast<long long>(a.n_tiles) * m_tiles, s, "gemm_dgrad_h");
  if (rc != MOE_OK) return rc;
  // weight gradients: dWg = dg^T xp ; dWu = du^T xp (dg, du still warm) ; dWd = dyp^T h
  struct W { const uint16_t* A; const uint16_t* B; uint16_t* O; int M, N; const char* name; };
  const W jobs[3] = {{dg, U16(xp), dWg, f, d, "gemm_wgrad_gate"},
                     {du, U16(xp), dWu, f, d, "gemm_wgrad_up"},
                     {U16(dyp), U16(h), dWd, d, f, "gemm_wgrad_down"}};
  for (const W& j : jobs) {
    GemmArgs w{};
    w.offsets = expert_offsets; w.E = E;
    w.A0 = j.A; w.B0 = j.B; w.O0 = j.O; w.M = j.M; w.N = j.N;
    w.n_tiles = (j.N + BN - 1) / BN;
    w.m_tiles_cap = (j.M + BM - 1) / BM;   // row tiles of one expert's dW
    rc = launch_gemm<WGRAD>(w, static_cast<long long>(w.n_tiles) * w.m_tiles_cap * E, s, j.name);
    if (rc != MOE_OK) return rc;
  }
  // dxp = dg . Wg + du . Wu  (last, so that the dx reduction that follows finds dxp in the last-level cache)
  GemmArgs b{};
  b.offsets = expert_offsets; b.E = E; b.m_tiles_cap = m_tiles;
  b.A0 = dg; b.A1 = du; b.B0 = U16(Wg); b.B1 = U16(Wu); b.O0 = dxp;
  b.K = f; b.N = d; b.n_tiles = (d + BN - 1) / BN;
  return launch_gemm<DGRAD_X>(b, static_cast<long long>(b.n_tiles) * m_tiles, s, "gemm_dgrad_x");
}
