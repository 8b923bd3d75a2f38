// Stage 4 of Algorithm 1 (the three Grouped_mm calls around Silu(gate)*up) and
// its derivative, as grouped bf16 MFMA GEMMs: one launch covers every expert.
//
// One workgroup (8 waves) computes one 256x256 output tile with a 64-deep K step.  The two
// operand tiles of a step (32 KB each) live in LDS, in a ring of five tile slots (160 KB, all
// there is): A(t) sits in slot 2t mod 5, B(t) in slot (2t+1) mod 5.  All operand traffic is
// direct-to-LDS (global_load_lds_dwordx4, eight per wave and step).  Two and a half steps fit,
// so after the barrier of step t the loads of B(t+2) go out first (they are needed one step
// later) and those of A(t+3) follow between the MFMAs (needed two steps later): the urgent
// half of a step's loads is then small enough for the texture path to deliver within the step.
// The waves form a 2 (M) x 4 (N) grid; each owns a 128x64
// piece = 4x2 v_mfma_f32_32x32x16_bf16 accumulators (128 fp32 registers per lane).
//
// What the main loop is built around: while the matrix pipe of a SIMD is saturated, vector-ALU
// instructions of either wave on that SIMD (address arithmetic for loads and LDS reads) are
// served very slowly, and everything queued behind them stalls.  So the loop contains no
// vector-ALU instruction at all: global loads use the scalar-base form (SGPR base that is
// advanced by scalar adds + a 32-bit per-lane offset computed once per tile), LDS fragment
// reads use per-lane addresses computed once per tile + immediate offsets (the K loop is
// unrolled by five, the period of the slot pattern, so that slots are compile-time constants).  MFMA fragments are
// double-buffered in registers: the LDS reads of the next 16-deep sub-step are issued before
// the MFMAs of the current one.  One s_barrier per step, placed before the last MFMA group,
// publishes the tiles that were awaited and frees the two slots that were just read.
//
// Tile layouts.  An operand that is contiguous along K in memory (activations [rows, K],
// forward weights [N, K]) is kept as [256 rows][64 k] with 128-byte rows whose eight 16-byte
// pieces are XOR-swizzled by the row, so that fragment reads (one ds_read_b128 per lane) spread
// over all banks; the swizzle is applied on the global side of the fill (which piece a lane
// fetches), since a direct-to-LDS load writes LDS linearly.  An operand that is contiguous
// along its other dimension (weights in dgrad, both operands in wgrad) is kept as it lies in
// memory, [64 k][256 n] with 512-byte rows, and read with the transposing LDS load
// ds_read_b64_tr_b16, two per fragment.
//
// The MFMAs are issued as (weight fragment) x (activation fragment), so a lane
// ends up with four consecutive output COLUMNS of one row.  The epilogue rounds
// to bf16, stages each wave's 128x64 piece in that wave's own 16 KB of LDS and
// writes it out in full 128-byte row segments; the SwiGLU forward and backward
// formulas are applied on the way, on the fp32 accumulators.
//
// Tiles of the row-grouped products are found on the device from
// expert_offsets: every wave turns the tile number into (expert, first row, column tile)
// with a wave-wide prefix sum over ceil(rows_e / 256) * column tiles (no LDS is left for a table);
// inside an expert the row tiles are innermost; experts without rows own no tile; rows past an
// expert's end are clamped on load and masked on store.
#include <type_traits>
#include "common.h"



namespace {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int GEMM_THREADS = 512;
constexpr int TILE_BYTES = BM * BK * 2;               // one operand tile (32 KB)
constexpr int NSLOT = 5;                              // ring of operand tile slots
constexpr int LDS_BYTES = NSLOT * TILE_BYTES;         // 160 KB: everything a workgroup can have
constexpr int WAVE_STAGE_BYTES = 16384;               // epilogue staging per wave
constexpr int slot_of_a(int p) { return (2 * p) % NSLOT; }       // p = step mod 5
constexpr int slot_of_b(int p) { return (2 * p + 1) % NSLOT; }

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef short s16x4 __attribute__((ext_vector_type(4)));
#define GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

enum GemmMode { GATE_UP = 0, DOWN = 1, DGRAD_H = 2, DGRAD_X = 3, WGRAD = 4, WGRAD_GATHER = 5, DGRAD_H_GATE = 6,
                WGRAD_GATHER_A = 7 };
// WGRAD_GATHER / WGRAD_GATHER_A: a weight gradient whose B / A operand rows are token rows found through
// row_token.  DGRAD_H_GATE: DGRAD_H for a forward pass that folded the gate weight into h: its A rows are
// rows of dout found through row_token, its epilogue scales by the row's gate weight and also emits the
// row's partial dot product with h = silu(g) u (the gradient of the gate weight).
constexpr bool is_wgrad(int mode) { return mode == WGRAD || mode == WGRAD_GATHER || mode == WGRAD_GATHER_A; }
constexpr bool is_dgrad_h(int mode) { return mode == DGRAD_H || mode == DGRAD_H_GATE; }

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
  const int32_t* row_token;   // not null: rows of the activation operand are gathered, row r lies at A0[row_token[r]]
                              // (GATE_UP, DGRAD_H_GATE, WGRAD_GATHER_A: the A operand; WGRAD_GATHER: the B operand)
  const float* row_weight;    // GATE_UP: not null = h is scaled by the row's gate weight; DGRAD_H_GATE: required
  float* dgate_part;          // DGRAD_H_GATE: [R_cap][N / 64] partial dot products, one per row and 64-column strip
  int E;
  int K;                // reduction length of one phase (modes 0-3)
  int N;                // output columns (per half for GATE_UP)
  int n_tiles;          // column tiles
  int m_tiles_cap;      // upper bound on row tiles (modes 0-3); row tiles of one dW (WGRAD)
  // WGRAD: out[e][M][N] = sum over the expert's rows of A[r][M] * B[r][N]
  int M;
};

// 512 bytes of zeros: what the reduction rows past an expert's end read in the weight-gradient products.
__device__ __attribute__((aligned(512))) uint32_t g_zero_block[128];

// [256 rows][64 k] tile: byte offset of the 16-byte piece `chunk` (0..7) of `row`.
__device__ __forceinline__ int kc_off(int row, int chunk) {
  return row * 128 + ((chunk ^ ((row ^ (row >> 3)) & 7)) << 4);
}
// [64 k][256 n] tile: 16-byte pieces of a k row are XOR-swizzled with 4*(k & 3), which spreads the
// four k rows that 16 lanes of a transposing read touch over four different 64-byte bank groups.
__device__ __forceinline__ int kn_piece(int krow, int piece) { return piece ^ ((krow & 3) << 2); }

// LDS fragment reads are written as inline assembly with immediate offsets and awaited by hand
// (lds_wait): the fragments are read one sub-step ahead, across the loop back edge, and the
// compiler's own wait insertion would drain the LDS queue completely at the first use.
template <int OFF> __device__ __forceinline__ bf16x8_t lds_read_b128(uint32_t addr) {
  bf16x8_t v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
  return v;
}
template <int OFF> __device__ __forceinline__ s16x4 lds_read_tr_b64(uint32_t addr) {
  s16x4 v;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
  return v;
}
// Direct-to-LDS loads (16 bytes per lane, lane l lands at lds_addr + 16 l) are written as inline
// assembly too, so that the (scalar base) + (32-bit lane offset) form is certain: with 64-bit lane
// addresses every load needs vector-ALU work.  M0 carries the LDS address; nothing else in this
// file uses M0.
template <int OFF> __device__ __forceinline__ void dma16(uint32_t lds_base, uint32_t voff, const char* sbase) {
  asm volatile("s_add_i32 m0, %0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(lds_base), "v"(voff), "s"(sbase), "n"(OFF) : "memory", "scc");
}
template <int OFF> __device__ __forceinline__ void dma16_lane(uint32_t lds_base, const char* p) {
  asm volatile("s_add_i32 m0, %0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
               :: "s"(lds_base), "v"(p), "n"(OFF) : "memory", "scc");
}
// A 4-byte load as (scalar base) + (32-bit lane offset) + immediate, awaited by hand like the loads
// above (the compiler's own wait would count only the loads it knows of and so drain the whole queue).
template <int OFF> __device__ __forceinline__ int load_i32(uint32_t voff, const int32_t* sbase) {
  int v;
  asm volatile("global_load_dword %0, %1, %2 offset:%3" : "=v"(v) : "v"(voff), "s"(sbase), "n"(OFF) : "memory");
  return v;
}
template <int N> __device__ __forceinline__ void lds_wait() { asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory"); }

// Per-lane address of a fragment (32 tile columns starting at col0) of a [64 k][256 n] tile at
// LDS address `tile`, K sub-step 0, first half.  Within 16 lanes, lane i supplies the address of
// four consecutive n of k row i/4, n block i%4, and lane l receives k rows 0..3 of column l; two
// such loads (the second 4 k rows = 2048 bytes further) give the eight consecutive k of a column,
// and sub-step ks lies ks * 8192 bytes further.
__device__ __forceinline__ uint32_t kn_frag_addr(uint32_t tile, int col0, int lane) {
  const int i = lane & 15, kg = lane >> 5;
  const int n = col0 + ((lane >> 4) & 1) * 16 + 4 * (i & 3);
  const int krow = kg * 8 + (i >> 2);
  return tile + krow * 512 + kn_piece(krow, n >> 3) * 16 + (n & 7) * 2;
}
template <int OFF> __device__ __forceinline__ bf16x8_t lds_read_kn(uint32_t addr) {
  union { s16x4 h[2]; bf16x8_t v; } u;
  u.h[0] = lds_read_tr_b64<OFF>(addr);
  u.h[1] = lds_read_tr_b64<OFF + 2048>(addr);
  return u.v;
}

// sigmoid through the hardware exp2 and reciprocal (each about 1 ulp): far inside bf16 rounding.
// exp2 overflows to +inf for very negative g and the reciprocal then returns 0, as it should.
__device__ __forceinline__ float sigmoid_f(float g) {
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g));
}
__device__ __forceinline__ float silu_f(float g) { return g * sigmoid_f(g); }

template <int N> __device__ __forceinline__ void wait_vm() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }
__device__ __forceinline__ void wg_barrier() {
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_sched_barrier(0);
}

// Row tiles of the grouped products: expert e owns ceil(rows_e / 256) consecutive tile numbers.
// Both functions are evaluated by a whole wave (64 experts per pass) and return wave-uniform values.
__device__ __forceinline__ int wave_incl_scan(int v, int lane) {
#pragma unroll
  for (int s = 1; s < 64; s <<= 1) {
    const int u = __shfl_up(v, s, 64);
    if (lane >= s) v += u;
  }
  return v;
}
__device__ __forceinline__ int count_row_tiles(const int32_t* offsets, int E, int lane) {
  int total = 0;
  for (int e0 = 0; e0 < E; e0 += 64) {
    const int ee = e0 + lane;
    const int rows = ee < E ? offsets[ee + 1] - offsets[ee] : 0;
    total += __shfl(wave_incl_scan((rows + BM - 1) / BM, lane), 63, 64);
  }
  return __builtin_amdgcn_readfirstlane(total);
}
// Tile number `tile` of a row-grouped product -> expert, first row, column tile.  An expert's tiles are
// numbered column tile by column tile, its row tiles innermost: the workgroups of an XCD, which take a
// run of consecutive tiles, then share each weight panel among all row tiles of the expert at the same
// time, so that it is fetched from memory once (weights are the larger operand and are used by only
// rows_e / 256 tiles each; activations of a row tile recur every rows_e / 256 tiles).
// With at most 64 experts the lane's two offsets are read once per kernel (lo0, hi0) instead of once
// per tile: the lookup then needs no memory access, which would otherwise sit in front of every
// tile's first loads.
__device__ __forceinline__ void find_tile(const int32_t* offsets, int E, int lo0, int hi0, int n_tiles, int tile, int lane,
                                          int& e, int& m0, int& m_end, int& nt) {
  int base = 0;
  e = 0; m0 = 0; m_end = 0; nt = 0;
  for (int e0 = 0; e0 < E; e0 += 64) {
    const int ee = e0 + lane;
    int lo, hi;
    if (E <= 64) { lo = lo0; hi = hi0; }
    else { lo = ee < E ? offsets[ee] : 0; hi = ee < E ? offsets[ee + 1] : 0; }
    const int row_tiles = (hi - lo + BM - 1) / BM;
    const int tiles = row_tiles * n_tiles;
    const int inc = wave_incl_scan(tiles, lane);
    const int excl = base + inc - tiles;
    const unsigned long long hit = __ballot(tiles > 0 && excl <= tile && tile < excl + tiles);
    if (hit) {
      const int l = __ffsll(hit) - 1;
      e = e0 + l;
      const int q = tile - __shfl(excl, l, 64);
      const int rt = __shfl(row_tiles, l, 64);
      nt = q / rt;
      m0 = __shfl(lo, l, 64) + (q - nt * rt) * BM;
      m_end = __shfl(hi, l, 64);
      return;
    }
    base += __shfl(inc, 63, 64);
  }
}

// The kernel arguments again, through a pointer the compiler cannot see through: what is read from
// it is loaded afresh (scalar loads from the argument segment) instead of being kept in scalar
// registers across the main loop, which needs them for itself.
typedef const __attribute__((address_space(4))) GemmArgs* ArgPtr;
template <int ARG> __device__ __forceinline__ ArgPtr reload_args() {   // ARG: which of the kernel's GemmArgs
  ArgPtr p = (ArgPtr)__builtin_amdgcn_kernarg_segment_ptr() + ARG;
  asm volatile("" : "+s"(p));
  return p;
}

// One product's tile list, walked by this workgroup from list position first_tile in steps of
// gridDim.x.  Returns the position at which the workgroup left the list, counted from its end:
// where it enters a list that follows in the same launch.
template <int MODE, int ARG>
__device__ __forceinline__ int gemm_tile_list(const GemmArgs& a, int first_tile) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int tid0 = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid0 >> 6);
  const int wm = wave >> 2, wn = wave & 3;

  // ---------------- tile list ---------------------------------------------------
  int total;
  int lo0 = 0, hi0 = 0;   // this lane's expert's row range, kept for the whole kernel when E <= 64
  // WGRAD / WGRAD_GATHER with a second A operand (A1 -> O1): two weight gradients that share their B
  // operand in one launch; an expert's tiles of the first come before its tiles of the second
  int wpair = 1;
  if constexpr (MODE == WGRAD_GATHER || MODE == WGRAD) wpair = a.A1 != nullptr ? 2 : 1;
  if constexpr (is_wgrad(MODE)) {
    total = a.E * a.m_tiles_cap * a.n_tiles * wpair;
  } else {
    total = count_row_tiles(a.offsets, a.E, tid0 & 63) * a.n_tiles;
    if (a.E <= 64 && (tid0 & 63) < a.E) { lo0 = a.offsets[tid0 & 63]; hi0 = a.offsets[(tid0 & 63) + 1]; }
  }
  int tile = first_tile;
  for (; tile < total; tile += gridDim.x) {
  // the thread id is laundered per tile so that lane-dependent address pieces are recomputed for
  // every tile instead of staying live (and spilling) across the whole loop
  int tid = tid0;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63;
  int e, m0, m_end, nt;
  bool second = false;                  // tile of the second weight gradient of a pair
  if constexpr (is_wgrad(MODE)) {
    nt = tile % a.n_tiles;
    const int rest = tile / a.n_tiles;
    const int per_expert = a.m_tiles_cap * wpair;
    e = rest / per_expert;
    int mi = rest % per_expert;
    if (mi >= a.m_tiles_cap) { mi -= a.m_tiles_cap; second = true; }
    m0 = mi * BM;                       // output row of dW
    m_end = a.M;
  } else {
    find_tile(a.offsets, a.E, lo0, hi0, a.n_tiles, tile, lane, e, m0, m_end, nt);
    nt = __builtin_amdgcn_readfirstlane(nt);
  }
  // tile coordinates are wave-uniform: keep them in scalar registers, so that everything derived
  // from them (operand base addresses in particular) is scalar too
  e = __builtin_amdgcn_readfirstlane(e);
  m0 = __builtin_amdgcn_readfirstlane(m0);
  m_end = __builtin_amdgcn_readfirstlane(m_end);
  const int n0 = nt * (MODE == GATE_UP ? BN / 2 : BN);
  // 32-row fragments of this wave that hold at least one valid row (the others are skipped)
  int nfa = (m_end - m0 - wm * 128 + 31) >> 5;
  nfa = nfa < 0 ? 0 : (nfa > 4 ? 4 : nfa);
  nfa = __builtin_amdgcn_readfirstlane(nfa);

  // The 32 tile rows this wave loads of every activation tile (rows 32 * wave ..) are one fragment of
  // some wave; if none of them is a valid row nobody reads them, and the wave skips those loads
  // (a row tile with few rows is bound by its loads, not by its MFMAs).
  bool a_live = true;
  if constexpr (!is_wgrad(MODE)) a_live = wave * 32 < m_end - m0;

  constexpr bool A_KN = is_wgrad(MODE);                                       // stored [k][m]
  constexpr bool B_KN = (is_wgrad(MODE) || is_dgrad_h(MODE) || MODE == DGRAD_X);  // stored [k][n]

  // ---------------- operand sources -------------------------------------------
  // A tile <-> output rows m0 + r ; B tile <-> output columns.  Per step and operand a wave issues
  // four direct-to-LDS loads of 1 KB each, as (scalar base) + (32-bit lane offset):
  //  K-contiguous source ([row][k]): load i of wave w fills LDS rows (4w+i)*8 .. +8 of the tile;
  //    lane l -> row + l/8, physical piece l%8, i.e. the logical piece that kc_off maps there.
  //    The base advances by 64 elements per step.
  //  n-contiguous source ([k][n]): load i of wave w fills k rows (4w+i)*2, +1 of the tile;
  //    lane l -> k row + l/32, physical piece l%32 = logical piece kn_piece(k row, l%32).
  //    The base advances by 64 rows per step.
  uint32_t voa[4], vob[4];              // lane offsets in bytes
  const char* abase;                    // step 0 of phase 0
  const char* bbase;
  ptrdiff_t a_phase = 0, b_phase = 0;   // byte offset of the second K phase (DGRAD_X)
  size_t a_step, b_step;                // bytes per step
  int k_lo = 0, k_hi = 0;               // WGRAD: the expert's row range is the reduction
  constexpr bool GATHER_B = (MODE == WGRAD_GATHER);
  constexpr bool GATHER_A = (MODE == WGRAD_GATHER_A);
  const int32_t* row_tok = nullptr;     // GATHER_A/B: token of the expert's first reduction row onwards
  uint32_t vcb[4] = {0, 0, 0, 0};       // GATHER_A/B: byte offset of the lane's columns within a token row
  int tokn[4] = {0, 0, 0, 0};           // GATHER_A/B: tokens of the lane's four reduction rows of a coming step
  int tokn1[4] = {0, 0, 0, 0};          // the same for step 1, while a tile's first loads are set up
  int nk, nk_phase;                     // steps in total / in the first K phase

  if constexpr (is_wgrad(MODE)) {
    k_lo = __builtin_amdgcn_readfirstlane(a.offsets[e]);
    k_hi = __builtin_amdgcn_readfirstlane(a.offsets[e + 1]);
    nk = (k_hi - k_lo + BK - 1) / BK;
    nk_phase = nk;
    if constexpr (GATHER_A) {
      abase = reinterpret_cast<const char*>(a.A0 + m0);
      a_step = 0;
      row_tok = a.row_token + k_lo;
    } else {
      abase = reinterpret_cast<const char*>((second ? a.A1 : a.A0) + static_cast<size_t>(k_lo) * a.M + m0);
      a_step = static_cast<size_t>(BK) * a.M * 2;
    }
    if constexpr (GATHER_B) {
      // the base stays at the first token row; a load's lane offset carries its token (set per step)
      bbase = reinterpret_cast<const char*>(a.B0 + n0);
      b_step = 0;
      row_tok = a.row_token + k_lo;
    } else {
      bbase = reinterpret_cast<const char*>(a.B0 + static_cast<size_t>(k_lo) * a.N + n0);
      b_step = static_cast<size_t>(BK) * a.N * 2;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int krow = (wave * 4 + i) * 2 + (lane >> 5);
      const int piece = kn_piece(krow, lane & 31);
      int ca = piece * 8;  if (m0 + ca > a.M - 8) ca = a.M - 8 - m0;
      int cb = piece * 8;  if (n0 + cb > a.N - 8) cb = a.N - 8 - n0;
      voa[i] = static_cast<uint32_t>((krow * a.M + ca) * 2);
      vob[i] = static_cast<uint32_t>((krow * a.N + cb) * 2);
      if constexpr (GATHER_B) vcb[i] = static_cast<uint32_t>(cb * 2);
      if constexpr (GATHER_A) vcb[i] = static_cast<uint32_t>(ca * 2);
    }
  } else {
    nk = a.K / BK;
    nk_phase = nk;
    abase = reinterpret_cast<const char*>(a.A0 + static_cast<size_t>(m0) * a.K);
    a_step = BK * 2;
    bool gathered = false;
    if constexpr (MODE == GATE_UP) gathered = a.row_token != nullptr;
    if constexpr (MODE == DGRAD_H_GATE) gathered = true;
    if (gathered) abase = reinterpret_cast<const char*>(a.A0);   // lane offsets carry the token row
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = (wave * 4 + i) * 8 + (lane >> 3);
      const int chunk = (kc_off(row, lane & 7) >> 4) & 7;   // the swizzle is its own inverse
      int r = row;
      if (m0 + r > m_end - 1) r = m_end - 1 - m0;
      if (gathered) voa[i] = (static_cast<uint32_t>(a.row_token[m0 + r]) * a.K + chunk * 8) * 2u;
      else voa[i] = static_cast<uint32_t>((r * a.K + chunk * 8) * 2);
    }
    if constexpr (MODE == DGRAD_X) { a_phase = (a.A1 - a.A0) * 2; nk *= 2; }
    const size_t wsz = static_cast<size_t>(a.N) * a.K;
    if constexpr (!B_KN) {
      // GATE_UP: LDS rows 0..127 hold Wg rows n0.., rows 128..255 hold Wu rows n0.. (waves 4-7 fill those)
      const uint16_t* w = a.B0;
      int rsub = 0;
      if constexpr (MODE == GATE_UP) {
        if (wave >= 4) { w = a.B1; rsub = BN / 2; }
      }
      bbase = reinterpret_cast<const char*>(w + static_cast<size_t>(e) * wsz + static_cast<size_t>(n0) * a.K);
      b_step = BK * 2;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = (wave * 4 + i) * 8 + (lane >> 3);   // LDS row of the B tile
        const int chunk = (kc_off(row, lane & 7) >> 4) & 7;
        int col = row - rsub;
        if (n0 + col > a.N - 1) col = a.N - 1 - n0;
        vob[i] = static_cast<uint32_t>((col * a.K + chunk * 8) * 2);
      }
    } else {  // DGRAD_H / DGRAD_X: weights stored [K][N]
      bbase = reinterpret_cast<const char*>(a.B0 + static_cast<size_t>(e) * wsz + n0);
      b_step = static_cast<size_t>(BK) * a.N * 2;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int krow = (wave * 4 + i) * 2 + (lane >> 5);
        int cb = kn_piece(krow, lane & 31) * 8;
        if (n0 + cb > a.N - 8) cb = a.N - 8 - n0;
        vob[i] = static_cast<uint32_t>((krow * a.N + cb) * 2);
      }
      if constexpr (MODE == DGRAD_X) b_phase = (a.B1 - a.B0) * 2;
    }
  }

  // Both bases live in scalar registers and are advanced by scalar adds: steps are loaded in order.
  auto scalarize = [](const char* p) __attribute__((always_inline)) {
    const uint64_t u = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(u));
    const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(u >> 32));
    return reinterpret_cast<const char*>((static_cast<uint64_t>(hi) << 32) | lo);
  };
  const uint32_t lds_fill = __builtin_amdgcn_readfirstlane(
      static_cast<uint32_t>(reinterpret_cast<size_t>(LDS_PTR(lds))) + wave * 4096);   // this wave's share of a tile
  const char* sa_next = scalarize(abase);
  const char* sb_next = scalarize(bbase);
  const char* sa_phase1 = nullptr;
  const char* sb_phase1 = nullptr;
  if constexpr (MODE == DGRAD_X) { sa_phase1 = scalarize(abase + a_phase); sb_phase1 = scalarize(bbase + b_phase); }

  // Loads come per operand tile ("unit"), in order of the steps: part i of a unit is this wave's
  // i-th load of it, unit_end advances the operand's running base.
  using J0 = std::integral_constant<int, 0>;
  using J1 = std::integral_constant<int, 1>;
  using J2 = std::integral_constant<int, 2>;
  using J3 = std::integral_constant<int, 3>;
  auto a_part = [&](int kt, auto slot_tag, auto i_tag) __attribute__((always_inline)) {
    constexpr int SLOT = decltype(slot_tag)::value, i = decltype(i_tag)::value;
    constexpr int OFF = SLOT * TILE_BYTES + i * 1024;
    if constexpr (GATHER_A) {
      dma16<OFF>(lds_fill, voa[i], sa_next);   // rows past the expert's end were clamped when their tokens were fetched
    } else if constexpr (is_wgrad(MODE)) {
      if (k_lo + (kt + 1) * BK > k_hi) {
        // last, partial step of the expert: reduction rows at or past its end read zeros
        // (per-lane 64-bit addresses; once per tile)
        const int krow = k_lo + kt * BK + (wave * 4 + i) * 2 + (lane >> 5);
        dma16_lane<OFF>(lds_fill, krow < k_hi ? sa_next + voa[i]
                                   : reinterpret_cast<const char*>(g_zero_block) + (lane & 31) * 16);
      } else {
        dma16<OFF>(lds_fill, voa[i], sa_next);
      }
    } else {
      dma16<OFF>(lds_fill, voa[i], sa_next);
    }
  };
  auto b_part = [&](int kt, auto slot_tag, auto i_tag) __attribute__((always_inline)) {
    constexpr int SLOT = decltype(slot_tag)::value, i = decltype(i_tag)::value;
    constexpr int OFF = SLOT * TILE_BYTES + i * 1024;
    if constexpr (GATHER_B) {
      dma16<OFF>(lds_fill, vob[i], sb_next);   // rows past the expert's end were clamped when their tokens were fetched
    } else if constexpr (GATHER_A) {
      if (k_lo + (kt + 1) * BK > k_hi) {
        // the gathered operand repeats the expert's last row past its end: this one reads zeros there
        const int krow = k_lo + kt * BK + (wave * 4 + i) * 2 + (lane >> 5);
        dma16_lane<OFF>(lds_fill, krow < k_hi ? sb_next + vob[i]
                                   : reinterpret_cast<const char*>(g_zero_block) + (lane & 31) * 16);
      } else {
        dma16<OFF>(lds_fill, vob[i], sb_next);
      }
    } else if constexpr (MODE == WGRAD) {
      if (k_lo + (kt + 1) * BK > k_hi) {
        // ... and the other operand reads its last valid row there, so that zero times it is zero
        const int krow = k_lo + kt * BK + (wave * 4 + i) * 2 + (lane >> 5);
        dma16_lane<OFF>(lds_fill, sb_next + vob[i] - (krow < k_hi ? 0 : static_cast<size_t>(krow - (k_hi - 1)) * a.N * 2));
      } else {
        dma16<OFF>(lds_fill, vob[i], sb_next);
      }
    } else {
      dma16<OFF>(lds_fill, vob[i], sb_next);
    }
  };
  auto a_end = [&](int kt) __attribute__((always_inline)) {
    sa_next += a_step;
    if constexpr (MODE == DGRAD_X) {
      if (kt + 1 == nk_phase) sa_next = sa_phase1;
    }
  };
  auto b_end = [&](int kt) __attribute__((always_inline)) {
    sb_next += b_step;
    if constexpr (MODE == DGRAD_X) {
      if (kt + 1 == nk_phase) sb_next = sb_phase1;
    }
  };
  // GATHER_B: the tokens of the lane's four reduction rows of step kt, loaded without any vector-ALU
  // work except in an expert's last, partial step (rows past its end repeat its last row: the other
  // operand is zero there), and their turn into lane offsets of the B loads.  The loads are asynchronous:
  // apply_tok may only run after a wait that covers them.
  const uint32_t tok_voff = static_cast<uint32_t>(((wave * 4) * 2 + (lane >> 5)) * 4);   // row of load 0; load i: + 2 i rows
  auto fetch_tok = [&](int kt, int (&tk)[4]) __attribute__((always_inline)) {
    if constexpr (GATHER_B || GATHER_A) {
      if (k_lo + (kt + 1) * BK > k_hi) {
        const int last = k_hi - k_lo - 1;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          int r = kt * BK + (wave * 4 + i) * 2 + (lane >> 5);
          if (r > last) r = last;
          tk[i] = load_i32<0>(static_cast<uint32_t>(r) * 4u, row_tok);
        }
      } else {
        const int32_t* base = row_tok + static_cast<size_t>(kt) * BK;
        tk[0] = load_i32<0>(tok_voff, base);
        tk[1] = load_i32<8>(tok_voff, base);
        tk[2] = load_i32<16>(tok_voff, base);
        tk[3] = load_i32<24>(tok_voff, base);
      }
    }
  };
  auto apply_tok = [&](int (&tk)[4]) __attribute__((always_inline)) {
    if constexpr (GATHER_B || GATHER_A) {
      const uint32_t row_bytes = static_cast<uint32_t>(GATHER_B ? a.N : a.M) * 2u;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        asm volatile("" : "+v"(tk[i]));   // not before the wait that precedes this call
        const uint32_t off = static_cast<uint32_t>(tk[i]) * row_bytes + vcb[i];
        if constexpr (GATHER_B) vob[i] = off; else voa[i] = off;
      }
    }
  };
  auto a_unit = [&](int kt, auto slot_tag) __attribute__((always_inline)) {
    a_part(kt, slot_tag, J0{}); a_part(kt, slot_tag, J1{}); a_part(kt, slot_tag, J2{}); a_part(kt, slot_tag, J3{});
    a_end(kt);
  };
  auto b_unit = [&](int kt, auto slot_tag) __attribute__((always_inline)) {
    b_part(kt, slot_tag, J0{}); b_part(kt, slot_tag, J1{}); b_part(kt, slot_tag, J2{}); b_part(kt, slot_tag, J3{});
    b_end(kt);
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
  const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<size_t>(LDS_PTR(lds)));
  // Per-lane fragment addresses.  Slot, fragment and sub-step are immediate offsets of the LDS
  // reads, which reach 64 KB: one set of addresses serves slots 0-1, one slots 2-3, one slot 4.
  //  [row][k] tile: an address per sub-step, for the wave's first fragment.  Fragment i lies
  //    32 i rows = 4096 i bytes further, and an odd i flips bit 2 of the row swizzle, which is the
  //    same as taking sub-step ks ^ 2.
  //  [k][n] tile: an address per fragment (its swizzle depends on the column block); sub-step and
  //    half are immediates.
  const int b_row0 = (MODE == GATE_UP) ? wn * 32 : wn * 64;
  uint32_t fa_base[3][4], fb_base[3][B_KN ? 2 : 4];
#pragma unroll
  for (int st = 0; st < 3; ++st) {
    const uint32_t org = lds0 + st * 2 * TILE_BYTES;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if constexpr (A_KN) fa_base[st][q] = kn_frag_addr(org, wm * 128 + q * 32, lane);
      else fa_base[st][q] = org + kc_off(wm * 128 + lrow, q * 2 + lgrp);
    }
    if constexpr (B_KN) {
      fb_base[st][0] = kn_frag_addr(org, b_row0, lane);
      fb_base[st][1] = kn_frag_addr(org, b_row0 + 32, lane);
    } else {
#pragma unroll
      for (int q = 0; q < 4; ++q) fb_base[st][q] = org + kc_off(b_row0 + lrow, q * 2 + lgrp);
    }
  }

  bf16x8_t fa[2][4], fb[2][2];   // two fragment sets: one feeds the MFMAs while the other is being read
  // LDS read instructions per fragment set when NFA activation fragments are live (none at all for NFA = 0)
  constexpr auto nreads = [](int nfa) { return nfa == 0 ? 0 : (A_KN ? 2 : 1) * nfa + (B_KN ? 4 : 2); };
  // Reads sub-step KS of the tiles in slots SA (A) and SB (B) into fragment set SET.  Activation
  // fragments without a valid row are not read: nothing would keep their registers reserved until
  // the data lands.
  auto read_frags = [&](auto sa_tag, auto sb_tag, auto ks_tag, auto set_tag, auto full_tag) __attribute__((always_inline)) {
    constexpr int NFA = decltype(full_tag)::value;
    if constexpr (NFA == 0) return;
    constexpr int SA = decltype(sa_tag)::value, SB = decltype(sb_tag)::value;
    constexpr int KS = decltype(ks_tag)::value, SET = decltype(set_tag)::value;
    constexpr int OA = (SA & 1) * TILE_BYTES, OB = (SB & 1) * TILE_BYTES;
    if constexpr (B_KN) {
      fb[SET][0] = lds_read_kn<OB + KS * 8192>(fb_base[SB >> 1][0]);
      fb[SET][1] = lds_read_kn<OB + KS * 8192>(fb_base[SB >> 1][1]);
    } else if constexpr (MODE == GATE_UP) {   // second fragment: the up half, 128 tile rows further
      fb[SET][0] = lds_read_b128<OB>(fb_base[SB >> 1][KS]);
      fb[SET][1] = lds_read_b128<OB + 128 * 128>(fb_base[SB >> 1][KS]);
    } else {
      fb[SET][0] = lds_read_b128<OB>(fb_base[SB >> 1][KS]);
      fb[SET][1] = lds_read_b128<OB + 4096>(fb_base[SB >> 1][KS ^ 2]);
    }
    if constexpr (A_KN) {
      if constexpr (NFA > 0) fa[SET][0] = lds_read_kn<OA + KS * 8192>(fa_base[SA >> 1][0]);
      if constexpr (NFA > 1) fa[SET][1] = lds_read_kn<OA + KS * 8192>(fa_base[SA >> 1][1]);
      if constexpr (NFA > 2) fa[SET][2] = lds_read_kn<OA + KS * 8192>(fa_base[SA >> 1][2]);
      if constexpr (NFA > 3) fa[SET][3] = lds_read_kn<OA + KS * 8192>(fa_base[SA >> 1][3]);
    } else {
      if constexpr (NFA > 0) fa[SET][0] = lds_read_b128<OA>(fa_base[SA >> 1][KS]);
      if constexpr (NFA > 1) fa[SET][1] = lds_read_b128<OA + 4096>(fa_base[SA >> 1][KS ^ 2]);
      if constexpr (NFA > 2) fa[SET][2] = lds_read_b128<OA + 8192>(fa_base[SA >> 1][KS]);
      if constexpr (NFA > 3) fa[SET][3] = lds_read_b128<OA + 12288>(fa_base[SA >> 1][KS ^ 2]);
    }
  };
  // weight fragment first: the lane then holds 4 consecutive output columns of one row.
  // the tag is the number of 32-row fragments of the wave that hold a valid row; the others issue no MFMA
  auto mma = [&](auto set_tag, auto full_tag) __attribute__((always_inline)) {
    constexpr int NFA = decltype(full_tag)::value;
    constexpr int set = decltype(set_tag)::value;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (i < NFA) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[set][j], fa[set][i], acc[i][j], 0, 0, 0);
      }
  };

  // One quarter of an MFMA group: the two MFMAs that share activation fragment i.  The loads of a
  // step are issued between such pairs, never in a burst: a wave whose load has to queue for the
  // texture path issues nothing else meanwhile, its MFMAs included.
  auto mma_pair = [&](auto set_tag, auto i_tag, auto full_tag) __attribute__((always_inline)) {
    constexpr int NFA = decltype(full_tag)::value;
    constexpr int set = decltype(set_tag)::value, i = decltype(i_tag)::value;
    if constexpr (i < NFA) {
      acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[set][0], fa[set][i], acc[i][0], 0, 0, 0);
      acc[i][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[set][1], fa[set][i], acc[i][1], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
  };

  const int grow0 = m0 + wm * 128;                                   // wave's first output row
  const int gcol0 = n0 + wn * (MODE == GATE_UP ? 32 : 64);           // wave's first output column
  // DGRAD_H: saved g / u rows of one part of the wave's 128 rows (a 64-row half; a 32-row quarter for
  // DGRAD_H_GATE, whose epilogue needs more registers for itself), 16 bytes per lane and pass
  constexpr int GU_PARTS = (MODE == DGRAD_H_GATE) ? 4 : 2;
  constexpr int GU_ROWS = 128 / GU_PARTS;
  constexpr int GU_PASSES = GU_ROWS / 8;
  u32x4 pg[GU_PASSES], pu[GU_PASSES];
  auto gu_load = [&](int hh, ArgPtr ap) __attribute__((always_inline)) {
    if constexpr (is_dgrad_h(MODE)) {
      const int ncol = ap->N;
      const uint16_t* gsrc = ap->G;
      const uint16_t* usrc = ap->U;
#pragma unroll
      for (int p = 0; p < GU_PASSES; ++p) {
        const int row = p * 8 + (lane >> 3), piece = lane & 7;
        int gr = grow0 + hh * GU_ROWS + row;  if (gr > m_end - 1) gr = m_end - 1;
        int gc = gcol0 + piece * 8;  if (gc > ncol - 8) gc = ncol - 8;
        const size_t o = static_cast<size_t>(gr) * ncol + gc;
        pg[p] = *reinterpret_cast<const u32x4*>(gsrc + o);
        pu[p] = *reinterpret_cast<const u32x4*>(usrc + o);
      }
    }
  };

  // Step kt (phase P = kt mod 5) reads A from slot 2P mod 5 and B from slot (2P+1) mod 5.  Its
  // barrier comes before its last MFMA group, after every wave has (a) seen its own loads of
  // A(kt+1) and B(kt+1) land (the four loads of A(kt+2), issued last, may still be in flight) and
  // (b) received its last fragments of step kt.  Behind it the tiles of step kt+1 are complete and
  // the two slots of step kt are free: B(kt+2) goes into A's slot at once, A(kt+3) into B's slot
  // between the MFMAs.
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  using I2 = std::integral_constant<int, 2>;
  using I3 = std::integral_constant<int, 3>;
  auto fence = [] { __builtin_amdgcn_sched_barrier(0); };
  auto step = [&](int kt, auto phase_tag, auto full_tag) __attribute__((always_inline)) {
    constexpr int P = decltype(phase_tag)::value;
    using SA = std::integral_constant<int, slot_of_a(P)>;
    using SB = std::integral_constant<int, slot_of_b(P)>;
    using NA = std::integral_constant<int, slot_of_a((P + 1) % NSLOT)>;
    using NB = std::integral_constant<int, slot_of_b((P + 1) % NSLOT)>;
    using LA = std::integral_constant<int, slot_of_a((P + 2) % NSLOT)>;   // where A(kt+2) goes: B(kt-1)'s slot
    const bool more = kt + 2 < nk;
    const bool more_a = more && a_live;
    if constexpr (GATHER_A) {
      // the tokens of A(kt+2) were fetched a step ago and are covered by that step's wait; those of
      // A(kt+3) are requested before the loads of A(kt+2), the only ones this step's wait leaves in flight
      if (more) apply_tok(tokn);
      if (kt + 3 < nk) fetch_tok(kt + 3, tokn);
    }
    read_frags(SA{}, SB{}, I1{}, I1{}, full_tag);
    lds_wait<nreads(decltype(full_tag)::value)>();  fence();
    mma_pair(I0{}, J0{}, full_tag);  mma_pair(I0{}, J1{}, full_tag);
    if (more_a) a_part(kt + 2, LA{}, J0{});
    fence();
    mma_pair(I0{}, J2{}, full_tag);  mma_pair(I0{}, J3{}, full_tag);
    if (more_a) a_part(kt + 2, LA{}, J1{});
    fence();
    read_frags(SA{}, SB{}, I2{}, I0{}, full_tag);
    lds_wait<nreads(decltype(full_tag)::value)>();  fence();
    mma_pair(I1{}, J0{}, full_tag);  mma_pair(I1{}, J1{}, full_tag);
    if (more_a) a_part(kt + 2, LA{}, J2{});
    fence();
    mma_pair(I1{}, J2{}, full_tag);  mma_pair(I1{}, J3{}, full_tag);
    if (more_a) { a_part(kt + 2, LA{}, J3{}); a_end(kt + 2); }
    fence();
    read_frags(SA{}, SB{}, I3{}, I1{}, full_tag);
    lds_wait<nreads(decltype(full_tag)::value)>();  fence();
    mma(I0{}, full_tag);  fence();
    if (kt + 1 < nk) {
      if (more_a) wait_vm<4>(); else wait_vm<0>();   // this wave's loads of A(kt+2), if it has any, may stay in flight
      lds_wait<0>();
      wg_barrier();
      read_frags(NA{}, NB{}, I0{}, I0{}, full_tag);
    } else {
      lds_wait<0>();
    }
    fence();
    // B(kt+2) goes into A(kt)'s slot, one load after each MFMA pair
    mma_pair(I1{}, J0{}, full_tag);
    if (more) { apply_tok(tokn); b_part(kt + 2, SA{}, J0{}); }
    fence();
    mma_pair(I1{}, J1{}, full_tag);
    if (more) b_part(kt + 2, SA{}, J1{});
    fence();
    mma_pair(I1{}, J2{}, full_tag);
    if (more) b_part(kt + 2, SA{}, J2{});
    fence();
    mma_pair(I1{}, J3{}, full_tag);
    if (more) { b_part(kt + 2, SA{}, J3{}); b_end(kt + 2); }
    if constexpr (GATHER_B) {
      // a whole step ahead of their use; the next step's wait for B(kt+2) covers them (they are older
      // than the loads of A(kt+3), the only ones that wait leaves in flight)
      if (kt + 3 < nk) fetch_tok(kt + 3, tokn);
    }
    fence();
  };
  auto main_loop = [&](auto full_tag) __attribute__((always_inline)) {
    if (nk > 0) {
      if constexpr (GATHER_B) {
        // the tokens of steps 0 and 1 are requested first and are older than the eight loads of A(0), A(1):
        // one wait for both
        fetch_tok(0, tokn);
        if (nk > 1) fetch_tok(1, tokn1);
        a_unit(0, std::integral_constant<int, slot_of_a(0)>{});
        if (nk > 1) {
          a_unit(1, std::integral_constant<int, slot_of_a(1)>{});
          wait_vm<8>();
        } else {
          wait_vm<4>();
        }
        apply_tok(tokn);
        b_unit(0, std::integral_constant<int, slot_of_b(0)>{});
        if (nk > 1) {
          apply_tok(tokn1);
          b_unit(1, std::integral_constant<int, slot_of_b(1)>{});
        }
      } else if constexpr (GATHER_A) {
        fetch_tok(0, tokn);
        if (nk > 1) fetch_tok(1, tokn1);
        b_unit(0, std::integral_constant<int, slot_of_b(0)>{});
        if (nk > 1) {
          b_unit(1, std::integral_constant<int, slot_of_b(1)>{});
          wait_vm<8>();
        } else {
          wait_vm<4>();
        }
        apply_tok(tokn);
        a_unit(0, std::integral_constant<int, slot_of_a(0)>{});
        if (nk > 1) {
          apply_tok(tokn1);
          if (nk > 2) fetch_tok(2, tokn);   // applied at the start of step 0: older than the loads of A(1)
          a_unit(1, std::integral_constant<int, slot_of_a(1)>{});
        }
      } else {
        // the weight tile first: its addresses are ready, while those of the activation tile may still
        // wait for the tokens of the tile's rows (gathered rows)
        b_unit(0, std::integral_constant<int, slot_of_b(0)>{});
        if (a_live) a_unit(0, std::integral_constant<int, slot_of_a(0)>{});
        if (nk > 1) {
          b_unit(1, std::integral_constant<int, slot_of_b(1)>{});
          if (a_live) a_unit(1, std::integral_constant<int, slot_of_a(1)>{});
        }
      }
      if constexpr (GATHER_A || GATHER_B) {
        // only the last four loads (A(1) or B(1)) stay in flight: both tiles of step 0 are in, and so are
        // the tokens of A(2)
        if (nk > 1) wait_vm<4>(); else wait_vm<0>();
      } else {
        if (nk > 1 && a_live) wait_vm<8>(); else if (nk > 1) wait_vm<4>(); else wait_vm<0>();
      }
      wg_barrier();
      if constexpr (GATHER_B) {
        if (nk > 2) fetch_tok(2, tokn);
      }
      read_frags(std::integral_constant<int, slot_of_a(0)>{}, std::integral_constant<int, slot_of_b(0)>{}, I0{}, I0{}, full_tag);
    }
    for (int kt = 0; kt < nk; kt += NSLOT) {
      step(kt, I0{}, full_tag);
      if (kt + 1 < nk) step(kt + 1, I1{}, full_tag);
      if (kt + 2 < nk) step(kt + 2, I2{}, full_tag);
      if (kt + 3 < nk) step(kt + 3, I3{}, full_tag);
      if (kt + 4 < nk) step(kt + 4, std::integral_constant<int, 4>{}, full_tag);
    }
  };
  // one copy of the loop per number of live fragments: a wave whose 128 rows all lie past the
  // expert's end only keeps the loads and barriers going
  switch (nfa) {
    case 4: main_loop(std::integral_constant<int, 4>{}); break;
    case 3: main_loop(std::integral_constant<int, 3>{}); break;
    case 2: main_loop(std::integral_constant<int, 2>{}); break;
    case 1: main_loop(std::integral_constant<int, 1>{}); break;
    default: main_loop(std::integral_constant<int, 0>{}); break;
  }
  const ArgPtr ae = reload_args<ARG>();     // the epilogue reads its arguments afresh
  gu_load(0, ae);
  wg_barrier();                             // every wave is done with the operand tiles

  // ---------------- epilogue -----------------------------------------------------
  // acc[i][j][4q+c] is the wave's element (row, col) with row = i*32 + lrow and
  // col = j*32 + q*8 + lgrp*4 + c.  The wave stages bf16 rows of 128 bytes in its own
  // 16 KB of LDS (16-byte pieces swizzled by row & 7) and stores 16 bytes per lane.
  char* stage = lds + wave * WAVE_STAGE_BYTES;
  auto quad_addr = [&](int row, int piece) __attribute__((always_inline)) -> char* {
    return stage + row * 128 + ((piece ^ (row & 7)) << 4) + lgrp * 8;
  };
  auto put_quad = [&](int row, int piece, float v0, float v1, float v2, float v3) __attribute__((always_inline)) {
    u32x2 o;
    o.x = pack_bf16(v0, v1);
    o.y = pack_bf16(v2, v3);
    *reinterpret_cast<u32x2*>(quad_addr(row, piece)) = o;
  };
  // stores `rows` staged rows starting at staged row 0 to out (row stride ld); the first
  // `pieces` 16-byte pieces of each row go to columns col0 + piece*8 (pieces = 4 or 8)
  auto flush = [&](uint16_t* out, size_t ld, int first_row, int rows, int piece0, int pieces, int col0, int ncols) __attribute__((always_inline)) {
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
    // gate weight of the lane's four rows (1 unless the caller folds the weights into h)
    float wv[4] = {1.f, 1.f, 1.f, 1.f};
    if (ae->row_weight != nullptr) {
      const float* rw = ae->row_weight;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        int r = grow0 + i * 32 + lrow;  if (r > m_end - 1) r = m_end - 1;
        wv[i] = rw[r];
      }
    }
    // pass 1: g in pieces 0-3, u in pieces 4-7
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q)
          put_quad(i * 32 + lrow, j * 4 + q, acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
    __builtin_amdgcn_wave_barrier();
    flush(ae->O0, ae->N, grow0, 128, 0, 4, gcol0, ae->N);
    flush(ae->O1, ae->N, grow0, 128, 4, 4, gcol0, ae->N);
    __builtin_amdgcn_wave_barrier();
    // pass 2: h = silu(g) * u from the fp32 accumulators
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float h[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) h[c] = silu_f(acc[i][0][4 * q + c]) * acc[i][1][4 * q + c] * wv[i];
        put_quad(i * 32 + lrow, q, h[0], h[1], h[2], h[3]);
      }
    __builtin_amdgcn_wave_barrier();
    flush(ae->O2, ae->N, grow0, 128, 0, 4, gcol0, ae->N);
  } else if constexpr (is_dgrad_h(MODE)) {
    // in parts of GU_ROWS rows: g rows at stage[0, 8K), u rows at stage[8K, 16K).  The g/u rows of
    // the first part were requested at the end of the main loop, those of the next part are
    // requested before a part is processed, so their latency stays hidden.
    // DGRAD_H_GATE: the accumulators hold dh0 = dout[token] . Wd; the row's gate weight w turns them into
    // dh = w dh0, and sum over the wave's 64 columns of dh0 * silu(g) * u is the wave's share of the
    // gradient of w (a lane holds 32 of the columns of its row, lane ^ 32 the other 32).
    constexpr bool GATE = (MODE == DGRAD_H_GATE);
    char* ustage = stage + WAVE_STAGE_BYTES / 2;
    constexpr int NI = GU_ROWS / 32;    // 32-row accumulator blocks per part
#pragma unroll
    for (int hh = 0; hh < GU_PARTS; ++hh) {
      const int first = grow0 + hh * GU_ROWS;
      float wrow[2] = {1.f, 1.f}, dsum[2] = {0.f, 0.f};
      if constexpr (GATE) {
        const float* rw = ae->row_weight;
#pragma unroll
        for (int i2 = 0; i2 < NI; ++i2) {
          int r = first + i2 * 32 + lrow;  if (r > m_end - 1) r = m_end - 1;
          wrow[i2] = rw[r];
        }
      }
#pragma unroll
      for (int p = 0; p < GU_PASSES; ++p) {
        const int row = p * 8 + (lane >> 3), piece = lane & 7;
        const int so = row * 128 + ((piece ^ (row & 7)) << 4);
        *reinterpret_cast<u32x4*>(stage + so) = pg[p];
        *reinterpret_cast<u32x4*>(ustage + so) = pu[p];
      }
      if (hh + 1 < GU_PARTS) gu_load(hh + 1, ae);
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int i2 = 0; i2 < NI; ++i2)
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
              const float sg = sigmoid_f(g4[c]);
              if constexpr (GATE) {
                const float dh0 = acc[hh * NI + i2][j][4 * q + c];
                const float sl = g4[c] * sg;                 // silu(g)
                const float t0 = dh0 * u4[c];
                dsum[i2] = __builtin_fmaf(t0, sl, dsum[i2]);
                du[c] = (dh0 * wrow[i2]) * sl;
                dg[c] = (t0 * wrow[i2]) * (sg * __builtin_fmaf(g4[c], 1.0f - sg, 1.0f));
              } else {
                const float dh = acc[hh * NI + i2][j][4 * q + c];
                const float a = dh * sg;                     // shared by both derivatives
                du[c] = a * g4[c];
                dg[c] = (a * u4[c]) * __builtin_fmaf(g4[c], 1.0f - sg, 1.0f);
              }
            }
            u32x2 o;
            o.x = pack_bf16(dg[0], dg[1]);  o.y = pack_bf16(dg[2], dg[3]);
            *reinterpret_cast<u32x2*>(ga) = o;
            o.x = pack_bf16(du[0], du[1]);  o.y = pack_bf16(du[2], du[3]);
            *reinterpret_cast<u32x2*>(ua) = o;
          }
      if constexpr (GATE) {
        if (gcol0 < ae->N) {     // a strip past the last column holds repeated columns: no share
          const int strips = ae->N >> 6;
          float* part = ae->dgate_part + (gcol0 >> 6);
#pragma unroll
          for (int i2 = 0; i2 < NI; ++i2) {
            const float t = dsum[i2] + __shfl_xor(dsum[i2], 32, 64);
            const int r = first + i2 * 32 + lrow;
            if (lgrp == 0 && r < m_end) part[static_cast<size_t>(r) * strips] = t;
          }
        }
      }
      __builtin_amdgcn_wave_barrier();
      for (int p = 0; p < GU_PASSES; ++p) {
        const int row = p * 8 + (lane >> 3), piece = lane & 7;
        const int so = row * 128 + ((piece ^ (row & 7)) << 4);
        const u32x4 dgv = *reinterpret_cast<const u32x4*>(stage + so);
        const u32x4 duv = *reinterpret_cast<const u32x4*>(ustage + so);
        const int gr = first + row, gc = gcol0 + piece * 8;
        if (gr < m_end && gc < ae->N) {
          const size_t o = static_cast<size_t>(gr) * ae->N + gc;
          *reinterpret_cast<u32x4*>(ae->O0 + o) = dgv;
          *reinterpret_cast<u32x4*>(ae->O1 + o) = duv;
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
    uint16_t* out = second ? ae->O1 : ae->O0;
    if constexpr (is_wgrad(MODE)) out += static_cast<size_t>(e) * ae->M * ae->N;
    flush(out, ae->N, grow0, 128, 0, 8, gcol0, ae->N);
  }
  __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0): this wave's staging reads are done
  wg_barrier();      // the staging area becomes operand stages again
  }  // tile loop
  return tile - total;
}

// The launch is persistent: gridDim.x workgroups (one per compute unit) walk the tile list.
// Workgroups are dealt to the 8 XCDs round-robin, so workgroup b takes position
// (b % 8) * (gridDim.x / 8) + b / 8 of every round: each XCD then works on a run of
// consecutive tiles (same expert, neighbouring panels) that share its L2.
__device__ __forceinline__ int first_list_position() {
  const int per_xcd = gridDim.x >> 3;
  return (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
}

template <int MODE>
__global__ __launch_bounds__(GEMM_THREADS) void grouped_gemm_kernel(GemmArgs a) {
  gemm_tile_list<MODE, 0>(a, first_list_position());
}

// Two products that do not depend on each other in one launch: the tile list of the second follows
// that of the first, so the workgroups that run out of tiles of the first go on with the second
// instead of idling until the next launch (one tail and one start-up instead of two).
template <int MODE_A, int MODE_B>
__global__ __launch_bounds__(GEMM_THREADS) void grouped_gemm_pair_kernel(GemmArgs a, GemmArgs b) {
  const int next = gemm_tile_list<MODE_A, 0>(a, first_list_position());
  gemm_tile_list<MODE_B, 1>(b, next);
}

// Workgroups of the persistent launch: one per compute unit (the 160 KB of LDS allow no more),
// a multiple of 8 so that every XCD gets the same share, and no more than there can be tiles.
// Per-device facts, looked up once per device: HIP keeps function attributes and the number of compute
// units per device, and a process may drive several.  Races between host threads are benign (both write
// the same values).
constexpr int MAX_DEVICES = 64;
int current_device() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); dev = 0; }
  return dev >= 0 && dev < MAX_DEVICES ? dev : 0;
}
int persistent_grid(long long max_tiles) {
  static int cus_of[MAX_DEVICES] = {};
  const int dev = current_device();
  int cus = cus_of[dev];
  if (cus == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 8) {
      (void)hipGetLastError();
      n = 256;
    }
    cus = cus_of[dev] = n & ~7;
  }
  long long g = (max_tiles + 7) & ~7ll;
  if (g > cus) g = cus;
  if (g < 8) g = 8;
  return static_cast<int>(g);
}
// Raises the kernel's dynamic-LDS limit on the current device, once per device.
template <typename K>
int configure_lds(K kernel, bool (&done)[MAX_DEVICES]) {
  const int dev = current_device();
  if (done[dev]) return MOE_OK;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES) !=
      hipSuccess) {
    (void)hipGetLastError();
    return MOE_ERR_LAUNCH;
  }
  done[dev] = true;
  return MOE_OK;
}

template <int MODE>
int launch_gemm(const GemmArgs& a, long long max_tiles, hipStream_t s, const char* name) {
  const dim3 grid(persistent_grid(max_tiles));
  static bool configured[MAX_DEVICES] = {};
  if (configure_lds(&grouped_gemm_kernel<MODE>, configured) != MOE_OK) return MOE_ERR_LAUNCH;
  MOE_LAUNCH(name, grouped_gemm_kernel<MODE>, grid, dim3(GEMM_THREADS), LDS_BYTES, s, a);
  return moe_check_launch();
}

template <int MODE_A, int MODE_B>
int launch_gemm_pair(const GemmArgs& a, const GemmArgs& b, long long max_tiles, hipStream_t s, const char* name) {
  const dim3 grid(persistent_grid(max_tiles));
  static bool configured[MAX_DEVICES] = {};
  if (configure_lds(&grouped_gemm_pair_kernel<MODE_A, MODE_B>, configured) != MOE_OK) return MOE_ERR_LAUNCH;
  MOE_LAUNCH(name, (grouped_gemm_pair_kernel<MODE_A, MODE_B>), grid, dim3(GEMM_THREADS), LDS_BYTES, s, a, b);
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
  if (T <= 0 || k <= 0 || E <= 0 || d <= 0 || f <= 0) return 0;
  const unsigned long long rows = static_cast<unsigned long long>(T) * static_cast<unsigned long long>(k);
  if (rows > 0x7FFFFFFFull) return 0;   // no call takes that many routed rows
  const int R_cap = static_cast<int>(rows);
  // the largest of every workspace any call may ask for on a layer of this shape
  const size_t sizes[] = {moe_permute_workspace_bytes(T, k, E), moe_grouped_gemm_bwd_workspace_bytes(R_cap, f),
                          moe_grouped_gemm_bwd_folded_workspace_bytes(R_cap, f), moe_router_bwd_workspace_bytes(T, d, E)};
  size_t m = 0;
  for (size_t v : sizes) m = v > m ? v : m;
  return m;
}

namespace {
// xp grouped rows, or (row_token not null) the token rows themselves, gathered by the GEMM's loads
int gemm_fwd(const moe_bf16* xp, const int32_t* row_token, const float* row_weight, const int32_t* expert_offsets, const moe_bf16* Wg,
             const moe_bf16* Wu, const moe_bf16* Wd, int E, int R_cap, int d, int f, moe_bf16* g, moe_bf16* u,
             moe_bf16* h, moe_bf16* yp, void* stream) {
  if (!xp || !expert_offsets || !Wg || !Wu || !Wd || !g || !u || !h || !yp) return MOE_ERR_INVALID;
  if (bad_gemm_dims(E, R_cap, d, f)) return MOE_ERR_INVALID;
  const void* ptrs[] = {xp, expert_offsets, Wg, Wu, Wd, g, u, h, yp};
  for (const void* p : ptrs) if (!moe_aligned16(p)) return MOE_ERR_INVALID;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int m_tiles = R_cap / BM + E;

  GemmArgs a{};
  a.offsets = expert_offsets; a.E = E; a.m_tiles_cap = m_tiles; a.row_token = row_token; a.row_weight = row_weight;
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

// byte offsets of gathered rows are 32-bit lane offsets from the start of x
bool bad_gather(const moe_bf16* x, int T, const int32_t* row_token, int width) {
  return !x || !row_token || T <= 0 || !moe_aligned16(row_token) ||
         static_cast<unsigned long long>(T) * width * sizeof(moe_bf16) > 0xFFFFFFFFull;
}
}  // namespace

extern "C" int moe_grouped_gemm_fwd(const moe_bf16* xp, const int32_t* expert_offsets, const moe_bf16* Wg,
                                    const moe_bf16* Wu, const moe_bf16* Wd, int E, int R_cap, int d, int f,
                                    moe_bf16* g, moe_bf16* u, moe_bf16* h, moe_bf16* yp, void* stream) {
  return gemm_fwd(xp, nullptr, nullptr, expert_offsets, Wg, Wu, Wd, E, R_cap, d, f, g, u, h, yp, stream);
}

extern "C" int moe_grouped_gemm_fwd_gather(const moe_bf16* x, int T, const int32_t* row_token,
                                           const int32_t* expert_offsets, const moe_bf16* Wg, const moe_bf16* Wu,
                                           const moe_bf16* Wd, int E, int R_cap, int d, int f, moe_bf16* g,
                                           moe_bf16* u, moe_bf16* h, moe_bf16* yp, void* stream) {
  if (bad_gather(x, T, row_token, d)) return MOE_ERR_INVALID;
  return gemm_fwd(x, row_token, nullptr, expert_offsets, Wg, Wu, Wd, E, R_cap, d, f, g, u, h, yp, stream);
}

extern "C" int moe_grouped_gemm_fwd_folded(const moe_bf16* x, int T, const int32_t* row_token, const float* row_weight,
                                           const int32_t* expert_offsets, const moe_bf16* Wg, const moe_bf16* Wu,
                                           const moe_bf16* Wd, int E, int R_cap, int d, int f, moe_bf16* g,
                                           moe_bf16* u, moe_bf16* hw, moe_bf16* ypw, void* stream) {
  if (bad_gather(x, T, row_token, d) || !row_weight || !moe_aligned16(row_weight)) return MOE_ERR_INVALID;
  return gemm_fwd(x, row_token, row_weight, expert_offsets, Wg, Wu, Wd, E, R_cap, d, f, g, u, hw, ypw, stream);
}

namespace {
// xp grouped rows, or (row_token not null) the token rows themselves, gathered by the loads of the
// two weight-gradient products that read them
int gemm_bwd(const moe_bf16* dyp, const moe_bf16* xp, const int32_t* row_token, const moe_bf16* g, const moe_bf16* u,
             const moe_bf16* h, const int32_t* expert_offsets, const moe_bf16* Wg, const moe_bf16* Wu,
             const moe_bf16* Wd, int E, int R_cap, int d, int f, moe_bf16* dxp, moe_bf16* dWg, moe_bf16* dWu,
             moe_bf16* dWd, void* ws, size_t ws_bytes, void* stream) {
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

  // Two launches of two independent products each (the second list of a launch takes over the workgroups
  // that the first leaves idle at its end).
  // dh = dyp . Wd, then the SwiGLU derivative -> dg, du (first: its tiles are the long ones) ; dWd = dyp^T h
  GemmArgs wd{};
  wd.offsets = expert_offsets; wd.E = E;
  wd.A0 = U16(dyp); wd.B0 = U16(h); wd.O0 = dWd; wd.M = d; wd.N = f;
  wd.n_tiles = (f + BN - 1) / BN;
  wd.m_tiles_cap = (d + BM - 1) / BM;   // row tiles of one expert's dW
  GemmArgs a{};
  a.offsets = expert_offsets; a.E = E; a.m_tiles_cap = m_tiles;
  a.A0 = U16(dyp); a.B0 = U16(Wd); a.G = U16(g); a.U = U16(u); a.O0 = dg; a.O1 = du;
  a.K = d; a.N = f; a.n_tiles = (f + BN - 1) / BN;
  int rc = launch_gemm_pair<DGRAD_H, WGRAD>(a, wd, static_cast<long long>(wd.n_tiles) * wd.m_tiles_cap * E +
                                                       static_cast<long long>(a.n_tiles) * m_tiles,
                                            s, "gemm_dgrad_h+wgrad_down");
  if (rc != MOE_OK) return rc;
  // dWg = dg^T xp and dWu = du^T xp (one list: both read the same rows of xp) ; dxp = dg . Wg + du . Wu
  // (last, so that the dx reduction that follows finds dxp in the last-level cache)
  GemmArgs w{};
  w.offsets = expert_offsets; w.E = E; w.row_token = row_token;
  w.A0 = dg; w.A1 = du; w.B0 = U16(xp); w.O0 = dWg; w.O1 = dWu; w.M = f; w.N = d;
  w.n_tiles = (d + BN - 1) / BN;
  w.m_tiles_cap = (f + BM - 1) / BM;
  GemmArgs b{};
  b.offsets = expert_offsets; b.E = E; b.m_tiles_cap = m_tiles;
  b.A0 = dg; b.A1 = du; b.B0 = U16(Wg); b.B1 = U16(Wu); b.O0 = dxp;
  b.K = f; b.N = d; b.n_tiles = (d + BN - 1) / BN;
  const long long tiles = 2ll * w.n_tiles * w.m_tiles_cap * E + static_cast<long long>(b.n_tiles) * m_tiles;
  if (row_token != nullptr) return launch_gemm_pair<WGRAD_GATHER, DGRAD_X>(w, b, tiles, s, "gemm_wgrad_gate_up+dgrad_x");
  return launch_gemm_pair<WGRAD, DGRAD_X>(w, b, tiles, s, "gemm_wgrad_gate_up+dgrad_x");
}
}  // namespace

extern "C" int moe_grouped_gemm_bwd(const moe_bf16* dyp, const moe_bf16* xp, const moe_bf16* g, const moe_bf16* u,
                                    const moe_bf16* h, const int32_t* expert_offsets, const moe_bf16* Wg,
                                    const moe_bf16* Wu, const moe_bf16* Wd, int E, int R_cap, int d, int f,
                                    moe_bf16* dxp, moe_bf16* dWg, moe_bf16* dWu, moe_bf16* dWd, void* ws,
                                    size_t ws_bytes, void* stream) {
  return gemm_bwd(dyp, xp, nullptr, g, u, h, expert_offsets, Wg, Wu, Wd, E, R_cap, d, f, dxp, dWg, dWu, dWd, ws,
                  ws_bytes, stream);
}

extern "C" int moe_grouped_gemm_bwd_gather(const moe_bf16* dyp, const moe_bf16* x, int T, const int32_t* row_token,
                                           const moe_bf16* g, const moe_bf16* u, const moe_bf16* h,
                                           const int32_t* expert_offsets, const moe_bf16* Wg, const moe_bf16* Wu,
                                           const moe_bf16* Wd, int E, int R_cap, int d, int f, moe_bf16* dxp,
                                           moe_bf16* dWg, moe_bf16* dWu, moe_bf16* dWd, void* ws, size_t ws_bytes,
                                           void* stream) {
  if (bad_gather(x, T, row_token, d)) return MOE_ERR_INVALID;
  return gemm_bwd(dyp, x, row_token, g, u, h, expert_offsets, Wg, Wu, Wd, E, R_cap, d, f, dxp, dWg, dWu, dWd, ws,
                  ws_bytes, stream);
}

// ---------------------------------------------------------------------------------------------
// Backward of a forward pass that folded the gate weights into h (moe_grouped_gemm_fwd_folded).
namespace {
// dgate[t, i] = sum over the column strips of the row's partial dot products (0 for a slot without a local row)
__global__ __launch_bounds__(256) void dgate_finish_kernel(const float* __restrict__ part, int strips,
                                                           const int32_t* __restrict__ slot_row, int n,
                                                           float* __restrict__ dgate) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= n) return;
  const int row = slot_row[idx];
  float sum = 0.f;
  if (row >= 0) {
    const float* p = part + static_cast<size_t>(row) * strips;
    for (int c = 0; c < strips; ++c) sum += p[c];
  }
  dgate[idx] = sum;
}

size_t folded_part_bytes(int R_cap, int f) {
  return (static_cast<size_t>(f / 64) * R_cap * sizeof(float) + 255) & ~static_cast<size_t>(255);
}
}  // namespace

extern "C" size_t moe_grouped_gemm_bwd_folded_workspace_bytes(int R_cap, int f) {
  if (R_cap <= 0 || f <= 0) return 0;
  return moe_grouped_gemm_bwd_workspace_bytes(R_cap, f) + folded_part_bytes(R_cap, f);
}

extern "C" int moe_grouped_gemm_bwd_folded(const moe_bf16* dout, const moe_bf16* x, int T, int k,
                                           const int32_t* row_token, const float* row_weight, const int32_t* slot_row,
                                           const moe_bf16* g, const moe_bf16* u, const moe_bf16* hw,
                                           const int32_t* expert_offsets, const moe_bf16* Wg, const moe_bf16* Wu,
                                           const moe_bf16* Wd, int E, int R_cap, int d, int f, moe_bf16* dxp,
                                           moe_bf16* dWg, moe_bf16* dWu, moe_bf16* dWd, float* dgate, void* ws,
                                           size_t ws_bytes, void* stream) {
  if (!dout || !g || !u || !hw || !expert_offsets || !Wg || !Wu || !Wd || !dxp || !dWg || !dWu || !dWd || !dgate ||
      !ws || !row_weight || !slot_row || k <= 0)
    return MOE_ERR_INVALID;
  if (bad_gemm_dims(E, R_cap, d, f) || bad_gather(x, T, row_token, d) || bad_gather(dout, T, row_token, d))
    return MOE_ERR_INVALID;
  const void* ptrs[] = {dout, x, g, u, hw, expert_offsets, Wg, Wu, Wd, dxp, dWg, dWu, dWd, dgate, ws, row_weight, slot_row};
  for (const void* p : ptrs) if (!moe_aligned16(p)) return MOE_ERR_INVALID;
  if (ws_bytes < moe_grouped_gemm_bwd_folded_workspace_bytes(R_cap, f)) return MOE_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int m_tiles = R_cap / BM + E;
  const size_t one = moe_grouped_gemm_bwd_workspace_bytes(R_cap, f) / 2;
  uint16_t* dg = static_cast<uint16_t*>(ws);
  uint16_t* du = reinterpret_cast<uint16_t*>(static_cast<char*>(ws) + one);
  float* part = reinterpret_cast<float*>(static_cast<char*>(ws) + 2 * one);

  // Two launches of two independent products each (the second list of a launch takes over the workgroups
  // that the first leaves idle at its end).
  // dh0 = dout[token] . Wd; dh = w dh0 -> dg, du; partial dot products of dh0 with h for the gate gradient
  // (first: its tiles are the long ones);
  // dWd = (w dout[token])^T h = dout[token]^T hw: rows of dout gathered by the loads of the A operand
  GemmArgs wd{};
  wd.offsets = expert_offsets; wd.E = E; wd.row_token = row_token;
  wd.A0 = U16(dout); wd.B0 = U16(hw); wd.O0 = dWd; wd.M = d; wd.N = f;
  wd.n_tiles = (f + BN - 1) / BN;
  wd.m_tiles_cap = (d + BM - 1) / BM;
  const long long wd_tiles = static_cast<long long>(wd.n_tiles) * wd.m_tiles_cap * E;
  GemmArgs a{};
  a.offsets = expert_offsets; a.E = E; a.m_tiles_cap = m_tiles; a.row_token = row_token; a.row_weight = row_weight;
  a.dgate_part = part;
  a.A0 = U16(dout); a.B0 = U16(Wd); a.G = U16(g); a.U = U16(u); a.O0 = dg; a.O1 = du;
  a.K = d; a.N = f; a.n_tiles = (f + BN - 1) / BN;
  int rc = launch_gemm_pair<DGRAD_H_GATE, WGRAD_GATHER_A>(a, wd, wd_tiles + static_cast<long long>(a.n_tiles) * m_tiles, s,
                                                          "gemm_dgrad_h+wgrad_down");
  if (rc != MOE_OK) return rc;
  const int n = T * k;
  MOE_LAUNCH("dgate_finish", dgate_finish_kernel, dim3((n + 255) / 256), dim3(256), 0, s, static_cast<const float*>(part),
             f / 64, slot_row, n, dgate);
  // dWg = dg^T x[token] and dWu = du^T x[token] (one list: both read the same gathered rows of x), then
  // dxp = dg . Wg + du . Wu
  GemmArgs w{};
  w.offsets = expert_offsets; w.E = E; w.row_token = row_token;
  w.A0 = dg; w.A1 = du; w.B0 = U16(x); w.O0 = dWg; w.O1 = dWu; w.M = f; w.N = d;
  w.n_tiles = (d + BN - 1) / BN;
  w.m_tiles_cap = (f + BM - 1) / BM;
  GemmArgs b{};
  b.offsets = expert_offsets; b.E = E; b.m_tiles_cap = m_tiles;
  b.A0 = dg; b.A1 = du; b.B0 = U16(Wg); b.B1 = U16(Wu); b.O0 = dxp;
  b.K = f; b.N = d; b.n_tiles = (d + BN - 1) / BN;
  return launch_gemm_pair<WGRAD_GATHER, DGRAD_X>(w, b, 2ll * w.n_tiles * w.m_tiles_cap * E + static_cast<long long>(b.n_tiles) * m_tiles,
                                                 s, "gemm_wgrad_gate_up+dgrad_x");
}
